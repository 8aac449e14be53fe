"""Helpers shared by the GPU parity tests."""
import numpy as np
import torch


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.view(dtype) if t.element_size() == torch.empty((), dtype=dtype).element_size() and t.dtype != dtype else t.to(dtype)
    return t.cuda()


def bf16_dev(bits):
    """uint16 bf16 bit patterns -> torch.bfloat16 GPU tensor with the same bits."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).cuda()


def bf16_bits(t):
    """torch.bfloat16 tensor -> numpy uint16 bit patterns."""
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def host(t):
    return t.detach().cpu().numpy()


def tie_free_uniforms(margins_of, uniforms, rng, tries=200):
    """The inputs' tie guard for sampled verification: sequences in which some decision sits too
    close to its threshold for an fp32 device path get fresh uniforms (seeded), until none does.
    margins_of(uniforms) -> bool[B], True where the sequence is decided clear of every threshold
    (computed by the CPU oracle).  Returns the uniforms to use; every sequence can then be compared."""
    u = np.array(uniforms, np.float32, copy=True)
    for _ in range(tries):
        ok = margins_of(u)
        if ok.all():
            return u
        bad = np.nonzero(~ok)[0]
        u[bad] = rng.random((len(bad),) + u.shape[1:], dtype=np.float32)
    raise AssertionError("no tie-free uniforms found")
