"""GPU check of radar_draft_expand_noalloc (the entry point that allocates nothing: its scratch is
a device array of the library) against radar_draft_expand with a caller-owned workspace: same
kernels, so every output must be bit-identical; two calls in a row, the second smaller than the
first (the array keeps the first call's contents), then shapes the array cannot hold."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2512_14069_amd import synth
from gpu_util import dev, host

pytestmark = pytest.mark.gpu

FIELDS = ("cand_tokens", "cand_scores", "frontier_pool_idx", "frontier_tokens", "frontier_scores", "frontier_conf")


def both(b, oracle, logits, ps, pidx, k, pre):
    F, V = logits.shape
    cap = pre + F * k
    pa, pb = b.DraftPool(cap), b.DraftPool(cap)
    pa.count = pb.count = pre
    ref = b.radar_draft_expand(dev(logits), dev(ps), dev(pidx), k, pa)
    got = b.radar_draft_expand_noalloc(dev(logits), dev(ps), dev(pidx), k, pb)
    torch.cuda.synchronize()
    for n in FIELDS:
        assert torch.equal(getattr(got, n), getattr(ref, n)), (n, F, V, k)
    for n in ("tokens", "scores", "parents"):
        assert torch.equal(getattr(pb, n)[pre:], getattr(pa, n)[pre:]), (n, F, V, k)
    # and, like the existing entry point, against the oracle
    cp = dict(tokens=np.zeros(cap, np.int32), scores=np.zeros(cap, np.float32), parents=np.zeros(cap, np.int32))
    r = oracle.draft_expand(logits, ps, pidx, k, cp, pre)
    assert np.array_equal(host(got.cand_tokens).reshape(F, k), r["cand_tokens"])
    assert np.max(np.abs(host(got.cand_scores).reshape(F, k).astype(np.float64) - r["cand_scores"])) <= 1e-5
    assert np.array_equal(host(got.frontier_pool_idx), r["frontier_pool_idx"])
    return got


def test_two_calls_in_a_row_second_smaller(oracle):
    from paper_2512_14069_amd import binding as b
    rng = np.random.default_rng(synth.seed_for(61, 0))
    # the 8B shape (10 rows x 128256), then a smaller call whose chunks and counters reuse the head of the array
    for (F, V, k, pre) in ((10, 128256, 10, 100), (3, 5001, 4, 0), (10, 128256, 10, 10), (1, 777, 16, 5)):
        logits = synth.expand_logits(rng, F, V, 3.0)
        ps = (-rng.random(F)).astype(np.float32)
        pidx = rng.integers(0, max(pre, 1), F).astype(np.int32)
        both(b, oracle, logits, ps, pidx, k, pre)


def test_chain_of_draft_calls_without_a_workspace(oracle):
    """A whole drafting chain (root call, then k rows per call) through the static array."""
    from paper_2512_14069_amd import binding as b
    rng = np.random.default_rng(synth.seed_for(61, 1))
    k, V, steps = 10, 32000, 4
    cap = k + (steps - 1) * k * k
    gp = b.DraftPool(cap)
    cp = dict(tokens=np.zeros(cap, np.int32), scores=np.zeros(cap, np.float32), parents=np.zeros(cap, np.int32))
    ps, ppi = np.zeros(1, np.float32), np.full(1, -1, np.int32)
    for _ in range(steps):
        logits = synth.expand_logits(rng, len(ps), V, 3.0)
        pre = gp.count
        r = oracle.draft_expand(logits, ps, ppi, k, cp, pre)
        g = b.radar_draft_expand_noalloc(dev(logits), dev(ps), dev(ppi), k, gp)
        torch.cuda.synchronize()
        assert np.array_equal(host(g.cand_tokens).reshape(-1, k), r["cand_tokens"])
        assert np.array_equal(host(g.frontier_pool_idx), r["frontier_pool_idx"])
        assert np.array_equal(host(gp.tokens)[:gp.count], cp["tokens"][:gp.count])
        ps, ppi = r["frontier_scores"].copy(), r["frontier_pool_idx"].copy()


def test_shapes_beyond_the_array_are_refused():
    from paper_2512_14069_amd import binding as b
    lib = b.load()
    one = ctypes.c_void_p(256)                                      # never dereferenced: rejected first
    d = b.expand_desc(64, 1 << 20, 10, 0, 5000)                     # 64 rows x 1M logits: 2.3 MB of scratch
    assert b.radar_draft_expand_workspace_bytes(d) > b.RADAR_NOALLOC_SCRATCH_BYTES
    assert lib.radar_draft_expand_noalloc(*([one] * 12), ctypes.byref(d), None) == -2
    d = b.expand_desc(10, 128256, 10, 0, 50)                        # pool too small: the usual argument error
    assert lib.radar_draft_expand_noalloc(*([one] * 12), ctypes.byref(d), None) == -1
