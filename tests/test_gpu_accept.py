"""GPU parity: radar_verify_accept (through the C ABI) against the CPU oracle.
Accepted lengths, paths and bonus tokens must be bit-exact, for EVERY sequence.  In sampling
mode the inputs are made tie-free first: a sequence in which the oracle reports a decision
within MARGIN of its threshold gets fresh seeded uniforms (the margins themselves are pinned
in tests/test_oracle_margins.py).  Over a 128K vocabulary one token carries about 1e-5 of the
mass, so the inverse-CDF draw always lands within that distance of a boundary and the device
has to resolve far finer than that.  It sums exponentials in fp64 (fp32 only inside expf),
which leaves about 1e-8; MARGIN sits an order of magnitude above."""
import numpy as np
import pytest
import torch

from paper_2512_14069_amd import synth
from gpu_util import dev, host, tie_free_uniforms

pytestmark = pytest.mark.gpu

MARGIN = 2e-7


def run_gpu(b, x, mode, temperature=1.0, D_max=None, ws=None, use_n_nodes=True):
    out = b.radar_verify_accept(dev(x["target_logits"]), dev(x["draft_tokens"]), dev(x["parents"]),
                                dev(x["n_nodes"]) if use_n_nodes else None,
                                dev(x["uniforms"]) if mode == 1 else None,
                                mode=mode, temperature=temperature, D_max=D_max, workspace=ws)
    torch.cuda.synchronize()
    return [host(t) for t in out]


def compare(oracle, b, x, mode, temperature=1.0):
    if mode == 1:
        def clear(u):
            m = oracle.accept_margins(x["target_logits"], x["draft_tokens"], x["parents"], x["n_nodes"], u, temperature)
            return (m[:, 0] > MARGIN) & (m[:, 1] > MARGIN)
        x = dict(x, uniforms=tie_free_uniforms(clear, x["uniforms"], np.random.default_rng(int(x["uniforms"].size))))
    ref = oracle.verify_accept(x["target_logits"], x["draft_tokens"], x["parents"], x["n_nodes"],
                               x["uniforms"] if mode == 1 else None, mode=mode, temperature=temperature)
    got = run_gpu(b, x, mode, temperature)
    for name, g, r in zip(("accept_len", "accept_path", "bonus_token"), got, ref):
        assert np.array_equal(g, r), (name, np.nonzero((g != r).reshape(len(r), -1).any(axis=1))[0][:8])
    return ref, got


def small_shape(B, T, nn, dep, k=4):
    return synth.AttnShape(B=B, Hq=1, Hkv=1, D=8, T=T, ctx_lens=(0,) * B, n_nodes=nn, depths=dep, k=k)


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("V", [4096, 5000, 128256])
def test_single_sequence(oracle, mode, V):
    from paper_2512_14069_amd import binding as b
    a = small_shape(1, 16, (16,), (4,))
    x = synth.accept_inputs(a, V, seed=synth.seed_for(1, V % 97 + mode), plant=0.8)
    if mode == 1:   # correlate tokens with the target so that some are accepted
        x["target_logits"] = (x["target_logits"] * 0.5).astype(np.float32)
    ref, _ = compare(oracle, b, x, mode)
    if mode == 0:
        assert ref[0][0] >= 1          # planting gives a non-trivial path


@pytest.mark.parametrize("mode", [0, 1])
def test_config2_shape(oracle, mode):
    from paper_2512_14069_amd import binding as b
    c = synth.config(2)
    x = synth.accept_inputs(c.attn, c.vocab, seed=synth.seed_for(2, mode), plant=0.75)
    compare(oracle, b, x, mode)


def test_config4_ragged_full_size(oracle):
    """Configuration 4 at full size: 16 sequences with trees of 2..60 nodes, V = 128256, greedy."""
    from paper_2512_14069_amd import binding as b
    c = synth.config(4)
    x = synth.accept_inputs(c.attn, c.vocab, seed=synth.seed_for(4, 3), plant=0.75)
    ref, _ = compare(oracle, b, x, 0)
    assert ref[0].max() >= 2 and ref[0].min() <= 1       # accepted lengths are spread


@pytest.mark.parametrize("mode", [0, 1])
def test_config5_full_size(oracle, mode):
    """Configuration 5 at full size: four sequences of 60 rows, V = 128256, greedy and sampled."""
    from paper_2512_14069_amd import binding as b
    c = synth.config(5)
    x = synth.accept_inputs(c.attn, c.vocab, seed=synth.seed_for(5, mode), plant=0.75)
    compare(oracle, b, x, mode)


@pytest.mark.parametrize("mode,temperature", [(0, 1.0), (1, 1.0), (1, 0.6)])
def test_ragged_batch(oracle, mode, temperature):
    from paper_2512_14069_amd import binding as b
    B = 6
    rng = np.random.default_rng(17)
    dep = tuple(int(d) for d in rng.integers(1, 6, B))
    nn = tuple(int(rng.integers(d + 1, min(30, 1 + 4 + 16 * (d - 1)) + 1)) for d in dep)
    nn = (1,) + nn[1:]                    # a sequence that is only its root
    dep = (1,) + dep[1:]
    a = small_shape(B, 30, nn, dep)
    x = synth.accept_inputs(a, 20011, seed=99 + mode, plant=0.7, shuffle=True)
    compare(oracle, b, x, mode, temperature)


def test_sampling_many_uniform_vectors_small_tree(oracle):
    """Many sequences share one small tree and logits; only the uniforms differ, so every
    branch of the walk (accept first / later sibling, reject all, leaf) is exercised."""
    from paper_2512_14069_amd import binding as b
    B, T, V = 256, 9, 1000
    rng = np.random.default_rng(3)
    parents, tokens, depths = synth.make_tree(rng, T, 3, 3, V)
    logits = synth.normal_logits(rng, (T, V), 2.0)
    for c in range(1, T):                   # give the draft tokens real mass
        logits[parents[c], tokens[c]] = 8.0
    x = dict(target_logits=np.broadcast_to(logits, (B, T, V)).copy(),
             draft_tokens=np.broadcast_to(tokens, (B, T)).copy(),
             parents=np.broadcast_to(parents, (B, T)).copy(),
             n_nodes=np.full(B, T, np.int32), uniforms=rng.random((B, T + 1), dtype=np.float32))
    ref, got = compare(oracle, b, x, 1)
    assert len(set(ref[0].tolist())) >= 3       # several different accepted lengths occurred


def test_greedy_extremes_and_dmax(oracle):
    from paper_2512_14069_amd import binding as b
    V, n = 128256, 60
    rng = np.random.default_rng(8)
    parents = synth.chain_tree(n)
    tokens = rng.integers(0, V, n).astype(np.int32)
    logits = synth.gumbel_logits(rng, (n, V))
    for i in range(n - 1):
        logits[i, tokens[i + 1]] = 70.0
    x = dict(target_logits=logits[None], draft_tokens=tokens[None], parents=parents[None],
             n_nodes=np.array([n], np.int32), uniforms=None)
    ref, got = compare(oracle, b, x, 0)
    assert got[0][0] == n - 1                   # chain fully accepted: depth 59
    # walk capped by D_max
    got = run_gpu(b, x, 0, D_max=5)
    assert got[0][0] == 5 and list(got[1][0]) == [0, 1, 2, 3, 4, 5]
    # n_nodes = NULL means every slot is a node
    got = run_gpu(b, x, 0, use_n_nodes=False)
    assert got[0][0] == n - 1


def test_workspace_reuse_and_determinism(oracle):
    from paper_2512_14069_amd import binding as b
    c = synth.config(2)
    x = synth.accept_inputs(c.attn, c.vocab, seed=5)
    ws = b.new_workspace(b.radar_verify_accept_workspace_bytes(b.accept_desc(1, 60, c.vocab, 59, 1, 1.0)))
    first = run_gpu(b, x, 1, ws=ws)
    for mode in (0, 1, 1):
        again = run_gpu(b, x, mode, ws=ws)
        if mode == 1:
            assert all(np.array_equal(p, q) for p, q in zip(first, again))
    assert int(ws[:4096].view(torch.int32).abs().sum().item()) == 0


def test_wide_levels_and_duplicate_sibling_tokens(oracle):
    """Star-shaped trees (up to 63 children of the root, tried all at once on the device) whose
    sibling tokens repeat: the earliest sibling with a token wins, later copies are skipped, and
    the residual draw removes every tried token.  Uniforms differ per sequence."""
    from paper_2512_14069_amd import binding as b
    B, T, V = 192, 64, 3000
    rng = np.random.default_rng(11)
    parents = synth.star_tree(T)
    parents[40:] = rng.integers(1, 8, size=T - 40)          # a second, narrower level under nodes 1..7
    tokens = rng.integers(0, V, size=T).astype(np.int32)
    tokens[5] = tokens[2]; tokens[17] = tokens[2]; tokens[30] = tokens[9]     # repeated sibling tokens
    logits = synth.normal_logits(rng, (T, V), 1.5)
    for c in range(1, T):
        logits[parents[c], tokens[c]] = 3.0 + 0.02 * c       # every draft token carries visible mass
    x = dict(target_logits=np.broadcast_to(logits, (B, T, V)).copy(),
             draft_tokens=np.broadcast_to(tokens, (B, T)).copy(),
             parents=np.broadcast_to(parents, (B, T)).copy(),
             n_nodes=np.full(B, T, np.int32), uniforms=rng.random((B, T + 1), dtype=np.float32))
    ref, got = compare(oracle, b, x, 1)
    assert len(set(ref[0].tolist())) >= 2 and (ref[0] == 0).any() and (ref[0] > 0).any()
    compare(oracle, b, x, 0)


@pytest.mark.parametrize("mode", [0, 1])
def test_large_vocabulary_many_blocks(oracle, mode):
    """More than 128 blocks of 1024 logits per row: the merge and the residual scan loop."""
    from paper_2512_14069_amd import binding as b
    V = 300001
    a = small_shape(2, 12, (12, 7), (3, 2), k=3)
    x = synth.accept_inputs(a, V, seed=77)
    compare(oracle, b, x, mode)
