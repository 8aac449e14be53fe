"""GPU parity: radar_draft_expand / radar_draft_rerank (through the C ABI) against the
CPU oracle on the same seeded inputs.  Token ids, frontier choices, kept node sets,
parents and depths must be bit-exact; cumulative log-probabilities within 1e-5."""
import numpy as np
import pytest
import torch

from paper_2512_14069_amd import synth
from gpu_util import dev, host

pytestmark = pytest.mark.gpu

SCORE_TOL = 1e-5      # log-prob tolerance of the baseline description
GAP = 1e-4            # selections decided by less than this are not compared bit-exactly


def np_pool(cap):
    return dict(tokens=np.zeros(cap, np.int32), scores=np.zeros(cap, np.float32), parents=np.zeros(cap, np.int32))


def min_boundary_gap(scores_sorted, k):
    """Smallest gap between neighbours among the k+1 best scores."""
    top = scores_sorted[:k + 1].astype(np.float64)
    return np.min(-np.diff(top)) if len(top) > 1 else np.inf


def run_both_step(oracle, b, logits, ps, ppi, k, gpu_pool, cpu_pool, ws=None):
    count = gpu_pool.count
    r = oracle.draft_expand(logits, ps, ppi, k, cpu_pool, count)
    g = b.radar_draft_expand(dev(logits), dev(ps), dev(ppi), k, gpu_pool, workspace=ws)
    torch.cuda.synchronize()
    F = logits.shape[0]
    assert np.array_equal(host(g.cand_tokens).reshape(F, k), r["cand_tokens"])
    assert np.max(np.abs(host(g.cand_scores).reshape(F, k).astype(np.float64) - r["cand_scores"])) <= SCORE_TOL
    flat = np.sort(r["cand_scores"].reshape(-1))[::-1]
    if min_boundary_gap(flat, k) > GAP:
        assert np.array_equal(host(g.frontier_pool_idx), r["frontier_pool_idx"])
        assert np.array_equal(host(g.frontier_tokens), r["frontier_tokens"])
        assert np.max(np.abs(host(g.frontier_scores).astype(np.float64) - r["frontier_scores"])) <= SCORE_TOL
        assert np.allclose(host(g.frontier_conf), r["frontier_conf"], rtol=2e-5, atol=0)
    else:   # near-tie: the GPU's choice must still be a valid top-k of its own scores
        gs = host(g.cand_scores)
        assert np.min(gs[host(g.frontier_pool_idx) - count]) >= np.sort(gs)[::-1][k - 1]
    n = count + F * k
    assert np.array_equal(host(gpu_pool.tokens)[count:n], cpu_pool["tokens"][count:n])
    assert np.array_equal(host(gpu_pool.parents)[count:n], cpu_pool["parents"][count:n])
    assert np.max(np.abs(host(gpu_pool.scores)[count:n].astype(np.float64) - cpu_pool["scores"][count:n])) <= SCORE_TOL
    return r, g


@pytest.mark.parametrize("F,V,k", [
    (4, 4096, 4),          # config 1
    (1, 128256, 10),       # first draft call of the paper's schedule
    (10, 128256, 10),      # config 3 shape
    (3, 4097, 5),          # ragged tail, unaligned rows (scalar loads)
    (2, 10, 10),           # k == V
    (7, 12290, 16),        # largest k, tail of two elements
    (64, 8192, 2),         # most rows
    (2, 300000, 10),       # more than 64 chunks per row: chunk lists and partials are merged in several blocks
    (40, 128256, 10),      # too many workgroups for 4 or 8 logits per lane: 16 per lane
    (5, 20000, 1),         # k = 1
])
def test_expand_step_matches_oracle(oracle, F, V, k):
    from paper_2512_14069_amd import binding as b
    rng = np.random.default_rng(synth.seed_for(3, F * 7 + k))
    logits = synth.expand_logits(rng, F, V, 3.0, normalised=(V % 2 == 0))
    ps = (-rng.random(F) * 4).astype(np.float32)
    ppi = rng.integers(-1, 5, F).astype(np.int32)
    gp, cp = b.DraftPool(5 + F * k + 3), np_pool(5 + F * k + 3)
    gp.count = 5
    gp.tokens.fill_(-7)
    cp["tokens"][:] = -7
    run_both_step(oracle, b, logits, ps, ppi, k, gp, cp)
    assert np.all(host(gp.tokens)[:5] == -7) and np.all(host(gp.tokens)[5 + F * k:] == -7)


def test_expand_exact_ties_and_special_values(oracle):
    """Equal logits are ordered by token id everywhere: duplicates inside a chunk, across
    chunks, across the top-k boundary; -inf entries and -0.0 / +0.0."""
    from paper_2512_14069_amd import binding as b
    V, k, F = 20000, 8, 4
    rng = np.random.default_rng(5)
    logits = synth.normal_logits(rng, (F, V), 1.0)
    logits[0, :] = 0.25                                   # constant row
    logits[1, [3, 4100, 8200, 12300, 16400, 19999, 7, 8]] = 9.0     # same value in several chunks
    logits[2, ::3] = -np.inf
    logits[2, [5, 4099]] = [0.0, -0.0]
    logits[2, logits[2] > 0] *= -1                        # zero is the maximum: +0.0 and -0.0 tie
    logits[3, :] = np.arange(V, dtype=np.float32) / 8     # many equal neighbours after rounding? no: strictly increasing
    ps = np.zeros(F, np.float32)
    ppi = np.full(F, -1, np.int32)
    gp, cp = b.DraftPool(F * k), np_pool(F * k)
    r = oracle.draft_expand(logits, ps, ppi, k, cp, 0)
    g = b.radar_draft_expand(dev(logits), dev(ps), dev(ppi), k, gp)
    torch.cuda.synchronize()
    assert np.array_equal(host(g.cand_tokens).reshape(F, k), r["cand_tokens"])
    assert np.array_equal(r["cand_tokens"][0], np.arange(k))
    assert np.max(np.abs(host(g.cand_scores).reshape(F, k) - r["cand_scores"])) <= SCORE_TOL


@pytest.mark.parametrize("cfg,first_F", [(1, 1), (3, 1), (3, 10)])
def test_expand_chain_and_rerank_match_oracle(oracle, cfg, first_F):
    """The whole drafting phase of a cycle: the paper's schedule (first call on the root
    alone, then k rows per call) or the timed shape (k rows every call), each step checked
    on identical inputs, then rerank to the best N and every tree field compared."""
    from paper_2512_14069_amd import binding as b
    c = synth.config(cfg)
    rng = np.random.default_rng(synth.seed_for(cfg, first_F))
    k, V, steps, N = c.k, c.vocab, c.expand_steps, c.N
    cap = first_F * k + (steps - 1) * k * k
    gp, cp = b.DraftPool(cap), np_pool(cap)
    ws = b.new_workspace(b.radar_draft_expand_workspace_bytes(b.expand_desc(k, V, k, 0, cap)))
    ps = np.zeros(first_F, np.float32) if first_F == 1 else (-rng.random(first_F)).astype(np.float32)
    ppi = np.full(first_F, -1, np.int32)
    for s in range(steps):
        logits = synth.expand_logits(rng, len(ps), V, c.logit_std, normalised=True)
        r, g = run_both_step(oracle, b, logits, ps, ppi, k, gp, cp, ws=ws)   # one workspace reused by all steps
        ps, ppi = r["frontier_scores"].copy(), r["frontier_pool_idx"].copy()
    assert gp.count == cap
    tree = oracle.draft_rerank(cp, cap, N, root_token=1234)
    # feed the GPU rerank the oracle's pool so that both order identical scores
    gp.tokens.copy_(dev(cp["tokens"])); gp.scores.copy_(dev(cp["scores"])); gp.parents.copy_(dev(cp["parents"]))
    t = b.radar_draft_rerank(gp, N, 1234)
    torch.cuda.synchronize()
    assert int(host(t.n_nodes)[0]) == tree["n_nodes"]
    for name in ("tokens", "parents", "depth", "pool_idx"):
        assert np.array_equal(host(getattr(t, name)), tree[name]), name
    assert np.array_equal(host(t.scores), tree["scores"])
    bad = b.radar_debug_validate_tree(t.parents.view(1, -1), t.n_nodes)
    assert int(host(bad)[0]) == 0


@pytest.mark.parametrize("count,N", [(0, 5), (3, 10), (64, 63), (810, 60), (4096, 60), (257, 1)])
def test_rerank_sizes_and_ties(oracle, count, N):
    from paper_2512_14069_amd import binding as b
    rng = np.random.default_rng(count + N)
    gp = b.DraftPool(max(count, 1))
    cp = np_pool(max(count, 1))
    # a forest whose scores never grow downwards, with exact score ties
    for i in range(count):
        par = -1 if i < 4 or rng.random() < 0.1 else int(rng.integers(0, i))
        drop = float(rng.integers(0, 4)) * 0.25            # many exact ties (including 0 drop)
        cp["parents"][i] = par
        cp["scores"][i] = (cp["scores"][par] if par >= 0 else 0.0) - drop
        cp["tokens"][i] = int(rng.integers(0, 1000))
    gp.tokens.copy_(dev(cp["tokens"])); gp.scores.copy_(dev(cp["scores"])); gp.parents.copy_(dev(cp["parents"]))
    gp.count = count
    tree = oracle.draft_rerank(cp, count, N, root_token=7)
    t = b.radar_draft_rerank(gp, N, 7)
    torch.cuda.synchronize()
    assert int(host(t.n_nodes)[0]) == tree["n_nodes"]
    for name in ("tokens", "parents", "depth", "pool_idx", "scores"):
        assert np.array_equal(host(getattr(t, name)), tree[name]), name


def test_expand_is_deterministic_and_workspace_reusable(oracle):
    from paper_2512_14069_amd import binding as b
    rng = np.random.default_rng(1)
    logits = dev(synth.expand_logits(rng, 10, 128256, 3.0))
    ps, ppi = dev(np.zeros(10, np.float32)), dev(np.full(10, -1, np.int32))
    ws = b.new_workspace(b.radar_draft_expand_workspace_bytes(b.expand_desc(10, 128256, 10, 0, 100)))
    outs = []
    for _ in range(3):
        gp = b.DraftPool(100)
        g = b.radar_draft_expand(logits, ps, ppi, 10, gp, workspace=ws)
        torch.cuda.synchronize()
        outs.append((host(g.cand_tokens).copy(), host(g.cand_scores).copy(), host(g.frontier_pool_idx).copy()))
    for o in outs[1:]:
        assert all(np.array_equal(x, y) for x, y in zip(o, outs[0]))
    assert int(ws[:16384].view(torch.int32).abs().sum().item()) == 0    # counters left clean
