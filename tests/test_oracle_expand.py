"""Pins for the CPU oracle's draft expansion and rerank (App. A.1 walkthrough;
Sec. 2.3 confidence-ordered reordering and pruning; Sec. 4.2, Eq. 3: the state
is k confidences in [0,1])."""
import numpy as np
import pytest
from scipy.special import log_softmax

from paper_2512_14069_amd import synth


def new_pool(cap):
    return dict(tokens=np.full(cap, -7, np.int32), scores=np.full(cap, np.nan, np.float32),
                parents=np.full(cap, -7, np.int32))


def sorted_topk(values, k):
    """Exhaustive: full stable sort of (-value, index)."""
    order = np.lexsort((np.arange(len(values)), -values.astype(np.float64)))
    return order[:k]


@pytest.mark.parametrize("F,V,k", [(1, 50, 3), (4, 4096, 4), (10, 3001, 10), (3, 17, 17)])
def test_topk_and_scores_against_full_sort(oracle, F, V, k):
    rng = np.random.default_rng(F * 1000 + V)
    logits = synth.normal_logits(rng, (F, V), 2.0)
    # force exact duplicates, also across the selection boundary
    logits[:, 5] = logits[:, 2]
    logits[0, :8] = logits[0].max()
    ps = (-rng.random(F) * 3).astype(np.float32)
    ppi = np.arange(F, dtype=np.int32) + 3
    pool = new_pool(3 + F * k + 2)
    r = oracle.draft_expand(logits, ps, ppi, k, pool, 3)
    lp = log_softmax(logits.astype(np.float64), axis=1)
    for f in range(F):
        idx = sorted_topk(logits[f], k)
        assert np.array_equal(r["cand_tokens"][f], idx)
        assert np.allclose(r["cand_scores"][f], ps[f] + lp[f, idx], rtol=0, atol=1e-6)
        # nothing left out beats the last one kept
        rest = np.setdiff1d(np.arange(V), idx)
        if len(rest):
            last = idx[-1]
            assert np.all((logits[f, rest] < logits[f, last]) |
                          ((logits[f, rest] == logits[f, last]) & (rest > last)))
    # frontier = exhaustive top-k over the F*k candidates by cumulative score
    flat = r["cand_scores"].reshape(-1)
    fidx = sorted_topk(flat, k)
    assert np.array_equal(r["frontier_pool_idx"], 3 + fidx)
    assert np.array_equal(r["frontier_tokens"], r["cand_tokens"].reshape(-1)[fidx])
    assert np.array_equal(r["frontier_scores"], flat[fidx])
    assert np.allclose(r["frontier_conf"], np.exp(flat[fidx].astype(np.float64)), rtol=1e-6)
    assert np.all(np.diff(r["frontier_scores"]) <= 0)
    # pool append, in candidate order, untouched elsewhere
    assert np.array_equal(pool["tokens"][3:3 + F * k], r["cand_tokens"].reshape(-1))
    assert np.array_equal(pool["scores"][3:3 + F * k], flat)
    assert np.array_equal(pool["parents"][3:3 + F * k], np.repeat(ppi, k))
    assert np.all(pool["tokens"][:3] == -7) and np.all(pool["tokens"][3 + F * k:] == -7)


def test_closed_form_rows(oracle):
    V, k = 1000, 5
    logits = np.stack([np.arange(V, dtype=np.float32), np.full(V, 1.5, np.float32)])
    pool = new_pool(2 * k)
    r = oracle.draft_expand(logits, np.zeros(2, np.float32), np.array([-1, -1], np.int32), k, pool, 0)
    assert np.array_equal(r["cand_tokens"][0], np.arange(V - 1, V - 1 - k, -1))
    assert np.array_equal(r["cand_tokens"][1], np.arange(k))
    # constant row: every token has probability 1/V
    assert np.allclose(r["cand_scores"][1], -np.log(V), atol=1e-6)
    # arange row: geometric series, log p(V-1-j) = -j - log(sum_{i<V} e^-i)
    lz = np.log(np.sum(np.exp(-np.arange(V, dtype=np.float64))))
    assert np.allclose(r["cand_scores"][0], -np.arange(k) - lz, atol=1e-6)


def test_normalised_rows_pass_through(oracle):
    """Rows that already are log-probabilities keep their values (logsumexp = 0)."""
    rng = np.random.default_rng(3)
    x = synth.expand_logits(rng, 3, 5000, 3.0, normalised=True)
    pool = new_pool(30)
    r = oracle.draft_expand(x, np.zeros(3, np.float32), np.full(3, -1, np.int32), 10, pool, 0)
    for f in range(3):
        assert np.allclose(r["cand_scores"][f], x[f, r["cand_tokens"][f]], atol=2e-6)


def test_confidences_are_probabilities_that_sum_to_one_over_a_row(oracle):
    rng = np.random.default_rng(4)
    V = 64
    x = synth.normal_logits(rng, (1, V), 2.0)
    pool = new_pool(V)
    r = oracle.draft_expand(x, np.zeros(1, np.float32), np.array([-1], np.int32), V, pool, 0)
    p = np.exp(r["cand_scores"][0].astype(np.float64))
    assert abs(p.sum() - 1) < 1e-6
    assert np.all((p >= 0) & (p <= 1))
    assert np.all((r["frontier_conf"] >= 0) & (r["frontier_conf"] <= 1))


def run_schedule(oracle, rng, V, k, steps, N, std=3.0, first_F=1):
    """The paper's schedule (App. A.1): the first draft call sees the root only,
    every later one the k frontier nodes of the previous step."""
    cap = first_F * k + (steps - 1) * k * k
    pool = new_pool(cap)
    count = 0
    ps = np.zeros(first_F, np.float32)
    ppi = np.full(first_F, -1, np.int32)
    rows_of = {}
    history = []
    for s in range(steps):
        F = len(ps)
        x = synth.expand_logits(rng, F, V, std, normalised=(s % 2 == 0))
        r = oracle.draft_expand(x, ps, ppi, k, pool, count)
        for f in range(F):
            rows_of[int(ppi[f])] = x[f]
        history.append((count, F, r))
        count += F * k
        ps, ppi = r["frontier_scores"].copy(), r["frontier_pool_idx"].copy()
    tree = oracle.draft_rerank(pool, count, N, root_token=42)
    return pool, count, tree, rows_of, history


def test_walkthrough_structure_k2(oracle):
    """App. A.1 with k = 2: the first call yields 2 tokens, the second 4 candidates of
    which the 2 most confident form the next frontier."""
    rng = np.random.default_rng(6)
    pool, count, tree, _, hist = run_schedule(oracle, rng, V=97, k=2, steps=3, N=5)
    import os
    golden = os.path.join(os.path.dirname(__file__), "golden", "appendix_a1_walkthrough.txt")
    rows = [tuple(int(t) for t in ln.split()) for ln in open(golden) if ln.strip() and not ln.startswith("#")]
    for call, rows_in, cands, frontier in rows:
        start, F, r = hist[call - 1]
        assert F == rows_in and r["cand_tokens"].size == cands and r["frontier_pool_idx"].size == frontier
    assert [h[1] * 2 for h in hist] == [2, 4, 4]
    assert count == 10
    for _, F, r in hist:
        assert r["frontier_pool_idx"].shape == (2,)
    # second frontier is chosen among the 4 candidates of the second call
    assert set(hist[1][2]["frontier_pool_idx"]) <= set(range(2, 6))
    assert np.all(pool["parents"][:2] == -1)
    assert set(pool["parents"][2:6]) == set(hist[0][2]["frontier_pool_idx"])


@pytest.mark.parametrize("k,steps,N", [(4, 4, 15), (10, 8, 60), (3, 5, 200)])
def test_rerank_against_full_sort_and_tree_invariants(oracle, k, steps, N):
    rng = np.random.default_rng(100 + k)
    pool, count, tree, rows_of, _ = run_schedule(oracle, rng, V=2048, k=k, steps=steps, N=N)
    n = tree["n_nodes"]
    assert n == 1 + min(N, count)
    order = np.lexsort((np.arange(count), -pool["scores"][:count].astype(np.float64)))[:n - 1]
    assert np.array_equal(tree["pool_idx"][1:n], order)
    assert np.array_equal(tree["tokens"][1:n], pool["tokens"][order])
    assert np.array_equal(tree["scores"][1:n], pool["scores"][order])
    assert tree["tokens"][0] == 42 and tree["parents"][0] == -1 and tree["scores"][0] == 0
    # ancestor-closed, parents first, scores never increase downwards, depth consistent
    node_of = {-1: 0}
    for i in range(1, n):
        node_of[int(tree["pool_idx"][i])] = i
    for i in range(1, n):
        pp = int(pool["parents"][tree["pool_idx"][i]])
        assert pp in node_of
        assert tree["parents"][i] == node_of[pp] < i
        assert tree["scores"][i] <= tree["scores"][tree["parents"][i]]
        assert tree["depth"][i] == tree["depth"][tree["parents"][i]] + 1
    assert tree["depth"][:n].max() <= steps
    # a node's score is the sum of local log-probabilities along its path, recomputed
    # independently from the draft rows
    for i in range(1, n):
        total, j = 0.0, i
        while j > 0:
            pp = int(pool["parents"][tree["pool_idx"][j]])
            row = rows_of[pp].astype(np.float64)
            total += log_softmax(row)[tree["tokens"][j]]
            j = int(tree["parents"][j])
        assert abs(total - tree["scores"][i]) < 1e-5
    # padding past n_nodes
    assert np.all(tree["tokens"][n:] == -1) and np.all(tree["parents"][n:] == -1)
    if N >= count:
        assert n == count + 1


def test_running_top_n_equals_final_top_n(oracle):
    """Pruning to the best N after every step never changes the final kept set."""
    rng = np.random.default_rng(12)
    pool, count, tree, _, hist = run_schedule(oracle, rng, V=512, k=4, steps=5, N=12)
    final = set(int(x) for x in tree["pool_idx"][1:tree["n_nodes"]])
    keep = []
    for start, F, r in hist:
        keep += list(range(start, start + F * 4))
        keep = sorted(keep, key=lambda c: (-float(pool["scores"][c]), c))[:12]
    assert set(keep) == final


def test_bad_arguments(oracle):
    pool = new_pool(4)
    x = np.zeros((1, 8), np.float32)
    with pytest.raises(oracle.OracleError):
        oracle.draft_expand(x, np.zeros(1, np.float32), np.array([-1], np.int32), 5, pool, 0)   # pool too small
    with pytest.raises(oracle.OracleError):
        oracle.draft_expand(x, np.zeros(1, np.float32), np.array([-1], np.int32), 9, new_pool(20), 0)  # k > V
    # orphan: a kept child whose parent is not kept
    p = dict(tokens=np.array([1, 2], np.int32), scores=np.array([-2.0, -1.0], np.float32),
             parents=np.array([-1, 0], np.int32))
    with pytest.raises(oracle.OracleError):
        oracle.draft_rerank(p, 2, 1, 0)


def test_rerank_rejects_a_pool_entry_that_is_its_own_parent():
    """Scores never grow from parent to child, so a kept candidate's parent is kept and ranked earlier; an
    entry that names itself (or nothing valid) as parent is a malformed pool, not a tree."""
    import oracle
    pool = dict(tokens=np.arange(4, dtype=np.int32), scores=np.array([0.0, -1.0, -2.0, -3.0], np.float32),
                parents=np.array([-1, 0, 2, 1], np.int32))          # entry 2 is its own parent
    with pytest.raises(oracle.OracleError):
        oracle.draft_rerank(pool, 4, 4, 7)
    pool["parents"][2] = 1
    t = oracle.draft_rerank(pool, 4, 4, 7)
    assert t["parents"].tolist() == [-1, 0, 1, 2, 2] and t["depth"].tolist() == [0, 1, 2, 3, 3]
