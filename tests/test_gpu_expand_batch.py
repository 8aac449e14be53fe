"""GPU parity: radar_draft_expand_batch (one draft call for B sequences in one launch, through the
C ABI) against the CPU oracle run sequence by sequence on the same seeded inputs: plain calls, and
whole cycles in which every sequence stops at its own draft call (Sec. 4.1-4.2).  Token ids,
frontier choices, pool contents, stop steps and trees must be equal; scores within 1e-5."""
import types

import numpy as np
import pytest
import torch

from paper_2512_14069_amd import synth
from gpu_util import dev, host
from test_gpu_cycle import K, N, T_MAX, CAP, POLICY_TOL, make_inputs, oracle_cycle

pytestmark = pytest.mark.gpu

SCORE_TOL = 1e-5
GAP = 1e-4


@pytest.mark.parametrize("B,F,V,k,pre", [
    (5, 10, 32000, 10, 37),        # several sequences, pools already holding candidates
    (16, 10, 128256, 10, 0),       # the 8B shape for a batch of 16: 16 logits per lane, several rounds of workgroups
    (3, 1, 128256, 10, 0),         # first draft call of the paper's schedule (the root alone)
    (7, 3, 4097, 5, 11),           # ragged tail, unaligned rows (scalar loads)
    (2, 64, 8192, 2, 0),           # most rows
    (1, 4, 4096, 4, 0),            # B = 1 through the batched entry point
    (40, 3, 40001, 16, 11),        # streaming path (>= 4 Mi logits): odd V (scalar loads), ragged last wavefront, largest k
    (64, 10, 8192, 2, 0),          # streaming path with eight lists per row
    (4, 10, 128256, 10, 700),      # streaming path at its smallest 8B-shaped batch, pools nearly full
])
def test_batched_call_matches_oracle_per_sequence(oracle, B, F, V, k, pre):
    from paper_2512_14069_amd import binding as b
    rng = np.random.default_rng(synth.seed_for(9, B * 1000 + F + k))
    cap = pre + F * k
    logits = np.stack([synth.expand_logits(rng, F, V, 2.5) for _ in range(B)])
    ps = (-rng.random((B, F))).astype(np.float32)
    ppi = (rng.integers(0, pre, (B, F)).astype(np.int32) if pre else np.full((B, F), -1, np.int32))
    gp = b.DraftPool(cap, B=B)
    gp.tokens.fill_(-5); gp.parents.fill_(-5)            # what the call must not touch stays recognisable
    gp.count = pre
    g, pol = b.radar_draft_expand_batch(dev(logits), dev(ps), dev(ppi), k, gp)
    torch.cuda.synchronize()
    assert pol is None and gp.count == cap
    assert np.all(host(gp.tokens)[:, :pre] == -5)
    for s in range(B):
        cp = dict(tokens=np.zeros(cap, np.int32), scores=np.zeros(cap, np.float32), parents=np.zeros(cap, np.int32))
        r = oracle.draft_expand(logits[s], ps[s], ppi[s], k, cp, pre)
        assert np.array_equal(host(g.cand_tokens)[s].reshape(F, k), r["cand_tokens"]), s
        assert np.max(np.abs(host(g.cand_scores)[s].reshape(F, k).astype(np.float64) - r["cand_scores"])) <= SCORE_TOL
        flat = np.sort(r["cand_scores"].reshape(-1))[::-1][:k + 1].astype(np.float64)
        if len(flat) < 2 or np.min(-np.diff(flat)) > GAP:
            assert np.array_equal(host(g.frontier_pool_idx)[s], r["frontier_pool_idx"]), s
            assert np.array_equal(host(g.frontier_tokens)[s], r["frontier_tokens"]), s
            assert np.max(np.abs(host(g.frontier_scores)[s].astype(np.float64) - r["frontier_scores"])) <= SCORE_TOL
            assert np.allclose(host(g.frontier_conf)[s], r["frontier_conf"], rtol=2e-5, atol=0)
        assert np.array_equal(host(gp.tokens)[s, pre:cap], cp["tokens"][pre:cap]), s
        assert np.array_equal(host(gp.parents)[s, pre:cap], cp["parents"][pre:cap]), s
        assert np.max(np.abs(host(gp.scores)[s, pre:cap].astype(np.float64) - cp["scores"][pre:cap])) <= SCORE_TOL


@pytest.mark.parametrize("V,stops", [
    (32000, (1, 3, 8, 5, 2, 8)),       # single-launch form throughout
    (128256, (4, 8, 1)),
    (128256, (2, 8, 5, 1, 7)),         # calls with k rows stream in two launches (the root-only first call does not)
])
def test_batched_cycles_stop_sequence_by_sequence(oracle, V, stops):
    """t_max batched draft calls with the prediction model and per-sequence cycle states: every sequence
    stops where its own oracle chain stops, the others go on; a stopped sequence's arrays stay as its
    last executed call left them.  Run twice on the same buffers without resetting the states."""
    from paper_2512_14069_amd import binding as b
    B = len(stops)
    rng = np.random.default_rng(synth.seed_for(43, V % 1000 + B))
    p = synth.policy_params(rng, K, 128, 128, 2.0)
    pp = b.policy_params({n: dev(v) for n, v in p.items()})
    pool = b.DraftPool(CAP, B=B)
    states = torch.full((B, 4), 77, dtype=torch.int32, device="cuda")          # never initialised
    pout = b.PolicyOut(B, 128, "cuda")
    eouts = [b.ExpandOut(1 if s == 0 else K, K, "cuda", B=B) for s in range(T_MAX)]
    ws = b.new_workspace(b.radar_draft_expand_batch_workspace_bytes(b.expand_desc(K, V, K, 0, CAP), B))
    ps0 = torch.zeros((B, 1), dtype=torch.float32, device="cuda")
    pi0 = torch.full((B, 1), -1, dtype=torch.int32, device="cuda")
    for rep in range(2):
        order = stops if rep == 0 else stops[::-1]
        xs = [make_inputs(rng, V, st) for st in order]
        refs = [oracle_cycle(oracle, x, p, V) for x in xs]
        assert [r["steps"] for r in refs] == list(order)
        logits = [dev(np.stack([x["logits"][s] for x in xs])) for s in range(T_MAX)]
        uni = dev(np.stack([x["uni"] for x in xs]))                              # [B, T_MAX]
        ps, pi, count_max = ps0, pi0, 0
        for s in range(T_MAX):
            decide = s + 1 < T_MAX
            b.radar_draft_expand_batch(
                logits[s], ps, pi, K, pool, states=states, pool_count_max=count_max, params=pp if decide else None,
                h=pout.h if decide and s > 0 else None, c=pout.c if decide and s > 0 else None,
                uniform=uni[:, s].contiguous() if decide else None, out=eouts[s], policy_out=pout if decide else None,
                workspace=ws)
            count_max += (1 if s == 0 else K) * K
            ps, pi = eouts[s].frontier_scores, eouts[s].frontier_pool_idx
        # the batch's trees in one launch, then the verify walk over the ragged batch
        roots = dev(np.arange(1000, 1000 + B, dtype=np.int32))
        tb = b.radar_draft_rerank_batch(pool, N, roots, states=states, pool_count_max=CAP)
        target = dev(np.concatenate([x["target"] for x in xs]))                  # [B, N+1, V]
        acc_uni = dev(np.concatenate([x["acc_uni"] for x in xs]))                # [B, N+2]
        alen, apath, bonus = b.radar_verify_accept(target, tb.tokens, tb.parents, tb.n_nodes, acc_uni,
                                                   mode=b.RADAR_ACCEPT_SAMPLE, D_max=N)
        torch.cuda.synchronize()
        st = host(states)
        for q, ref in enumerate(refs):
            assert st[q].tolist()[:3] == [1 if ref["steps"] < T_MAX else 0, ref["count"], ref["steps"]], (q, st[q])
            for s in range(ref["steps"]):
                e, r = eouts[s], ref["fronts"][s]
                assert np.array_equal(host(e.frontier_tokens)[q], r["frontier_tokens"]), (q, s)
                assert np.array_equal(host(e.frontier_pool_idx)[q], r["frontier_pool_idx"]), (q, s)
                assert np.max(np.abs(host(e.frontier_scores)[q] - r["frontier_scores"])) <= 1e-5
            n = ref["count"]
            assert np.array_equal(host(pool.tokens)[q, :n], ref["pool"]["tokens"][:n])
            assert np.array_equal(host(pool.parents)[q, :n], ref["pool"]["parents"][:n])
            assert np.max(np.abs(host(pool.scores)[q, :n] - ref["pool"]["scores"][:n])) <= 1e-5
            if ref["policy"]:
                last = ref["policy"][-1]
                for name in ("h", "c", "logits", "probs"):
                    assert np.max(np.abs(host(getattr(pout, name))[q] - last[name][0])) <= POLICY_TOL, (q, name)
                assert host(pout.action)[q] == last["action"][0]
            # the tree of sequence q: the device's rerank of its own pool against the oracle's, by the batched
            # call and by the single-sequence call on a view of the same arrays
            view = types.SimpleNamespace(tokens=pool.tokens[q], scores=pool.scores[q], parents=pool.parents[q], capacity=CAP)
            t = b.radar_draft_rerank_cycle(view, states[q], CAP, N, 1000 + q)
            torch.cuda.synchronize()
            gpool = dict(tokens=host(pool.tokens)[q].copy(), scores=host(pool.scores)[q].copy(), parents=host(pool.parents)[q].copy())
            tree = oracle.draft_rerank(gpool, n, N, 1000 + q)
            assert int(host(t.n_nodes)[0]) == int(host(tb.n_nodes)[q]) == tree["n_nodes"] == 1 + min(N, n)
            for name in ("tokens", "parents", "depth", "pool_idx", "scores"):
                assert np.array_equal(host(getattr(t, name)), tree[name]), (q, name)
                assert np.array_equal(host(getattr(tb, name))[q], tree[name]), (q, name)
            nn = np.array([tree["n_nodes"]], np.int32)
            x = xs[q]
            o_len, o_path, o_bonus = oracle.verify_accept(x["target"], tree["tokens"][None], tree["parents"][None], nn,
                                                          x["acc_uni"], mode=1, D_max=N)
            m = oracle.accept_margins(x["target"], tree["tokens"][None], tree["parents"][None], nn, x["acc_uni"])
            if (m > 2e-7).all():
                assert host(alen)[q] == o_len[0] and np.array_equal(host(apath)[q], o_path[0]) and host(bonus)[q] == o_bonus[0]


def test_streaming_path_with_cycle_states(oracle):
    """A batch large enough for the two-launch path, every sequence with its own cycle state: different
    pool counts, two sequences already stopped (left alone by both launches), no decision in the call."""
    from paper_2512_14069_amd import binding as b
    B, F, V, k = 6, 10, 128256, 10
    rng = np.random.default_rng(synth.seed_for(9, 77))
    counts = [10, 110, 50, 110, 20, 0]
    stopped = [0, 0, 1, 0, 1, 0]
    count_max, cap = 110, 110 + F * k
    logits = np.stack([synth.expand_logits(rng, F, V, 2.5) for _ in range(B)])
    ps = (-rng.random((B, F))).astype(np.float32)
    ppi = np.stack([rng.integers(0, max(c, 1), F).astype(np.int32) for c in counts])
    pool = b.DraftPool(cap, B=B)
    pool.tokens.fill_(-5)
    states = dev(np.array([[stopped[q], counts[q], 3, 1] for q in range(B)], np.int32))
    out = b.ExpandOut(F, k, "cuda", B=B)
    out.frontier_tokens.fill_(-7); out.cand_tokens.fill_(-7)
    b.radar_draft_expand_batch(dev(logits), dev(ps), dev(ppi), k, pool, states=states, pool_count_max=count_max, out=out)
    torch.cuda.synchronize()
    st = host(states)
    for q in range(B):
        if stopped[q]:
            assert st[q].tolist() == [1, counts[q], 3, 1]
            assert np.all(host(out.frontier_tokens)[q] == -7) and np.all(host(out.cand_tokens)[q] == -7)
            assert np.all(host(pool.tokens)[q] == -5)
            continue
        assert st[q].tolist() == [0, counts[q] + F * k, 4, 1], (q, st[q])
        cp = dict(tokens=np.zeros(cap, np.int32), scores=np.zeros(cap, np.float32), parents=np.zeros(cap, np.int32))
        r = oracle.draft_expand(logits[q], ps[q], ppi[q], k, cp, counts[q])
        lo, hi = counts[q], counts[q] + F * k
        assert np.array_equal(host(out.cand_tokens)[q].reshape(F, k), r["cand_tokens"]), q
        assert np.max(np.abs(host(out.cand_scores)[q].reshape(F, k).astype(np.float64) - r["cand_scores"])) <= SCORE_TOL
        assert np.array_equal(host(out.frontier_pool_idx)[q], r["frontier_pool_idx"]), q
        assert np.array_equal(host(out.frontier_tokens)[q], r["frontier_tokens"]), q
        assert np.array_equal(host(pool.tokens)[q, lo:hi], cp["tokens"][lo:hi]) and np.all(host(pool.tokens)[q, :lo] == -5)
        assert np.array_equal(host(pool.parents)[q, lo:hi], cp["parents"][lo:hi])
        assert np.max(np.abs(host(pool.scores)[q, lo:hi].astype(np.float64) - cp["scores"][lo:hi])) <= SCORE_TOL


@pytest.mark.parametrize("B,count,cap,N", [(5, 810, 900, 60), (3, 4096, 4096, 63), (4, 3, 10, 7), (2, 0, 4, 5), (70, 64, 64, 0)])
def test_batched_rerank_matches_oracle_per_sequence(oracle, B, count, cap, N):
    """radar_draft_rerank_batch without states: forests with exact score ties, every sequence its own."""
    from paper_2512_14069_amd import binding as b
    rng = np.random.default_rng(B * 7 + count + N)
    pool = b.DraftPool(cap, B=B)
    cps = []
    for q in range(B):
        cp = dict(tokens=np.zeros(cap, np.int32), scores=np.zeros(cap, np.float32), parents=np.zeros(cap, np.int32))
        for i in range(count):
            par = -1 if i < 4 or rng.random() < 0.1 else int(rng.integers(0, i))
            cp["parents"][i] = par
            cp["scores"][i] = (cp["scores"][par] if par >= 0 else 0.0) - float(rng.integers(0, 4)) * 0.25
            cp["tokens"][i] = int(rng.integers(0, 1000))
        cps.append(cp)
    for name in ("tokens", "scores", "parents"):
        getattr(pool, name).copy_(dev(np.stack([cp[name] for cp in cps])))
    pool.count = count
    roots = dev(np.arange(7, 7 + B, dtype=np.int32))
    t = b.radar_draft_rerank_batch(pool, N, roots)
    torch.cuda.synchronize()
    for q in range(B):
        tree = oracle.draft_rerank(cps[q], count, N, root_token=7 + q)
        assert int(host(t.n_nodes)[q]) == tree["n_nodes"]
        for name in ("tokens", "parents", "depth", "pool_idx", "scores"):
            assert np.array_equal(host(getattr(t, name))[q], tree[name]), (q, name)
    with pytest.raises(b.RadarError):                      # more candidates than the arrays hold
        pool.count = cap + 1
        b.radar_draft_rerank_batch(pool, N, roots)


def test_batched_call_argument_errors(oracle):
    from paper_2512_14069_amd import binding as b
    B, F, V, k = 3, 2, 4096, 4
    rng = np.random.default_rng(5)
    logits = dev(np.stack([synth.expand_logits(rng, F, V, 2.0) for _ in range(B)]))
    ps, ppi = dev(np.zeros((B, F), np.float32)), dev(np.full((B, F), -1, np.int32))
    desc = b.expand_desc(F, V, k, 0, F * k)
    assert b.radar_draft_expand_batch_workspace_bytes(desc, 1) == b.radar_draft_expand_workspace_bytes(desc)
    assert b.radar_draft_expand_batch_workspace_bytes(desc, 0) == 0
    assert b.radar_draft_expand_batch_workspace_bytes(desc, B) > 2 * b.radar_draft_expand_workspace_bytes(desc)
    with pytest.raises(b.RadarError):                      # a single sequence's workspace does not do for three
        b.radar_draft_expand_batch(logits, ps, ppi, k, b.DraftPool(F * k, B=B),
                                   workspace=b.new_workspace(b.radar_draft_expand_workspace_bytes(desc)))
    with pytest.raises(ValueError):                        # the pool must carry the batch dimension
        b.radar_draft_expand_batch(logits, ps, ppi, k, b.DraftPool(F * k))
    with pytest.raises(b.RadarError):                      # the pools would overflow
        b.radar_draft_expand_batch(logits, ps, ppi, k, b.DraftPool(F * k - 1, B=B))
