"""GPU: a whole drafting cycle whose stop decision stays on the device (radar_cycle_begin,
radar_draft_expand_cycle, radar_draft_rerank_cycle), eagerly and replayed from a captured graph,
against the oracle's pieces chained on the host (Sec. 4.1-4.2; App. A.1).

The oracle chain is test code: expansion, then the prediction model on the new confidences,
stop on action 0 or after t_max draft calls, rerank, verification.  Integer results (tokens,
parents, pool indices, stop step, tree, accepted path) must be equal; scores within 1e-5;
model outputs within the tolerance of the policy tests.  The rerank is compared on the pool the
device itself built (scores there may differ from the oracle's in the last bit, which may order
near-equal candidates differently).
"""
import numpy as np
import pytest
import torch

from paper_2512_14069_amd import synth
from gpu_util import dev, host

pytestmark = pytest.mark.gpu

K, N, T_MAX = 10, 60, 8
CAP = K + (T_MAX - 1) * K * K
POLICY_TOL = 5e-5


def make_inputs(rng, V, stop_after=None, std=2.0):
    """Logits of t_max draft calls (the root alone, then k rows), one uniform per decision (scripted:
    0 keeps drafting, 0.999999 stops after draft call `stop_after`), target logits for the verify walk."""
    logits = [synth.expand_logits(rng, 1 if s == 0 else K, V, std) for s in range(T_MAX)]
    if stop_after is None:
        uni = rng.random(T_MAX).astype(np.float32)
    else:
        uni = np.zeros(T_MAX, np.float32)
        if 1 <= stop_after < T_MAX:
            uni[stop_after - 1] = 0.999999
    target = synth.normal_logits(rng, (1, N + 1, V), 1.5)
    acc_uni = rng.random((1, N + 2), dtype=np.float32)
    return dict(logits=logits, uni=uni, target=target, acc_uni=acc_uni)


def oracle_cycle(oracle, x, p, V, sampled=True):
    pool = dict(tokens=np.zeros(CAP, np.int32), scores=np.zeros(CAP, np.float32), parents=np.zeros(CAP, np.int32))
    ps, pidx = np.zeros(1, np.float32), np.full(1, -1, np.int32)
    count, h, c, steps, pol, fronts = 0, None, None, 0, [], []
    for s in range(T_MAX):
        e = oracle.draft_expand(x["logits"][s], ps, pidx, K, pool, count)
        count += len(ps) * K
        steps += 1
        fronts.append(e)
        ps, pidx = e["frontier_scores"].copy(), e["frontier_pool_idx"].copy()
        if s + 1 < T_MAX:
            o = oracle.policy_step(e["frontier_conf"][None], p, h, c, x["uni"][s:s + 1] if sampled else None)
            pol.append(o)
            h, c = o["h"].astype(np.float32), o["c"].astype(np.float32)
            if o["action"][0] == 0:
                break
    return dict(pool=pool, count=count, steps=steps, policy=pol, fronts=fronts)


class DeviceCycle:
    """All buffers of one cycle, allocated once; enqueue() issues the whole cycle on the current stream."""

    def __init__(self, b, V, p, sampled=True):
        self.b, self.V, self.sampled = b, V, sampled
        self.pp = b.policy_params({n: dev(v) for n, v in p.items()})
        self.logits = [torch.zeros((1 if s == 0 else K, V), dtype=torch.float32, device="cuda") for s in range(T_MAX)]
        self.uni = torch.zeros(T_MAX, dtype=torch.float32, device="cuda")
        self.target = torch.zeros((1, N + 1, V), dtype=torch.float32, device="cuda")
        self.acc_uni = torch.zeros((1, N + 2), dtype=torch.float32, device="cuda")
        self.pool = b.DraftPool(CAP)
        self.state = b.new_cycle_state()
        self.ps0 = torch.zeros(1, dtype=torch.float32, device="cuda")
        self.pi0 = torch.full((1,), -1, dtype=torch.int32, device="cuda")
        self.eouts = [b.ExpandOut(1 if s == 0 else K, K, "cuda") for s in range(T_MAX)]
        self.pout = b.PolicyOut(1, 128, "cuda")
        self.tree = b.TreeOut(N, "cuda")
        self.ws = b.new_workspace(b.radar_draft_expand_workspace_bytes(b.expand_desc(K, V, K, 0, CAP)))
        adesc = b.accept_desc(1, N + 1, V, N, b.RADAR_ACCEPT_SAMPLE, 1.0)
        self.acc_ws = b.new_workspace(b.radar_verify_accept_workspace_bytes(adesc))
        self.acc_out = (torch.zeros(1, dtype=torch.int32, device="cuda"), torch.zeros((1, N + 1), dtype=torch.int32, device="cuda"),
                        torch.zeros(1, dtype=torch.int32, device="cuda"))

    def load(self, x):
        for s in range(T_MAX):
            self.logits[s].copy_(torch.from_numpy(x["logits"][s]))
        self.uni.copy_(torch.from_numpy(x["uni"]))
        self.target.copy_(torch.from_numpy(x["target"]))
        self.acc_uni.copy_(torch.from_numpy(x["acc_uni"]))

    def enqueue(self, begin=True):
        b = self.b
        if begin:                                        # optional: the first draft call starts the cycle itself
            b.radar_cycle_begin(self.state)
        ps, pi, count_max = self.ps0, self.pi0, 0
        for s in range(T_MAX):
            decide = s + 1 < T_MAX
            b.radar_draft_expand_cycle(
                self.logits[s], ps, pi, K, self.pool, count_max, self.state,
                params=self.pp if decide else None,
                h=self.pout.h if decide and s > 0 else None, c=self.pout.c if decide and s > 0 else None,
                uniform=self.uni[s:s + 1] if decide and self.sampled else None,
                out=self.eouts[s], policy_out=self.pout if decide else None, workspace=self.ws)
            count_max += (1 if s == 0 else K) * K
            ps, pi = self.eouts[s].frontier_scores, self.eouts[s].frontier_pool_idx
        b.radar_draft_rerank_cycle(self.pool, self.state, CAP, N, 1234, out=self.tree)
        b.radar_verify_accept(self.target, self.tree.tokens.view(1, -1), self.tree.parents.view(1, -1), self.tree.n_nodes,
                              self.acc_uni, mode=b.RADAR_ACCEPT_SAMPLE, D_max=N, out=self.acc_out, workspace=self.acc_ws)


def check(oracle, cyc, x, ref):
    torch.cuda.synchronize()
    st = host(cyc.state)
    assert st[2] == ref["steps"], (st, ref["steps"])
    assert st[1] == ref["count"]
    assert st[0] == (1 if ref["steps"] < T_MAX else 0)
    for s in range(ref["steps"]):
        e, r = cyc.eouts[s], ref["fronts"][s]
        assert np.array_equal(host(e.frontier_tokens), r["frontier_tokens"]), s
        assert np.array_equal(host(e.frontier_pool_idx), r["frontier_pool_idx"]), s
        assert np.max(np.abs(host(e.frontier_scores) - r["frontier_scores"])) <= 1e-5
    n = ref["count"]
    assert np.array_equal(host(cyc.pool.tokens)[:n], ref["pool"]["tokens"][:n])
    assert np.array_equal(host(cyc.pool.parents)[:n], ref["pool"]["parents"][:n])
    assert np.max(np.abs(host(cyc.pool.scores)[:n] - ref["pool"]["scores"][:n])) <= 1e-5
    if ref["policy"]:
        last = ref["policy"][-1]
        for name in ("h", "c", "logits", "probs"):
            assert np.max(np.abs(host(getattr(cyc.pout, name)) - last[name])) <= POLICY_TOL, name
        assert host(cyc.pout.action)[0] == last["action"][0]
    # the tree: the oracle's rerank of the pool the device built
    gp = dict(tokens=host(cyc.pool.tokens).copy(), scores=host(cyc.pool.scores).copy(), parents=host(cyc.pool.parents).copy())
    tree = oracle.draft_rerank(gp, n, N, 1234)
    assert int(host(cyc.tree.n_nodes)[0]) == tree["n_nodes"] == 1 + min(N, n)
    for name in ("tokens", "parents", "depth", "pool_idx", "scores"):
        assert np.array_equal(host(getattr(cyc.tree, name)), tree[name]), name
    # and the verify walk over it
    nn = np.array([tree["n_nodes"]], np.int32)
    alen, apath, bonus = oracle.verify_accept(x["target"], tree["tokens"][None], tree["parents"][None], nn, x["acc_uni"],
                                              mode=1, D_max=N)
    m = oracle.accept_margins(x["target"], tree["tokens"][None], tree["parents"][None], nn, x["acc_uni"])
    if (m > 2e-7).all():
        assert np.array_equal(host(cyc.acc_out[0]), alen) and np.array_equal(host(cyc.acc_out[1]), apath)
        assert np.array_equal(host(cyc.acc_out[2]), bonus)


@pytest.mark.parametrize("V,stop_after", [(32000, 1), (32000, 4), (32000, 7), (32000, 8), (128256, 3)])
def test_cycle_stops_on_the_device_where_the_oracle_chain_stops(oracle, V, stop_after):
    from paper_2512_14069_amd import binding as b
    rng = np.random.default_rng(synth.seed_for(41, V % 1000 + stop_after))
    p = synth.policy_params(rng, K, 128, 128, 2.0)
    x = make_inputs(rng, V, stop_after)
    ref = oracle_cycle(oracle, x, p, V)
    assert ref["steps"] == stop_after
    cyc = DeviceCycle(b, V, p)
    for _ in range(2):                                   # twice on the same buffers: a skipped call leaves no trace
        cyc.load(x)
        cyc.enqueue()
        check(oracle, cyc, x, ref)


def test_cycles_back_to_back_without_cycle_begin(oracle):
    """The first draft call of a cycle (descriptor count 0) ignores what the state holds and rewrites
    all of it: cycles that stop early, late and not at all follow each other with no reset in between."""
    from paper_2512_14069_amd import binding as b
    V = 32000
    rng = np.random.default_rng(synth.seed_for(41, 55))
    p = synth.policy_params(rng, K, 128, 128, 2.0)
    cyc = DeviceCycle(b, V, p)
    cyc.state.fill_(123)                                 # never initialised
    for stop_after in (2, 8, 1, 5, 8, 3):
        x = make_inputs(rng, V, stop_after)
        ref = oracle_cycle(oracle, x, p, V)
        assert ref["steps"] == stop_after
        cyc.load(x)
        cyc.enqueue(begin=False)
        check(oracle, cyc, x, ref)


def test_argmax_decisions_and_random_uniforms(oracle):
    """The model's own argmax decisions (no uniform) and unscripted uniform draws, several parameter sets."""
    from paper_2512_14069_amd import binding as b
    V = 32000
    seen = set()
    for trial in range(6):
        rng = np.random.default_rng(synth.seed_for(41, 100 + trial))
        p = synth.policy_params(rng, K, 128, 128, 3.0)
        p["b2"] = np.array([0.0, 0.15 * (trial - 1)], np.float32)          # tilt towards stop / continue
        x = make_inputs(rng, V, None)
        for sampled in (False, True):
            ref = oracle_cycle(oracle, x, p, V, sampled)
            margins = [abs(o["logits"][0, 1] - o["logits"][0, 0]) if not sampled else abs(float(x["uni"][i]) - o["probs"][0, 1])
                       for i, o in enumerate(ref["policy"])]
            if margins and min(margins) < 1e-3:
                continue                                   # too close to call in fp32
            cyc = DeviceCycle(b, V, p, sampled)
            cyc.load(x)
            cyc.enqueue()
            check(oracle, cyc, x, ref)
            seen.add(ref["steps"])
    assert len(seen) >= 2, seen


def test_graph_replays_match_eager_and_oracle(oracle):
    """The cycle captured once in a HIP graph and replayed with new inputs, eager work and
    synchronisations between the replays; every replay is checked."""
    from paper_2512_14069_amd import binding as b
    V = 32000
    rng = np.random.default_rng(synth.seed_for(41, 7))
    p = synth.policy_params(rng, K, 128, 128, 2.0)
    cyc = DeviceCycle(b, V, p)
    other = DeviceCycle(b, V, p)                           # eager twin, its own buffers
    x0 = make_inputs(rng, V, 5)
    cyc.load(x0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                          # warm-up outside the capture
        cyc.enqueue()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        cyc.enqueue()
    for i, stop_after in enumerate((2, 8, 1, 6, 8, 3)):
        x = make_inputs(rng, V, stop_after)
        ref = oracle_cycle(oracle, x, p, V)
        assert ref["steps"] == stop_after
        cyc.load(x)
        g.replay()
        check(oracle, cyc, x, ref)
        other.load(x)
        other.enqueue()                                    # the program's own eager work between replays
        check(oracle, other, x, ref)
        for name in ("tokens", "parents", "scores", "depth", "pool_idx", "n_nodes"):
            assert torch.equal(getattr(cyc.tree, name), getattr(other.tree, name)), (i, name)
        assert all(torch.equal(u, v) for u, v in zip(cyc.acc_out, other.acc_out))


def test_argument_errors(oracle):
    from paper_2512_14069_amd import binding as b
    V = 4096
    rng = np.random.default_rng(3)
    p = synth.policy_params(rng, K, 128, 128)
    cyc = DeviceCycle(b, V, p)
    with pytest.raises(b.RadarError):                      # the pool could overflow at this step
        b.radar_draft_expand_cycle(cyc.logits[1], cyc.eouts[0].frontier_scores, cyc.eouts[0].frontier_pool_idx, K, cyc.pool,
                                   CAP - 5, cyc.state)
    pp4 = b.policy_params({n: dev(v) for n, v in synth.policy_params(rng, 4, 128, 128).items()})
    with pytest.raises(b.RadarError):                      # model built for another k
        b.radar_draft_expand_cycle(cyc.logits[0], cyc.ps0, cyc.pi0, K, cyc.pool, 0, cyc.state, params=pp4)
    # a state that claims more candidates than the host allows turns a later call into a no-op
    cyc.state.copy_(torch.tensor([0, 50, 1, -1], dtype=torch.int32))
    cyc.eouts[1].frontier_tokens.fill_(-7)
    b.radar_draft_expand_cycle(cyc.logits[1], cyc.eouts[0].frontier_scores, cyc.eouts[0].frontier_pool_idx, K, cyc.pool, K,
                               cyc.state, out=cyc.eouts[1])
    torch.cuda.synchronize()
    assert host(cyc.state).tolist() == [0, 50, 1, -1] and np.all(host(cyc.eouts[1].frontier_tokens) == -7)
    # while a call whose descriptor says 0 starts a cycle whatever the state holds
    cyc.state.copy_(torch.tensor([1, 50, 7, 0], dtype=torch.int32))
    b.radar_draft_expand_cycle(cyc.logits[0], cyc.ps0, cyc.pi0, K, cyc.pool, 0, cyc.state, out=cyc.eouts[0])
    torch.cuda.synchronize()
    assert host(cyc.state).tolist() == [0, K, 1, -1]
