"""GPU tests of the calls around the three steps: pre-marshalled calls and per-kernel timing."""
import numpy as np
import pytest
import torch

from paper_2512_14069_amd import synth
from gpu_util import bf16_dev, dev, host

pytestmark = pytest.mark.gpu


def test_prepared_calls_replay_the_same_work(oracle):
    from paper_2512_14069_amd import binding as b
    a = synth.config(1).attn
    x = synth.attention_inputs(a, seed=5)
    q, kc, vc = bf16_dev(x["q"]), bf16_dev(x["k_cache"]), bf16_dev(x["v_cache"])
    par, ctx, nn = dev(x["parents"]), dev(x["ctx_lens"]), dev(x["n_nodes"])
    direct = b.radar_tree_attention(q, kc, vc, par, ctx, nn)
    call = b.radar_tree_attention(q, kc, vc, par, ctx, nn, prepared=True)
    assert isinstance(call, b.BoundCall)
    call.out.fill_(7.0)
    out = call()
    torch.cuda.synchronize()
    assert torch.equal(out, direct)
    q.mul_(0.5)                                  # same pointers, new contents: a replay sees them
    again = b.radar_tree_attention(q, kc, vc, par, ctx, nn)
    assert torch.equal(call(), again)


def test_profile_reports_each_kernel(oracle):
    from paper_2512_14069_amd import binding as b
    rng = np.random.default_rng(2)
    F, V, k = 3, 5000, 4
    logits = dev(synth.normal_logits(rng, (F, V), 2.0))
    ps = torch.zeros(F, device="cuda")
    ppi = torch.full((F,), -1, dtype=torch.int32, device="cuda")
    pool = b.DraftPool(4 * F * k)
    b.radar_profile_begin(16)
    for _ in range(3):
        b.radar_draft_expand(logits, ps, ppi, k, pool)
    b.radar_draft_rerank(pool, 5, 1)
    torch.cuda.synchronize()
    t = b.radar_profile_end()
    assert t["expand"]["calls"] == 3 and t["rerank"]["calls"] == 1
    assert "zero_fill" in t                      # the workspaces made on the way were cleared by a kernel
    for v in t.values():
        assert 0.0 < v["min_us"] <= v["mean_us"] <= v["max_us"] < 1e5
    # nothing is recorded outside begin/end, and an empty session is fine
    b.radar_draft_rerank(pool, 5, 1)
    b.radar_profile_begin(4)
    assert b.radar_profile_end() == {}
    with pytest.raises(b.RadarError):
        b.radar_profile_begin(0)


def test_one_workspace_serves_several_entry_points_between_inits(oracle):
    """A workspace may go from one entry point (or descriptor) to another once it has been passed
    through radar_workspace_init again: the results equal those obtained with fresh workspaces."""
    from paper_2512_14069_amd import binding as b
    rng = np.random.default_rng(11)
    ws = b.new_workspace(64 << 20)

    # sampled verify-accept, two sequences
    a = synth.AttnShape(B=2, Hq=1, Hkv=1, D=8, T=20, ctx_lens=(0, 0), n_nodes=(20, 9), depths=(4, 3), k=4)
    x = synth.accept_inputs(a, 9000, seed=synth.seed_for(1, 41), plant=0.7)
    args = (dev(x["target_logits"]), dev(x["draft_tokens"]), dev(x["parents"]), dev(x["n_nodes"]), dev(x["uniforms"]))
    fresh = [host(t) for t in b.radar_verify_accept(*args, mode=1)]
    got = [host(t) for t in b.radar_verify_accept(*args, mode=1, workspace=ws)]
    assert all(np.array_equal(u, v) for u, v in zip(fresh, got))

    # expansion on the same memory
    b.radar_workspace_init(ws)
    F, V, k = 5, 12345, 6
    logits = dev(synth.normal_logits(rng, (F, V), 2.0))
    ps = torch.zeros(F, device="cuda")
    ppi = torch.full((F,), -1, dtype=torch.int32, device="cuda")
    p1, p2 = b.DraftPool(F * k), b.DraftPool(F * k)
    e1 = b.radar_draft_expand(logits, ps, ppi, k, p1)
    e2 = b.radar_draft_expand(logits, ps, ppi, k, p2, workspace=ws)
    torch.cuda.synchronize()
    for name in ("cand_tokens", "cand_scores", "frontier_pool_idx", "frontier_tokens", "frontier_scores", "frontier_conf"):
        assert torch.equal(getattr(e1, name), getattr(e2, name)), name

    # attention with several key ranges, then accept again with another shape
    b.radar_workspace_init(ws)
    s = synth.AttnShape(B=2, Hq=8, Hkv=2, D=128, T=24, ctx_lens=(300, 90), n_nodes=(24, 11), depths=(4, 3), k=4)
    y = synth.attention_inputs(s, seed=synth.seed_for(1, 43))
    q, kc, vc = bf16_dev(y["q"]), bf16_dev(y["k_cache"]), bf16_dev(y["v_cache"])
    targs = (q, kc, vc, dev(y["parents"]), dev(y["ctx_lens"]), dev(y["n_nodes"]))
    o1 = b.radar_tree_attention(*targs, keys_per_split=64)
    o2 = b.radar_tree_attention(*targs, keys_per_split=64, workspace=ws)
    assert torch.equal(o1, o2)

    b.radar_workspace_init(ws)
    a2 = synth.AttnShape(B=3, Hq=1, Hkv=1, D=8, T=33, ctx_lens=(0,) * 3, n_nodes=(33, 2, 17), depths=(6, 1, 4), k=4)
    x2 = synth.accept_inputs(a2, 20000, seed=synth.seed_for(1, 47), plant=0.7)
    args2 = (dev(x2["target_logits"]), dev(x2["draft_tokens"]), dev(x2["parents"]), dev(x2["n_nodes"]), dev(x2["uniforms"]))
    fresh2 = [host(t) for t in b.radar_verify_accept(*args2, mode=1)]
    got2 = [host(t) for t in b.radar_verify_accept(*args2, mode=1, workspace=ws)]
    assert all(np.array_equal(u, v) for u, v in zip(fresh2, got2))


def test_verify_step_replays_from_a_graph(oracle):
    """Tree attention (the library's plan on a short cache, and long ranges of a longer one) and sampled
    verify-accept captured once in a HIP graph and replayed with new inputs, with the program's own eager
    work and synchronisations between the replays; every replay is compared with the eager calls on the
    same inputs bit for bit, and the first with the oracle."""
    from paper_2512_14069_amd import binding as b
    from gpu_util import bf16_bits
    from test_gpu_attention import check_close
    V = 5000
    short = synth.AttnShape(B=2, Hq=8, Hkv=2, D=128, T=40, ctx_lens=(333, 70), n_nodes=(40, 17), depths=(5, 3), k=4)
    long_ = synth.AttnShape(B=2, Hq=8, Hkv=2, D=128, T=40, ctx_lens=(1100, 530), n_nodes=(40, 17), depths=(5, 3), k=4)

    def device_inputs(seed):
        xs, xl = synth.attention_inputs(short, seed=seed), synth.attention_inputs(long_, seed=seed + 1, shuffle=True)
        xa = synth.accept_inputs(short, V, seed=seed + 2, plant=0.7)
        return xs, xl, xa

    xs, xl, xa = device_inputs(100)
    bufs = dict(
        qs=bf16_dev(xs["q"]), ks=bf16_dev(xs["k_cache"]), vs=bf16_dev(xs["v_cache"]), ps=dev(xs["parents"]),
        cs=dev(xs["ctx_lens"]), ns=dev(xs["n_nodes"]),
        ql=bf16_dev(xl["q"]), kl=bf16_dev(xl["k_cache"]), vl=bf16_dev(xl["v_cache"]), pl=dev(xl["parents"]),
        cl=dev(xl["ctx_lens"]), nl=dev(xl["n_nodes"]),
        lg=dev(xa["target_logits"]), tk=dev(xa["draft_tokens"]), pa=dev(xa["parents"]), na=dev(xa["n_nodes"]),
        un=dev(xa["uniforms"]))

    def load(xs, xl, xa):
        for name, arr, bits in (("qs", xs["q"], True), ("ks", xs["k_cache"], True), ("vs", xs["v_cache"], True),
                                ("ql", xl["q"], True), ("kl", xl["k_cache"], True), ("vl", xl["v_cache"], True)):
            bufs[name].copy_(bf16_dev(arr))
        for name, arr in (("ps", xs["parents"]), ("pl", xl["parents"]), ("lg", xa["target_logits"]), ("tk", xa["draft_tokens"]),
                          ("pa", xa["parents"]), ("un", xa["uniforms"])):
            bufs[name].copy_(dev(arr))

    class Step:
        """One verify step with its own outputs and workspaces; run() enqueues it on the current stream."""
        def __init__(self):
            ds = b.attn_desc(bufs["qs"], bufs["ks"])
            dl = b.attn_desc(bufs["ql"], bufs["kl"], keys_per_split=512)
            self.ws = (b.new_workspace(b.radar_tree_attention_workspace_bytes(ds)),
                       b.new_workspace(b.radar_tree_attention_workspace_bytes(dl)),
                       b.new_workspace(b.radar_verify_accept_workspace_bytes(b.accept_desc(2, 40, V, 39, 1, 1.0))))
            self.out = (torch.empty_like(bufs["qs"]), torch.empty_like(bufs["ql"]),
                        (torch.empty(2, dtype=torch.int32, device="cuda"), torch.empty((2, 40), dtype=torch.int32, device="cuda"),
                         torch.empty(2, dtype=torch.int32, device="cuda")))

        def run(self):
            b.radar_tree_attention(bufs["qs"], bufs["ks"], bufs["vs"], bufs["ps"], bufs["cs"], bufs["ns"], out=self.out[0],
                                   workspace=self.ws[0])
            b.radar_tree_attention(bufs["ql"], bufs["kl"], bufs["vl"], bufs["pl"], bufs["cl"], bufs["nl"], out=self.out[1],
                                   keys_per_split=512, workspace=self.ws[1])
            b.radar_verify_accept(bufs["lg"], bufs["tk"], bufs["pa"], bufs["na"], bufs["un"], mode=1, out=self.out[2],
                                  workspace=self.ws[2])

    captured, eager = Step(), Step()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                          # warm-up outside the capture (one-time launch set-up)
        captured.run()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        captured.run()
    for i in range(4):
        xs, xl, xa = device_inputs(200 + 10 * i)
        load(xs, xl, xa)
        g.replay()
        torch.cuda.synchronize()
        got = captured.out
        eager.run()                                        # eager work between the replays
        torch.cuda.synchronize()
        ref = eager.out
        assert torch.equal(got[0], ref[0]) and torch.equal(got[1], ref[1]), i
        assert all(torch.equal(u, v) for u, v in zip(got[2], ref[2])), i
        if i == 0:
            for x, a, o in ((xs, short, got[0]), (xl, long_, got[1])):
                want = oracle.tree_attention(x["q"], x["k_cache"], x["v_cache"], x["parents"], x["ctx_lens"], x["n_nodes"])
                for bb in range(a.B):
                    n = a.n_nodes[bb]
                    check_close(bf16_bits(o)[bb, :n], want[bb, :n], f"graph replay b={bb}")
