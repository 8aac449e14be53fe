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
