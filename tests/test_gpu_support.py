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
