"""GPU parity: radar_policy_step (through the C ABI) against the CPU oracle (Sec. 4.2; App. A.3).

The device computes in fp32 (138-term dot products of O(1) values, library exp / tanh); the
oracle in fp64 on the same fp32 parameters.  Values agree within POLICY_TOL.  The action is an
integer decided by floating point: it must equal the oracle's wherever the oracle's margin
exceeds MARGIN, and it must always be the decision the device's own logits / probabilities
imply.
"""
import numpy as np
import pytest
import torch

from paper_2512_14069_amd import synth
from gpu_util import dev, host

pytestmark = pytest.mark.gpu

POLICY_TOL = 5e-5
MARGIN = 1e-3


def dev_params(b, p):
    return b.policy_params({n: dev(v) for n, v in p.items()})


def compare(ref, out, uniforms=None):
    torch.cuda.synchronize()
    for n in ("h", "c", "logits", "probs"):
        got = host(getattr(out, n))
        assert got.shape == ref[n].shape
        err = np.max(np.abs(got - ref[n]))
        assert err <= POLICY_TOL, (n, err)
    act, lg, pr = host(out.action), host(out.logits), host(out.probs)
    assert np.max(np.abs(pr.sum(axis=1) - 1.0)) <= 1e-6
    if uniforms is None:
        assert np.array_equal(act, (lg[:, 1] > lg[:, 0]).astype(np.int32))
        sure = np.abs(ref["logits"][:, 1] - ref["logits"][:, 0]) > MARGIN
    else:
        assert np.array_equal(act, (uniforms < pr[:, 1]).astype(np.int32))
        sure = np.abs(uniforms.astype(np.float64) - ref["probs"][:, 1]) > MARGIN
    assert np.array_equal(act[sure], ref["action"][sure])
    return int(sure.sum())


@pytest.mark.parametrize("B,k,M,gain", [(1, 10, 128, 1.0), (7, 10, 128, 2.0), (3, 16, 128, 1.0), (4, 1, 128, 1.0),
                                        (5, 10, 100, 2.0), (2, 7, 17, 1.0), (3, 10, 1, 1.0), (300, 10, 128, 2.0)])
def test_one_step_from_given_and_zero_state(oracle, B, k, M, gain):
    from paper_2512_14069_amd import binding as b
    rng = np.random.default_rng(synth.seed_for(22, 16 * B + k + M))
    p = synth.policy_params(rng, k, 128, M, gain)
    pp = dev_params(b, p)
    conf = synth.policy_conf(rng, B, k)[0]
    h0 = (rng.uniform(-1, 1, (B, 128))).astype(np.float32)
    c0 = (rng.standard_normal((B, 128)) * 1.5).astype(np.float32)
    n = compare(oracle.policy_step(conf, p), b.radar_policy_step(dev(conf), pp))
    n += compare(oracle.policy_step(conf, p, h0, c0), b.radar_policy_step(dev(conf), pp, dev(h0), dev(c0)))
    u = rng.random(B, dtype=np.float32)
    n += compare(oracle.policy_step(conf, p, h0, c0, u), b.radar_policy_step(dev(conf), pp, dev(h0), dev(c0), dev(u)), u)
    assert n >= 2 * B                              # most decisions are far from their threshold


def test_eight_draft_steps_state_kept_on_device(oracle):
    """The paper's setting: up to 8 draft calls per cycle, k = 10; the device hands its own
    state from step to step (in place), the oracle its own."""
    from paper_2512_14069_amd import binding as b
    B, k, steps = 4, 10, 8
    rng = np.random.default_rng(synth.seed_for(22, 1))
    p = synth.policy_params(rng, k, 128, 128, 2.0)
    pp = dev_params(b, p)
    conf = synth.policy_conf(rng, B, k, steps)
    out = b.PolicyOut(B, 128, "cuda")
    h = c = None
    for t in range(steps):
        ref = oracle.policy_step(conf[t], p, h, c)
        if t == 0:
            b.radar_policy_step(dev(conf[t]), pp, out=out)
        else:
            b.radar_policy_step(dev(conf[t]), pp, out.h, out.c, out=out)      # h_out, c_out alias the inputs
        compare(ref, out)
        h, c = ref["h"].astype(np.float32), ref["c"].astype(np.float32)


def test_saturated_gates_and_large_logits(oracle):
    """Pre-activations of +-40 (sigmoid and tanh at their limits, one logit far above the other)."""
    from paper_2512_14069_amd import binding as b
    rng = np.random.default_rng(synth.seed_for(22, 2))
    p = synth.policy_params(rng, 10, 128, 128, 1.0)
    p["b_ih"] = (rng.choice([-40.0, 40.0, 0.0], size=512)).astype(np.float32)
    p["b2"] = np.array([30.0, -30.0], np.float32)
    pp = dev_params(b, p)
    conf = synth.policy_conf(rng, 3, 10)[0]
    c0 = (rng.standard_normal((3, 128)) * 3).astype(np.float32)
    h0 = np.zeros((3, 128), np.float32)
    ref = oracle.policy_step(conf, p, h0, c0)
    out = b.radar_policy_step(dev(conf), pp, dev(h0), dev(c0))
    compare(ref, out)
    assert np.all(np.isfinite(host(out.probs))) and np.all(host(out.action) == 0)


def test_prepared_call_and_argument_errors(oracle):
    from paper_2512_14069_amd import binding as b
    rng = np.random.default_rng(synth.seed_for(22, 3))
    p = synth.policy_params(rng, 10, 128, 128, 1.0)
    pp = dev_params(b, p)
    conf = synth.policy_conf(rng, 2, 10)[0]
    ref = oracle.policy_step(conf, p)
    call = b.radar_policy_step(dev(conf), pp, prepared=True)
    for _ in range(3):
        call()
    compare(ref, call.out)
    with pytest.raises(ValueError):
        b.radar_policy_step(dev(conf[:, :9].copy()), pp)
    with pytest.raises(ValueError):
        b.radar_policy_step(dev(conf), pp, h=call.out.h)
    bad = synth.policy_params(rng, 10, 64, 128)                      # H = 64 is not built
    with pytest.raises(b.RadarError):
        b.radar_policy_step(dev(conf), dev_params(b, bad))
    bad = synth.policy_params(rng, 10, 128, 200)                     # M beyond the limit
    with pytest.raises(b.RadarError):
        b.radar_policy_step(dev(conf), dev_params(b, bad))


@pytest.mark.parametrize("F,V,k,with_state", [(1, 128256, 10, False), (10, 128256, 10, True), (10, 32000, 10, True),
                                              (3, 5000, 4, True), (64, 4099, 16, True), (2, 300000, 10, False)])
def test_expansion_with_policy_equals_the_two_calls(oracle, F, V, k, with_state):
    """One launch (expansion, then the model on the confidences still on chip) gives bit for bit what
    radar_draft_expand followed by radar_policy_step gives, and agrees with the oracle chain."""
    from paper_2512_14069_amd import binding as b
    rng = np.random.default_rng(synth.seed_for(23, F + V + k))
    p = synth.policy_params(rng, k, 128, 128, 2.0)
    pp = dev_params(b, p)
    logits = synth.expand_logits(rng, F, V, 2.0)
    ps = (-rng.random(F) * 3).astype(np.float32)
    pidx = np.arange(F, dtype=np.int32) - (1 if F == 1 else 0)
    h0 = rng.uniform(-1, 1, (1, 128)).astype(np.float32) if with_state else None
    c0 = rng.standard_normal((1, 128)).astype(np.float32) if with_state else None
    u = rng.random(1, dtype=np.float32)
    dl, dps, dpi = dev(logits), dev(ps), dev(pidx)
    dh, dc = (dev(h0), dev(c0)) if with_state else (None, None)
    for uni in (None, u):
        du = None if uni is None else dev(uni)
        pool_a, pool_b = b.DraftPool(F * k + 7), b.DraftPool(F * k + 7)
        pool_a.count = pool_b.count = 7
        ea = b.radar_draft_expand(dl, dps, dpi, k, pool_a)
        pa = b.radar_policy_step(ea.frontier_conf, pp, dh, dc, du)
        eb, pb = b.radar_draft_expand_policy(dl, dps, dpi, k, pool_b, pp, dh, dc, du)
        torch.cuda.synchronize()
        for n in ("cand_tokens", "cand_scores", "frontier_pool_idx", "frontier_tokens", "frontier_scores", "frontier_conf"):
            assert torch.equal(getattr(ea, n), getattr(eb, n)), n
        for n in ("tokens", "scores", "parents"):
            assert torch.equal(getattr(pool_a, n)[7:], getattr(pool_b, n)[7:]), n
        for n in ("h", "c", "logits", "probs", "action"):
            assert torch.equal(getattr(pa, n), getattr(pb, n)), n
        # oracle chain: its own expansion, its own confidences
        opool = dict(tokens=np.zeros(F * k + 7, np.int32), scores=np.zeros(F * k + 7, np.float32),
                     parents=np.zeros(F * k + 7, np.int32))
        oe = oracle.draft_expand(logits, ps, pidx, k, opool, 7)
        assert np.array_equal(host(eb.frontier_tokens), oe["frontier_tokens"])
        ref = oracle.policy_step(oe["frontier_conf"][None], p, h0, c0, uni)
        compare(ref, pb, uni)


def test_drafting_loop_with_fused_policy_on_one_workspace(oracle):
    """Eight draft steps as the paper runs them (k = 10, F = 1 then 10): the state stays on the
    device and is updated in place; one workspace and one pool serve every step."""
    from paper_2512_14069_amd import binding as b
    k, V, steps = 10, 32000, 8
    rng = np.random.default_rng(synth.seed_for(23, 1))
    p = synth.policy_params(rng, k, 128, 128, 2.0)
    pp = dev_params(b, p)
    pool = b.DraftPool(k + (steps - 1) * k * k)
    opool = dict(tokens=np.zeros(pool.capacity, np.int32), scores=np.zeros(pool.capacity, np.float32),
                 parents=np.zeros(pool.capacity, np.int32))
    ws = b.new_workspace(b.radar_draft_expand_workspace_bytes(b.expand_desc(k, V, k, 0, pool.capacity)))
    pout = b.PolicyOut(1, 128, "cuda")
    ps, pidx = np.zeros(1, np.float32), np.full(1, -1, np.int32)
    dps, dpi = dev(ps), dev(pidx)
    h = c = None
    ocount = 0
    for t in range(steps):
        F = 1 if t == 0 else k
        logits = synth.expand_logits(rng, F, V, 2.0)
        oe = oracle.draft_expand(logits, ps, pidx, k, opool, ocount)
        ocount += F * k
        ref = oracle.policy_step(oe["frontier_conf"][None], p, h, c)
        eo, po = b.radar_draft_expand_policy(dev(logits), dps, dpi, k, pool, pp, None if t == 0 else pout.h,
                                             None if t == 0 else pout.c, policy_out=pout, workspace=ws)
        torch.cuda.synchronize()
        assert np.array_equal(host(eo.frontier_tokens), oe["frontier_tokens"])
        assert np.array_equal(host(eo.frontier_pool_idx), oe["frontier_pool_idx"])
        compare(ref, po)
        ps, pidx = oe["frontier_scores"], oe["frontier_pool_idx"]
        dps, dpi = eo.frontier_scores, eo.frontier_pool_idx
        h, c = ref["h"].astype(np.float32), ref["c"].astype(np.float32)
    assert pool.count == ocount
