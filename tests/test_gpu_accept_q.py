"""GPU parity: radar_verify_accept_q (through the C ABI) against the CPU oracle (Sec. 3, Eq. 1-2).

Lengths, paths and bonus tokens are integers decided by floating point: the device takes fp32
exponentials and keeps the residual as fp32 (relative error about 1e-6 on either side of an
acceptance test, about 1e-7 of the residual's mass on its running sums), the oracle is fp64
throughout.  A sequence is compared when every acceptance test of the oracle's walk is at least
ACCEPT_MARGIN (relative to the threshold) and the bonus draw at least CDF_MARGIN (of the
residual's mass) away from flipping; a vocabulary of 128256 has that many CDF steps, so about
one draw in eight lands within 5e-7 of one.  Fixed seeds are asserted to leave most sequences
comparable.
"""
import numpy as np
import pytest
import torch

from paper_2512_14069_amd import synth
from gpu_util import dev, host, tie_free_uniforms

pytestmark = pytest.mark.gpu

ACCEPT_MARGIN = 1e-5
CDF_MARGIN = 5e-7


def tie_free(oracle, x, q_rows=True, **kw):
    """The inputs' tie guard: sequences with a decision too close to its threshold get fresh uniforms."""
    qr = x["q_rows"] if q_rows else None

    def clear(u):
        m = oracle.verify_accept_q(x["target_logits"], x["draft_logits"], x["draft_tokens"], x["parents"], x["n_nodes"],
                                   u, qr, want_margins=True, **kw)[3]
        return (m[:, 0] > ACCEPT_MARGIN) & (m[:, 1] > CDF_MARGIN)
    return dict(x, uniforms=tie_free_uniforms(clear, x["uniforms"], np.random.default_rng(int(x["uniforms"].size))))


def run_both(oracle, b, x, q_rows=True, **kw):
    qr = x["q_rows"] if q_rows else None
    x = tie_free(oracle, x, q_rows, **kw)
    ref = oracle.verify_accept_q(x["target_logits"], x["draft_logits"], x["draft_tokens"], x["parents"], x["n_nodes"],
                                 x["uniforms"], qr, want_margins=True, **kw)
    args = (dev(x["target_logits"]), dev(x["draft_logits"]), dev(x["draft_tokens"]), dev(x["parents"]),
            dev(x["n_nodes"]), dev(x["uniforms"]), None if qr is None else dev(qr))
    got = [host(t) for t in b.radar_verify_accept_q(*args, **kw)]
    # the same call with the walk kept to one workgroup per sequence (-1) and with the shared walk's
    # wait cut to one poll (1: its workgroups give up and the sequence is redone by one): same answers
    for limit in (-1, 1):
        alt = [host(t) for t in b.radar_verify_accept_q(*args, walk_spin_limit=limit, **kw)]
        for u, v in zip(got, alt):
            assert np.array_equal(u, v), ("walk_spin_limit", limit)
    torch.cuda.synchronize()
    return ref, got


def compare(ref, got):
    sure = (ref[3][:, 0] > ACCEPT_MARGIN) & (ref[3][:, 1] > CDF_MARGIN)
    assert sure.all()                                              # the guard above: every sequence is compared
    for name, r, g in zip(("accept_len", "accept_path", "bonus_token"), ref[:3], got):
        assert g.shape == r.shape, name
        bad = np.nonzero(sure & ~(g == r).reshape(len(sure), -1).all(axis=1))[0]
        assert len(bad) == 0, (name, bad[:5], g[bad[:5]], r[bad[:5]])
    # sequences too close to call still give a legal walk
    assert np.all(got[0] >= 0) and np.all(got[0] <= ref[1].shape[1] - 1)
    return sure


def ragged_trees(rng, B, T, k, V):
    out = []
    for i in range(B):
        n = T if i % 4 == 0 else int(rng.integers(1, T + 1))
        if n == 1:
            out.append(np.array([-1], np.int32))
            continue
        dmin = 1 if n - 1 <= k else 1 + -(-(n - 1 - k) // (k * k))          # levels hold k, k*k, k*k, ... nodes
        depth = int(rng.integers(dmin, max(dmin, min(n - 1, 6)) + 1))
        out.append(synth.make_tree(rng, n, depth, k, V)[0])
    return out


@pytest.mark.parametrize("V,T,shared", [(4096, 16, True), (5001, 20, False), (32000, 61, True), (128256, 24, True)])
def test_ragged_batch_matches_oracle(oracle, V, T, shared):
    from paper_2512_14069_amd import binding as b
    rng = np.random.default_rng(synth.seed_for(32, V % 1000 + T))
    B = 24 if V < 100000 else 10
    x = synth.sampled_draft_inputs(rng, ragged_trees(rng, B, T, 4, V), V, T, std=2.0, noise=1.0, shared_rows=shared)
    ref, got = run_both(oracle, b, x)
    compare(ref, got)
    assert len(set(ref[0].tolist())) >= 3                       # several accepted lengths occur
    if not shared:                                              # every node has its own row: the map may be left out
        ref2, got2 = run_both(oracle, b, x, q_rows=False)
        compare(ref2, got2)
        assert all(np.array_equal(p, q) for p, q in zip(ref[:3], ref2[:3]))


def test_many_rejections_at_one_node_and_the_depth_cut(oracle):
    """A poor draft (independent of the target) under a star: most children are rejected one after the
    other, each rejection one more pass of Eq. 2; then the same trees cut at depth 1 and 0."""
    from paper_2512_14069_amd import binding as b
    V, T, B = 12000, 40, 12
    rng = np.random.default_rng(synth.seed_for(32, 5))
    par = [synth.star_tree(T) if i % 2 == 0 else synth.make_tree(rng, T, 3, 10, V)[0] for i in range(B)]
    x = synth.sampled_draft_inputs(rng, par, V, T, std=1.5, noise=4.0, shared_rows=True)
    ref, got = run_both(oracle, b, x)
    compare(ref, got)
    for D in (1, 0):
        ref, got = run_both(oracle, b, x, D_max=D)
        compare(ref, got)
        assert got[1].shape == (B, D + 1)


def test_chain_with_temperatures_and_config3_shape(oracle):
    from paper_2512_14069_amd import binding as b
    V, T, B = 128256, 9, 6
    rng = np.random.default_rng(synth.seed_for(32, 6))
    x = synth.sampled_draft_inputs(rng, [synth.chain_tree(T)] * B, V, T, std=3.0, noise=1.5, shared_rows=False)
    ref, got = run_both(oracle, b, x, q_rows=False, temperature=0.7, draft_temperature=1.3)
    compare(ref, got)


def test_identical_distributions_and_point_mass(oracle):
    """q = p accepts the first child everywhere; a point-mass q reproduces radar_verify_accept's sampling walk."""
    from paper_2512_14069_amd import binding as b
    V, T, B = 3000, 14, 16
    rng = np.random.default_rng(synth.seed_for(32, 7))
    par = [synth.make_tree(rng, T, 3, 3, V)[0] for _ in range(B)]
    x = synth.sampled_draft_inputs(rng, par, V, T, std=2.0, shared_rows=True)
    x["draft_logits"] = x["target_logits"].copy()
    ref, got = run_both(oracle, b, x)
    compare(ref, got)
    assert got[0].min() >= 1                                   # the first child is always accepted
    y = dict(x)
    y["draft_logits"] = np.zeros_like(x["target_logits"])
    for i in range(B):
        y["draft_logits"][i, np.arange(T), x["draft_tokens"][i]] = 80.0
    for i in range(B):
        for c in range(1, T):
            y["target_logits"][i, x["parents"][i, c], x["draft_tokens"][i, c]] += 3.0
    y["uniforms"] = tie_free_uniforms(
        lambda u: (oracle.accept_margins(y["target_logits"], y["draft_tokens"], y["parents"], y["n_nodes"], u) > 1e-6).all(axis=1),
        x["uniforms"], rng)
    got_q = b.radar_verify_accept_q(dev(y["target_logits"]), dev(y["draft_logits"]), dev(y["draft_tokens"]), dev(y["parents"]),
                                    dev(y["n_nodes"]), dev(y["uniforms"]))
    got_p = b.radar_verify_accept(dev(y["target_logits"]), dev(y["draft_tokens"]), dev(y["parents"]), dev(y["n_nodes"]),
                                  dev(y["uniforms"]), mode=b.RADAR_ACCEPT_SAMPLE)
    torch.cuda.synchronize()
    ref_p = oracle.verify_accept(y["target_logits"], y["draft_tokens"], y["parents"], y["n_nodes"], y["uniforms"], mode=1)
    for p, q, r in zip(got_p, got_q, ref_p):
        assert np.array_equal(host(p), host(q)) and np.array_equal(host(p), r)


def test_workspace_reuse_prepared_call_and_errors(oracle):
    from paper_2512_14069_amd import binding as b
    V, T, B = 9000, 12, 5
    rng = np.random.default_rng(synth.seed_for(32, 8))
    xs = [synth.sampled_draft_inputs(rng, ragged_trees(rng, B, T, 3, V), V, T) for _ in range(3)]
    desc = b.accept_q_desc(B, T, T, V, T - 1)
    ws = b.new_workspace(b.radar_verify_accept_q_workspace_bytes(desc))
    for x in xs:                                                 # one workspace, different inputs, twice each
        x = tie_free(oracle, x)
        ref = oracle.verify_accept_q(x["target_logits"], x["draft_logits"], x["draft_tokens"], x["parents"], x["n_nodes"],
                                     x["uniforms"], x["q_rows"], want_margins=True)
        call = b.radar_verify_accept_q(dev(x["target_logits"]), dev(x["draft_logits"]), dev(x["draft_tokens"]),
                                       dev(x["parents"]), dev(x["n_nodes"]), dev(x["uniforms"]), dev(x["q_rows"]),
                                       workspace=ws, prepared=True)
        for _ in range(2):
            call()
            torch.cuda.synchronize()
            compare(ref, [host(t) for t in call.out])
    x = xs[0]
    with pytest.raises(b.RadarError):
        b.radar_verify_accept_q(dev(x["target_logits"]), dev(x["draft_logits"]), dev(x["draft_tokens"]), dev(x["parents"]),
                                dev(x["n_nodes"]), dev(x["uniforms"]), temperature=0.0)
    with pytest.raises(b.RadarError):
        b.radar_verify_accept_q(dev(x["target_logits"]), dev(x["draft_logits"][:, :5].copy()), dev(x["draft_tokens"]),
                                dev(x["parents"]), dev(x["n_nodes"]), dev(x["uniforms"]))      # no q_rows, Tq != T
