"""GPU parity on randomly drawn shapes (fixed seeds): every entry point against the CPU oracle at sizes
nobody picked by hand -- vocabularies that are not multiples of 4 or of a block, k equal to V, trees of one
node, group sizes that leave wavefronts idle, odd batch sizes.  Same bars as the hand-written cases.

RADAR_TEST_EXTRA_SEEDS=n in the environment adds n further seeds to every test of this file (a sweep of
n = 1000 takes about a minute on the GPU)."""
import os

import numpy as np
import pytest
import torch

from paper_2512_14069_amd import synth
from gpu_util import bf16_dev, bf16_bits, dev, host, tie_free_uniforms

pytestmark = pytest.mark.gpu

EXTRA = int(os.environ.get("RADAR_TEST_EXTRA_SEEDS", "0"))


def rand_tree(rng, n, k, V):
    if n == 1:
        return np.array([-1], np.int32), np.array([int(rng.integers(0, V))], np.int32)
    kk = max(1, min(k, V))
    dmin = 1 if n - 1 <= kk else 1 + -(-(n - 1 - kk) // (kk * kk))
    depth = int(rng.integers(dmin, max(dmin, min(n - 1, 8)) + 1))
    par, tok, _ = synth.make_tree(rng, n, depth, kk, V, shuffle=bool(rng.integers(0, 2)))
    return par, tok


@pytest.mark.parametrize("seed", range(12 + EXTRA))
def test_attention_random_shapes(oracle, seed):
    from paper_2512_14069_amd import binding as b
    rng = np.random.default_rng(synth.seed_for(51, seed))
    B = int(rng.integers(1, 4))
    Hkv = int(rng.integers(1, 4))
    G = int(rng.choice([1, 2, 3, 4, 5, 8]))
    D = int(rng.choice([64, 128]))
    T = int(rng.integers(1, 65))
    ctx = [int(rng.integers(0, 400)) for _ in range(B)]
    nn = [int(rng.integers(1, T + 1)) for _ in range(B)]
    nn[0] = T
    S = max(c + n for c, n in zip(ctx, nn)) + int(rng.integers(0, 40))
    q = synth.normal_bf16(rng, (B, T, Hkv * G, D))
    kc = synth.normal_bf16(rng, (B, Hkv, S, D))
    vc = synth.normal_bf16(rng, (B, Hkv, S, D))
    parents = np.full((B, T), -1, np.int32)
    for i in range(B):
        parents[i, :nn[i]] = rand_tree(rng, nn[i], 4, 1000)[0]
    ctx_a, nn_a = np.array(ctx, np.int32), np.array(nn, np.int32)
    ref = synth.bf16_bits_to_f32(oracle.tree_attention(q, kc, vc, parents, ctx_a, nn_a)).astype(np.float64)
    for kps in (0, 64, 192):
        out = b.radar_tree_attention(bf16_dev(q), bf16_dev(kc), bf16_dev(vc), dev(parents), dev(ctx_a), dev(nn_a),
                                     keys_per_split=kps)
        torch.cuda.synchronize()
        got = synth.bf16_bits_to_f32(bf16_bits(out)).astype(np.float64)
        assert np.abs(got - ref).max() <= 2e-2, (seed, kps, B, Hkv, G, D, T)
        assert np.all(np.abs(got - ref) <= 6e-3 + 8e-3 * np.abs(ref)), (seed, kps)      # per element, as in test_gpu_attention.py
        assert np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-30) <= 1e-2


@pytest.mark.parametrize("seed", range(8 + EXTRA))
def test_attention_random_long_ranges(oracle, seed):
    """Ranges of eight tiles or more (the long-range kernels): random group sizes, tree sizes, context
    lengths that end anywhere inside a tile, an odd or even number of tiles per range, one or two ranges."""
    from paper_2512_14069_amd import binding as b
    rng = np.random.default_rng(synth.seed_for(57, seed))
    B = int(rng.integers(1, 3))
    Hkv = int(rng.integers(1, 3))
    G = int(rng.choice([1, 2, 3, 4, 5, 8]))
    D = int(rng.choice([128, 128, 128, 64]))
    T = int(rng.integers(1, 65))
    ctx = [int(rng.integers(450, 2300)) for _ in range(B)]
    nn = [int(rng.integers(1, T + 1)) for _ in range(B)]
    nn[0] = T
    S = max(c + n for c, n in zip(ctx, nn)) + int(rng.integers(0, 70))
    q = synth.normal_bf16(rng, (B, T, Hkv * G, D))
    kc = synth.normal_bf16(rng, (B, Hkv, S, D))
    vc = synth.normal_bf16(rng, (B, Hkv, S, D))
    parents = np.full((B, T), -1, np.int32)
    for i in range(B):
        parents[i, :nn[i]] = rand_tree(rng, nn[i], 4, 1000)[0]
    ctx_a, nn_a = np.array(ctx, np.int32), np.array(nn, np.int32)
    ref = synth.bf16_bits_to_f32(oracle.tree_attention(q, kc, vc, parents, ctx_a, nn_a)).astype(np.float64)
    for kps in (512, 1024):
        out = b.radar_tree_attention(bf16_dev(q), bf16_dev(kc), bf16_dev(vc), dev(parents), dev(ctx_a), dev(nn_a),
                                     keys_per_split=kps)
        torch.cuda.synchronize()
        got = synth.bf16_bits_to_f32(bf16_bits(out)).astype(np.float64)
        assert np.all(np.isfinite(got)), (seed, kps)
        assert np.abs(got - ref).max() <= 2e-2, (seed, kps, B, Hkv, G, D, T)
        assert np.all(np.abs(got - ref) <= 6e-3 + 8e-3 * np.abs(ref)), (seed, kps)
        assert np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-30) <= 1e-2


@pytest.mark.parametrize("seed", range(16 + EXTRA))
def test_expand_random_shapes(oracle, seed):
    from paper_2512_14069_amd import binding as b
    rng = np.random.default_rng(synth.seed_for(52, seed))
    V = int(rng.choice([1, 2, 7, 16, 63, 64, 65, 1000, 1023, 4097, 9999, 33333, 70001]))
    k = int(rng.integers(1, min(16, V) + 1))
    F = int(rng.integers(1, 65))
    cap = F * k + 5
    logits = synth.expand_logits(rng, F, V, 3.0, normalised=bool(rng.integers(0, 2)))
    ps = (-rng.random(F) * 4).astype(np.float32)
    pidx = rng.integers(-1, 5, size=F).astype(np.int32)
    gp = b.DraftPool(cap)
    gp.count = 5
    cp = dict(tokens=np.zeros(cap, np.int32), scores=np.zeros(cap, np.float32), parents=np.zeros(cap, np.int32))
    cp["parents"][:5] = -1                              # five earlier candidates, children of the root
    cp["tokens"][:5] = rng.integers(0, V, size=5)
    cp["scores"][:5] = -0.01 * np.arange(5, dtype=np.float32)
    ps = np.minimum(ps, np.where(pidx >= 0, cp["scores"][np.maximum(pidx, 0)], 0).astype(np.float32))   # scores never grow downwards
    for n in ("tokens", "scores", "parents"):
        getattr(gp, n).copy_(dev(cp[n]))
    r = oracle.draft_expand(logits, ps, pidx, k, cp, 5)
    g = b.radar_draft_expand(dev(logits), dev(ps), dev(pidx), k, gp)
    torch.cuda.synchronize()
    # top-k per row: bit-exact unless the k-th and (k+1)-th logit of a row are closer than fp32 can tell
    assert np.array_equal(host(g.cand_tokens).reshape(F, k), r["cand_tokens"]), (seed, F, V, k)
    assert np.max(np.abs(host(g.cand_scores).reshape(F, k).astype(np.float64) - r["cand_scores"])) <= 1e-5
    assert np.array_equal(host(gp.parents)[5:], cp["parents"][5:])
    flat = np.sort(r["cand_scores"].reshape(-1))[::-1].astype(np.float64)
    if len(flat) <= k or np.min(-np.diff(flat[:k + 1])) > 1e-4:
        assert np.array_equal(host(g.frontier_pool_idx), r["frontier_pool_idx"]), (seed, F, V, k)
        assert np.array_equal(host(g.frontier_tokens), r["frontier_tokens"])
    N = int(rng.integers(0, 64))
    gp.scores.copy_(dev(cp["scores"]))
    t = b.radar_draft_rerank(gp, N, 9)
    torch.cuda.synchronize()
    tree = oracle.draft_rerank(cp, cap, N, 9)
    for name in ("tokens", "parents", "depth", "pool_idx"):
        assert np.array_equal(host(getattr(t, name)), tree[name]), (seed, name)


@pytest.mark.parametrize("seed", range(12 + EXTRA))
def test_expand_batch_random_shapes(oracle, seed):
    """radar_draft_expand_batch on batches on both sides of the size from which it streams in two launches."""
    from paper_2512_14069_amd import binding as b
    rng = np.random.default_rng(synth.seed_for(57, seed))
    V = int(rng.choice([63, 1000, 1023, 4097, 9999, 33333, 70001]))
    k = int(rng.integers(1, min(16, V) + 1))
    F = int(rng.integers(1, 33))
    target = (1 << 20) if seed % 2 else (5 << 20)
    B = int(max(2, min(-(-target // (F * V)), 65535 // F, 300)))
    pre = int(rng.integers(0, 8))
    cap = pre + F * k
    logits = np.stack([synth.expand_logits(rng, F, V, 3.0, normalised=bool(rng.integers(0, 2))) for _ in range(B)])
    ps = (-rng.random((B, F)) * 4).astype(np.float32)
    pidx = (rng.integers(0, pre, (B, F)) if pre else np.full((B, F), -1)).astype(np.int32)
    gp = b.DraftPool(cap, B=B)
    gp.count = pre
    g, _ = b.radar_draft_expand_batch(dev(logits), dev(ps), dev(pidx), k, gp)
    torch.cuda.synchronize()
    for q in range(B):
        cp = dict(tokens=np.zeros(cap, np.int32), scores=np.zeros(cap, np.float32), parents=np.zeros(cap, np.int32))
        r = oracle.draft_expand(logits[q], ps[q], pidx[q], k, cp, pre)
        assert np.array_equal(host(g.cand_tokens)[q].reshape(F, k), r["cand_tokens"]), (seed, q, B, F, V, k)
        assert np.max(np.abs(host(g.cand_scores)[q].reshape(F, k).astype(np.float64) - r["cand_scores"])) <= 1e-5
        assert np.array_equal(host(gp.tokens)[q, pre:], cp["tokens"][pre:]) and np.array_equal(host(gp.parents)[q, pre:], cp["parents"][pre:])
        flat = np.sort(r["cand_scores"].reshape(-1))[::-1].astype(np.float64)
        if len(flat) <= k or np.min(-np.diff(flat[:k + 1])) > 1e-4:
            assert np.array_equal(host(g.frontier_pool_idx)[q], r["frontier_pool_idx"]), (seed, q, B, F, V, k)
            assert np.array_equal(host(g.frontier_tokens)[q], r["frontier_tokens"])


@pytest.mark.parametrize("seed", range(16 + EXTRA))
def test_accept_random_shapes(oracle, seed):
    from paper_2512_14069_amd import binding as b
    rng = np.random.default_rng(synth.seed_for(53, seed))
    V = int(rng.choice([1, 3, 64, 1000, 1025, 4095, 4096, 10007, 50000]))
    B = int(rng.integers(1, 6))
    T = int(rng.integers(1, 65))
    nn = np.array([int(rng.integers(1, T + 1)) for _ in range(B)], np.int32)
    tl = synth.gumbel_logits(rng, (B, T, V))
    tokens = np.zeros((B, T), np.int32)
    parents = np.full((B, T), -1, np.int32)
    for i in range(B):
        p, t = rand_tree(rng, int(nn[i]), 5, V)
        parents[i, :nn[i]], tokens[i, :nn[i]] = p, t
        for c in range(1, int(nn[i])):
            if rng.random() < 0.6:
                tl[i, p[c], t[c]] += np.float32(np.log(V) + 2.0)
    temperature = float(rng.choice([1.0, 0.7, 1.5]))
    # tie guard of the inputs: every sequence is decided clear of its thresholds and is compared
    un = tie_free_uniforms(lambda u: (oracle.accept_margins(tl, tokens, parents, nn, u, temperature) > 1e-6).all(axis=1),
                           rng.random((B, T + 1), dtype=np.float32), rng)
    for mode in (0, 1):
        ref = oracle.verify_accept(tl, tokens, parents, nn, un if mode else None, mode=mode, temperature=temperature)
        got = b.radar_verify_accept(dev(tl), dev(tokens), dev(parents), dev(nn), dev(un) if mode else None, mode=mode,
                                    temperature=temperature)
        torch.cuda.synchronize()
        for r_, g_ in zip(ref, got):
            assert np.array_equal(r_, host(g_)), (seed, mode, B, T, V)
    dist = b.radar_accept_length_distribution(dev(tl), dev(tokens), dev(parents), dev(nn), temperature=temperature)
    torch.cuda.synchronize()
    dref = oracle.accept_length_distribution(tl, tokens, parents, nn, temperature=temperature)
    assert np.max(np.abs(host(dist) - dref)) <= 1e-6, (seed, B, T, V)


@pytest.mark.parametrize("seed", range(12 + EXTRA))
def test_accept_q_random_shapes(oracle, seed):
    from paper_2512_14069_amd import binding as b
    rng = np.random.default_rng(synth.seed_for(54, seed))
    V = int(rng.choice([2, 5, 64, 1000, 4097, 8192, 8193, 20011, 40000]))
    B = int(rng.integers(1, 5))
    T = int(rng.integers(1, 41))
    trees = [rand_tree(rng, int(rng.integers(1, T + 1)), 4, V)[0] for _ in range(B)]
    x = synth.sampled_draft_inputs(rng, trees, V, T, std=2.0, noise=float(rng.choice([0.5, 2.0])),
                                   shared_rows=bool(rng.integers(0, 2)))
    D_max = int(rng.integers(0, T)) if rng.random() < 0.3 else None
    kw = dict(temperature=float(rng.choice([1.0, 0.8])), draft_temperature=float(rng.choice([1.0, 1.2])), D_max=D_max)
    def clear(u):
        m = oracle.verify_accept_q(x["target_logits"], x["draft_logits"], x["draft_tokens"], x["parents"], x["n_nodes"],
                                   u, x["q_rows"], want_margins=True, **kw)[3]
        return (m[:, 0] > 1e-5) & (m[:, 1] > 5e-7)
    x["uniforms"] = tie_free_uniforms(clear, x["uniforms"], rng)          # every sequence is compared
    ref = oracle.verify_accept_q(x["target_logits"], x["draft_logits"], x["draft_tokens"], x["parents"], x["n_nodes"],
                                 x["uniforms"], x["q_rows"], **kw)
    for limit in (0, -1, 1):
        got = b.radar_verify_accept_q(dev(x["target_logits"]), dev(x["draft_logits"]), dev(x["draft_tokens"]),
                                      dev(x["parents"]), dev(x["n_nodes"]), dev(x["uniforms"]), dev(x["q_rows"]),
                                      walk_spin_limit=limit, **kw)
        torch.cuda.synchronize()
        for r_, g_ in zip(ref, got):
            assert np.array_equal(r_, host(g_)), (seed, limit, B, T, V)


@pytest.mark.parametrize("seed", range(8 + EXTRA))
def test_policy_random_shapes(oracle, seed):
    from paper_2512_14069_amd import binding as b
    rng = np.random.default_rng(synth.seed_for(55, seed))
    k, M, B = int(rng.integers(1, 17)), int(rng.integers(1, 129)), int(rng.integers(1, 40))
    p = synth.policy_params(rng, k, 128, M, float(rng.choice([1.0, 2.5])))
    pp = b.policy_params({n: dev(v) for n, v in p.items()})
    conf = synth.policy_conf(rng, B, k)[0]
    h0 = rng.uniform(-1, 1, (B, 128)).astype(np.float32)
    c0 = rng.standard_normal((B, 128)).astype(np.float32)
    ref = oracle.policy_step(conf, p, h0, c0)
    out = b.radar_policy_step(dev(conf), pp, dev(h0), dev(c0))
    torch.cuda.synchronize()
    for n in ("h", "c", "logits", "probs"):
        assert np.max(np.abs(host(getattr(out, n)) - ref[n])) <= 5e-5, (seed, n, k, M, B)
    # the same model inside an expansion launch
    V, F = int(rng.choice([777, 5000, 40000])), int(rng.integers(1, 20))
    if k <= V:
        logits = synth.expand_logits(rng, F, V, 2.0)
        ps, pidx = np.zeros(F, np.float32), np.full(F, -1, np.int32)
        pa, pb = b.DraftPool(F * k), b.DraftPool(F * k)
        e1 = b.radar_draft_expand(dev(logits), dev(ps), dev(pidx), k, pa)
        o1 = b.radar_policy_step(e1.frontier_conf, pp, dev(h0[:1]), dev(c0[:1]))
        e2, o2 = b.radar_draft_expand_policy(dev(logits), dev(ps), dev(pidx), k, pb, pp, dev(h0[:1]), dev(c0[:1]))
        torch.cuda.synchronize()
        for n in ("h", "c", "logits", "probs", "action"):
            assert torch.equal(getattr(o1, n), getattr(o2, n)), (seed, n)
        assert torch.equal(e1.frontier_tokens, e2.frontier_tokens)
