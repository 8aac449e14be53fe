"""Pins for the CPU oracle's tree attention (Sec. 1 / Sec. 3: the serialized draft
tree is verified with masked attention in one target pass).

The paper prints no numbers for this step, so the oracle is pinned to things the
mathematics fixes: a structurally different dense brute force, a library routine
on the chain special case, closed forms and invariances.
"""
import numpy as np
import pytest
import torch

from paper_2512_14069_amd import synth


def f32(bits):
    return synth.bf16_bits_to_f32(bits).astype(np.float64)


def ancestor_closure(parents):
    """reach[i, j] = j is i or an ancestor of i, by boolean matrix squaring of the
    parent adjacency (no chain walking)."""
    n = len(parents)
    A = np.eye(n, dtype=bool)
    for i, p in enumerate(parents):
        if p >= 0:
            A[i, p] = True
    R = A.copy()
    for _ in range(int(np.ceil(np.log2(max(n, 2)))) + 1):
        R = (R.astype(np.int64) @ R.astype(np.int64)) > 0
    return R


def brute_attention(q, kc, vc, parents, ctx_lens, n_nodes, scale=None):
    """Dense fp64 attention over the whole (L+n)x(L+n) additive mask; the last n
    rows are the tree rows.  Returns float64 [B,T,Hq,D] and lse [B,T,Hq]."""
    B, T, Hq, D = q.shape
    Hkv = kc.shape[1]
    G = Hq // Hkv
    scale = 1.0 / np.sqrt(D) if scale is None else scale
    out = np.zeros((B, T, Hq, D))
    lse = np.zeros((B, T, Hq))
    for b in range(B):
        L, n = int(ctx_lens[b]), int(n_nodes[b])
        reach = ancestor_closure(parents[b, :n])
        mask = np.full((L + n, L + n), -np.inf)
        mask[:, :L] = np.where(np.tril(np.ones((L + n, L), bool)), 0.0, -np.inf)
        mask[L:, :L] = 0.0
        mask[L:, L:] = np.where(reach, 0.0, -np.inf)
        for h in range(Hq):
            K = f32(kc[b, h // G, :L + n])
            V = f32(vc[b, h // G, :L + n])
            Qfull = np.zeros((L + n, D))
            Qfull[L:] = f32(q[b, :n, h])
            S = scale * (Qfull @ K.T) + mask
            S = S[L:]
            m = S.max(axis=1, keepdims=True)
            W = np.exp(S - m)
            den = W.sum(axis=1, keepdims=True)
            out[b, :n, h] = (W / den) @ V
            lse[b, :n, h] = (m + np.log(den))[:, 0]
    return out, lse


def bf16_close(bits, ref64, ulps=1.01):
    got = f32(bits)
    tol = np.maximum(np.abs(ref64), 2.0 ** -126) * (2.0 ** -8) * ulps
    return np.all(np.abs(got - ref64) <= tol), np.max(np.abs(got - ref64))


@pytest.mark.parametrize("shuffle", [False, True])
@pytest.mark.parametrize("shape", [
    dict(B=2, Hq=4, Hkv=2, D=16, T=9, ctx=(5, 11), nn=(9, 6), dep=(3, 2)),
    dict(B=1, Hq=4, Hkv=1, D=64, T=16, ctx=(40,), nn=(16,), dep=(4,)),
    dict(B=1, Hq=2, Hkv=2, D=8, T=12, ctx=(0,), nn=(12,), dep=(5,)),
])
def test_matches_dense_masked_brute_force(oracle, shape, shuffle):
    a = synth.AttnShape(B=shape["B"], Hq=shape["Hq"], Hkv=shape["Hkv"], D=shape["D"], T=shape["T"],
                        ctx_lens=shape["ctx"], n_nodes=shape["nn"], depths=shape["dep"], k=3)
    x = synth.attention_inputs(a, seed=11 + shape["T"], shuffle=shuffle)
    out, lse = oracle.tree_attention(x["q"], x["k_cache"], x["v_cache"], x["parents"], x["ctx_lens"],
                                     x["n_nodes"], want_lse=True)
    ref, ref_lse = brute_attention(x["q"], x["k_cache"], x["v_cache"], x["parents"], x["ctx_lens"], x["n_nodes"])
    for b in range(a.B):
        n = a.n_nodes[b]
        ok, err = bf16_close(out[b, :n], ref[b, :n])
        assert ok, f"max err {err}"
        assert np.allclose(lse[b, :n], ref_lse[b, :n], rtol=0, atol=2e-6)
        # rows past n_nodes are zero
        assert np.all(out[b, n:] == 0) and np.all(lse[b, n:] == 0)
    # the rounding is almost always identical
    n0 = a.n_nodes[0]
    same = np.mean(out[0, :n0] == synth.f32_to_bf16_bits(ref[0, :n0].astype(np.float32)))
    assert same > 0.98


def test_chain_tree_is_causal_attention_library(oracle):
    """parents[i] = i-1 makes the tree a sequence: the tree rows then equal the last
    T rows of ordinary causal attention (torch's CPU routine, fp32)."""
    B, Hq, Hkv, D, T, L = 1, 4, 2, 32, 7, 19
    rng = np.random.default_rng(5)
    q = synth.normal_bf16(rng, (B, T, Hq, D))
    kc = synth.normal_bf16(rng, (B, Hkv, L + T, D))
    vc = synth.normal_bf16(rng, (B, Hkv, L + T, D))
    parents = synth.chain_tree(T)[None]
    out = oracle.tree_attention(q, kc, vc, parents, np.array([L], np.int32))
    G = Hq // Hkv
    qt = torch.zeros(B, Hq, L + T, D)
    qt[:, :, L:] = torch.from_numpy(synth.bf16_bits_to_f32(q)).permute(0, 2, 1, 3)
    kt = torch.from_numpy(synth.bf16_bits_to_f32(kc)).repeat_interleave(G, dim=1)
    vt = torch.from_numpy(synth.bf16_bits_to_f32(vc)).repeat_interleave(G, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, is_causal=True)
    ref = ref[:, :, L:].permute(0, 2, 1, 3).numpy().astype(np.float64)
    assert np.max(np.abs(f32(out) - ref)) < 2e-2 * 0.5
    assert np.allclose(f32(out), ref, rtol=2 ** -7, atol=1e-5)


def test_equal_keys_give_mean_of_allowed_values(oracle):
    """If every K row is the same vector all scores are equal, so each node's output
    is the plain mean of the V rows it may see: prefix + itself + its ancestors."""
    B, Hq, Hkv, D, T, L = 1, 2, 1, 16, 10, 6
    rng = np.random.default_rng(8)
    a = synth.AttnShape(B, Hq, Hkv, D, T, (L,), (T,), (4,), k=3)
    x = synth.attention_inputs(a, seed=3)
    krow = synth.normal_bf16(rng, (D,))
    x["k_cache"][:] = krow
    out = oracle.tree_attention(x["q"], x["k_cache"], x["v_cache"], x["parents"], x["ctx_lens"])
    V = f32(x["v_cache"][0, 0])
    par = x["parents"][0]
    for i in range(T):
        rows = list(range(L))
        j = i
        while j >= 0:
            rows.append(L + j)
            j = par[j]
        expect = V[rows].mean(axis=0)
        for h in range(Hq):
            ok, err = bf16_close(out[0, i, h], expect)
            assert ok, (i, h, err)


def test_star_tree_sees_prefix_root_and_self_only(oracle):
    B, Hq, Hkv, D, T, L = 1, 2, 2, 8, 6, 4
    rng = np.random.default_rng(21)
    q = synth.normal_bf16(rng, (B, T, Hq, D))
    kc = synth.normal_bf16(rng, (B, Hkv, L + T, D))
    vc = synth.normal_bf16(rng, (B, Hkv, L + T, D))
    parents = synth.star_tree(T)[None]
    out = oracle.tree_attention(q, kc, vc, parents, np.array([L], np.int32))
    for i in range(1, T):
        rows = list(range(L)) + [L, L + i]
        for h in range(Hq):
            s = (f32(q[0, i, h]) @ f32(kc[0, h, rows]).T) / np.sqrt(D)
            w = np.exp(s - s.max())
            w /= w.sum()
            assert abs(w.sum() - 1) < 1e-12
            ok, err = bf16_close(out[0, i, h], w @ f32(vc[0, h, rows]))
            assert ok, err


def test_empty_prefix_root_returns_its_own_value(oracle):
    B, Hq, Hkv, D, T = 1, 4, 2, 16, 5
    a = synth.AttnShape(B, Hq, Hkv, D, T, (0,), (T,), (2,), k=3)
    x = synth.attention_inputs(a, seed=4)
    out = oracle.tree_attention(x["q"], x["k_cache"], x["v_cache"], x["parents"], x["ctx_lens"])
    for h in range(Hq):
        assert np.array_equal(out[0, 0, h], x["v_cache"][0, h // 2, 0])


def test_non_ancestors_and_padding_do_not_matter(oracle):
    """Changing K/V of a node that is not an ancestor of i, of rows past the tree,
    or parents past n_nodes leaves row i bit-identical."""
    a = synth.AttnShape(1, 4, 2, 16, 12, (9,), (10,), (3,), k=3)
    x = synth.attention_inputs(a, seed=77)
    base = oracle.tree_attention(x["q"], x["k_cache"], x["v_cache"], x["parents"], x["ctx_lens"], x["n_nodes"])
    par = x["parents"][0]
    L, n = 9, 10
    rng = np.random.default_rng(1)
    for victim in range(1, n):
        k2, v2 = x["k_cache"].copy(), x["v_cache"].copy()
        k2[0, :, L + victim] = synth.normal_bf16(rng, (2, 16))
        v2[0, :, L + victim] = synth.normal_bf16(rng, (2, 16))
        k2[0, :, L + n:] = synth.normal_bf16(rng, k2[0, :, L + n:].shape)
        p2 = x["parents"].copy()
        p2[0, n:] = 0
        out = oracle.tree_attention(x["q"], k2, v2, p2, x["ctx_lens"], x["n_nodes"])
        reach = ancestor_closure(par[:n])
        for i in range(n):
            if not reach[i, victim]:
                assert np.array_equal(out[0, i], base[0, i]), (victim, i)
            else:
                assert not np.array_equal(out[0, i], base[0, i])


def test_lse_is_log_of_softmax_denominator(oracle):
    from scipy.special import logsumexp
    a = synth.AttnShape(1, 2, 1, 32, 8, (33,), (8,), (3,), k=3)
    x = synth.attention_inputs(a, seed=9)
    _, lse = oracle.tree_attention(x["q"], x["k_cache"], x["v_cache"], x["parents"], x["ctx_lens"], want_lse=True)
    reach = ancestor_closure(x["parents"][0])
    for i in range(8):
        rows = list(range(33)) + [33 + j for j in range(8) if reach[i, j]]
        for h in range(2):
            s = f32(x["q"][0, i, h]) @ f32(x["k_cache"][0, 0, rows]).T / np.sqrt(32)
            assert abs(lse[0, i, h] - logsumexp(s)) < 2e-6


def test_scale_argument_and_bad_trees(oracle):
    a = synth.AttnShape(1, 2, 1, 8, 5, (3,), (5,), (2,), k=3)
    x = synth.attention_inputs(a, seed=2)
    o1 = oracle.tree_attention(x["q"], x["k_cache"], x["v_cache"], x["parents"], x["ctx_lens"], scale=0.25)
    ref, _ = brute_attention(x["q"], x["k_cache"], x["v_cache"], x["parents"], x["ctx_lens"], [5], scale=0.25)
    assert bf16_close(o1, ref)[0]
    bad = x["parents"].copy()
    bad[0, 2] = 3                      # parent after child
    with pytest.raises(oracle.OracleError):
        oracle.tree_attention(x["q"], x["k_cache"], x["v_cache"], bad, x["ctx_lens"])
