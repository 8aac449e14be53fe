"""Pins for the CPU oracle's acceptance walk (Sec. 3, Eq. 1-2; the tree form of
Sec. 4.3, Eq. 11-13; greedy = the temperature-0 rows of the appendix's
temperature table)."""
import numpy as np
import pytest
from scipy.special import softmax
from scipy.stats import chi2

from paper_2512_14069_amd import synth


def all_root_to_leaf_paths(parents):
    n = len(parents)
    kids = [[] for _ in range(n)]
    for c in range(1, n):
        kids[parents[c]].append(c)
    paths = []

    def rec(node, path):
        if not kids[node]:
            paths.append(path)
        for c in kids[node]:
            rec(c, path + [c])
    rec(0, [0])
    return paths


def brute_greedy(logits, tokens, parents):
    """Every root-to-leaf path; for each the longest prefix whose tokens follow the
    target's argmax chain; the longest over all paths (unique: sibling tokens differ)."""
    best = [0]
    for path in all_root_to_leaf_paths(parents):
        good = [0]
        for a, c in zip(path[:-1], path[1:]):
            if tokens[c] == int(np.argmax(logits[a])):
                good.append(c)
            else:
                break
        if len(good) > len(best):
            best = good
    return best


@pytest.mark.parametrize("seed", range(6))
def test_greedy_against_path_enumeration(oracle, seed):
    rng = np.random.default_rng(seed)
    V = 257
    depth = int(rng.integers(1, 6))
    n = int(rng.integers(depth + 1, min(24, 1 + 3 + 9 * (depth - 1)) + 1))
    parents, tokens, depths = synth.make_tree(rng, n, depth, 3, V, shuffle=bool(seed % 2))
    logits = synth.gumbel_logits(rng, (n, V))
    synth.plant_greedy_path(rng, logits, parents, tokens, prob=0.8)
    alen, path, bonus = oracle.verify_accept(logits[None], tokens[None], parents[None])
    ref = brute_greedy(logits, tokens, parents)
    assert alen[0] == len(ref) - 1
    assert list(path[0, :len(ref)]) == ref and np.all(path[0, len(ref):] == -1)
    assert bonus[0] == int(np.argmax(logits[ref[-1]]))
    assert alen[0] <= depths.max()
    for a, c in zip(ref[:-1], ref[1:]):
        assert parents[c] == a


def test_greedy_planted_chain_and_all_wrong(oracle):
    V, n = 100, 6
    rng = np.random.default_rng(0)
    parents = synth.chain_tree(n)
    tokens = rng.integers(0, V, n).astype(np.int32)
    logits = synth.gumbel_logits(rng, (n, V))
    for i in range(n - 1):
        logits[i, tokens[i + 1]] = 50.0
    alen, path, bonus = oracle.verify_accept(logits[None], tokens[None], parents[None])
    assert alen[0] == n - 1 and list(path[0]) == list(range(n))
    assert bonus[0] == int(np.argmax(logits[n - 1]))
    # no child ever matches
    logits2 = synth.gumbel_logits(rng, (n, V))
    for i in range(n - 1):
        logits2[i, tokens[i + 1]] = -50.0
    alen, path, bonus = oracle.verify_accept(logits2[None], tokens[None], parents[None])
    assert alen[0] == 0 and path[0, 0] == 0 and np.all(path[0, 1:] == -1)
    assert bonus[0] == int(np.argmax(logits2[0]))


def test_greedy_argmax_tie_takes_lowest_index_and_ragged_batch(oracle):
    V, T = 16, 5
    logits = np.zeros((2, T, V), np.float32)
    logits[0, 0, [3, 9]] = 2.0                     # tie: 3 wins
    parents = np.array([[-1, 0, 0, 1, 1], [-1, 0, 0, 0, 0]], np.int32)
    tokens = np.array([[0, 9, 3, 0, 1], [0, 0, 1, 2, 3]], np.int32)
    logits[0, 2, 7] = 1.0
    logits[1, 0, 3] = 5.0                          # node 4 carries token 3 but is past n_nodes
    n_nodes = np.array([5, 4], np.int32)
    alen, path, bonus = oracle.verify_accept(logits, tokens, parents, n_nodes=n_nodes)
    assert list(alen) == [1, 0]
    assert list(path[0, :2]) == [0, 2] and bonus[0] == 7
    assert bonus[1] == 3


# ---------------------------------------------------------------- sampling

def accept_length_distribution(P, tokens, parents, depths):
    """Eq. 11-13 with P_acc(child | parent) = p_parent(token of child):
    P_stop(v) = P_acc(path to v) * (1 - sum over children of p_v(token)),
    p_i = sum of P_stop over nodes of depth i."""
    n = len(parents)
    reach = np.zeros(n)
    reach[0] = 1.0
    dist = np.zeros(depths.max() + 1)
    for v in range(n):
        if v > 0:
            reach[v] = reach[parents[v]] * P[parents[v], tokens[v]]
    for v in range(n):
        kids = np.nonzero(parents == v)[0]
        dist[depths[v]] += reach[v] * (1.0 - P[v, tokens[kids]].sum())
    return dist


def tiny_sampling_case(seed, V=8, n=9, depth=3, k=3, temperature=1.0):
    rng = np.random.default_rng(seed)
    parents, tokens, depths = synth.make_tree(rng, n, depth, k, V)
    logits = synth.normal_logits(rng, (n, V), 1.5)
    P = softmax(logits.astype(np.float64) / temperature, axis=1)
    return rng, parents, tokens, depths, logits, P


@pytest.mark.parametrize("seed,temperature", [(1, 1.0), (2, 0.7), (3, 1.0)])
def test_sampling_matches_closed_form_length_distribution_and_is_lossless(oracle, seed, temperature):
    rng, parents, tokens, depths, logits, P = tiny_sampling_case(seed, temperature=temperature)
    n, V = logits.shape
    M = 200_000
    u = rng.random((M, n + 1), dtype=np.float32)
    alen, path, bonus = oracle.verify_accept(
        np.broadcast_to(logits, (M, n, V)), np.broadcast_to(tokens, (M, n)), np.broadcast_to(parents, (M, n)),
        uniforms=u, mode=1, temperature=temperature)
    # (1) acceptance-length histogram against Eq. 11-13
    dist = accept_length_distribution(P, tokens, parents, depths)
    assert abs(dist.sum() - 1.0) < 1e-12
    # the oracle's own Eq. 11-13 routine: same numbers as the formula written out above
    # (and so, through the histogram below, as the sampler it describes)
    od = oracle.accept_length_distribution(logits[None], tokens[None], parents[None], temperature=temperature)[0]
    # (the interface carries the temperature as fp32: 0.7 arrives as 0.69999999)
    assert np.allclose(od[:len(dist)], dist, rtol=0, atol=1e-8) and np.all(od[len(dist):] == 0)
    hist = np.bincount(alen, minlength=len(dist)) / M
    sigma = np.sqrt(dist * (1 - dist) / M)
    assert np.all(np.abs(hist - dist) <= 4 * sigma + 1e-9), (hist, dist)
    # (2) losslessness: the first emitted token follows the target's row-0 law
    first = np.where(alen >= 1, tokens[np.clip(path[:, 1], 0, n - 1)], bonus)
    counts = np.bincount(first, minlength=V)
    stat = np.sum((counts - M * P[0]) ** 2 / (M * P[0]))
    assert stat < chi2.ppf(1 - 1e-4, V - 1), stat
    # (3) second emitted token given the first accepted child is also the target's law
    c1 = int(np.nonzero(parents == 0)[0][0])
    sel = (alen >= 1) & (path[:, 1] == c1)
    second = np.where(alen[sel] >= 2, tokens[np.clip(path[sel, 2], 0, n - 1)], bonus[sel])
    cnt2 = np.bincount(second, minlength=V)
    m2 = sel.sum()
    stat2 = np.sum((cnt2 - m2 * P[c1]) ** 2 / (m2 * P[c1]))
    assert stat2 < chi2.ppf(1 - 1e-4, V - 1), stat2
    # paths are root chains and never longer than the tree is deep
    assert alen.max() <= depths.max()


def test_sampling_extreme_uniforms(oracle):
    rng, parents, tokens, depths, logits, P = tiny_sampling_case(5)
    n, V = logits.shape
    u0 = np.zeros((1, n + 1), np.float32)
    alen, path, bonus = oracle.verify_accept(logits[None], tokens[None], parents[None], uniforms=u0, mode=1)
    # u = 0: always the first child, down to a leaf; bonus = first token with mass
    cur, ref = 0, [0]
    while True:
        kids = np.nonzero(parents == cur)[0]
        if not len(kids):
            break
        cur = int(kids[0])
        ref.append(cur)
    assert list(path[0, :len(ref)]) == ref and alen[0] == len(ref) - 1
    assert bonus[0] == 0
    u1 = np.full((1, n + 1), np.nextafter(np.float32(1), np.float32(0)), np.float32)
    alen, path, bonus = oracle.verify_accept(logits[None], tokens[None], parents[None], uniforms=u1, mode=1)
    assert alen[0] == 0
    kids0 = set(int(t) for t in tokens[parents == 0])
    assert bonus[0] == max(v for v in range(V) if v not in kids0)


def test_sampling_bonus_is_inverse_cdf_of_residual(oracle):
    """Single node, no children: bonus = inverse CDF of softmax(row) at u; with
    children all rejected: their tokens are excluded and the rest renormalised."""
    rng = np.random.default_rng(9)
    V = 50
    logits = synth.normal_logits(rng, (1, 1, V), 1.0)
    p = softmax(logits[0, 0].astype(np.float64))
    cdf = np.cumsum(p)
    for uu in [0.0, 0.1, 0.37, 0.5, 0.93, 0.999]:
        u = np.array([[0.0, uu]], np.float32)
        _, _, bonus = oracle.verify_accept(logits, np.zeros((1, 1), np.int32), np.array([[-1]], np.int32),
                                           uniforms=u, mode=1)
        assert bonus[0] == int(np.searchsorted(cdf, np.float32(uu), side="right"))
    # root with two children that are both rejected (u = 1-)
    T = 3
    logits3 = np.repeat(logits, T, axis=1)
    tokens = np.array([[0, 7, 20]], np.int32)
    parents = np.array([[-1, 0, 0]], np.int32)
    hi = np.nextafter(np.float32(1), np.float32(0))
    for uu in [0.05, 0.5, 0.8]:
        u = np.array([[0, hi, hi, uu]], np.float32)
        alen, _, bonus = oracle.verify_accept(logits3, tokens, parents, uniforms=u, mode=1)
        assert alen[0] == 0
        pr = p.copy()
        pr[[7, 20]] = 0
        pr /= pr.sum()
        assert bonus[0] == int(np.searchsorted(np.cumsum(pr), np.float32(uu), side="right"))


def test_sampling_low_temperature_equals_greedy(oracle):
    rng = np.random.default_rng(13)
    V, n = 64, 14
    parents, tokens, depths = synth.make_tree(rng, n, 4, 3, V)
    logits = synth.gumbel_logits(rng, (n, V))
    synth.plant_greedy_path(rng, logits, parents, tokens, prob=0.9)
    g = oracle.verify_accept(logits[None], tokens[None], parents[None])
    u = rng.random((1, n + 1), dtype=np.float32) * 0.98 + 0.01
    s = oracle.verify_accept(logits[None], tokens[None], parents[None], uniforms=u, mode=1, temperature=1e-3)
    assert g[0][0] == s[0][0] and np.array_equal(g[1], s[1]) and g[2][0] == s[2][0]


def test_sampling_margins_and_bad_arguments(oracle):
    rng, parents, tokens, depths, logits, P = tiny_sampling_case(7)
    n, V = logits.shape
    u = rng.random((3, n + 1), dtype=np.float32)
    m = oracle.accept_margins(np.broadcast_to(logits, (3, n, V)), np.broadcast_to(tokens, (3, n)),
                              np.broadcast_to(parents, (3, n)), None, u)
    assert m.shape == (3, 2) and np.all(m >= 0)
    with pytest.raises(oracle.OracleError):
        oracle.verify_accept(logits[None], tokens[None], parents[None], mode=1)          # no uniforms
    with pytest.raises(oracle.OracleError):
        oracle.verify_accept(logits[None], tokens[None], parents[None], uniforms=u[:1], mode=1, temperature=0.0)
    with pytest.raises(oracle.OracleError):
        oracle.verify_accept(logits[None], tokens[None], synth.chain_tree(n)[None], D_max=1,
                             uniforms=np.zeros((1, n + 1), np.float32), mode=1)            # path longer than D_max


# ------------------------------------------------- acceptance-length distribution (Eq. 11-13)

def test_length_distribution_chain_closed_form(oracle):
    """Chain tree: length i means the first i tokens were accepted and token i+1 was not:
    dist[i] = a_1 ... a_i (1 - a_{i+1}), a_j = p_{j-1}(token j); the leaf keeps what reaches it."""
    rng = np.random.default_rng(21)
    n, V, temperature = 7, 11, 0.8
    parents = synth.chain_tree(n)
    tokens = rng.integers(0, V, size=n).astype(np.int32)
    logits = synth.normal_logits(rng, (n, V), 1.0)
    P = softmax(logits.astype(np.float64) / np.float64(np.float32(temperature)), axis=1)
    a = np.array([P[j - 1, tokens[j]] for j in range(1, n)])
    want = np.array([np.prod(a[:i]) * (1 - a[i] if i < n - 1 else 1.0) for i in range(n)])
    got = oracle.accept_length_distribution(logits[None], tokens[None], parents[None], temperature=temperature)[0]
    assert np.allclose(got, want, rtol=0, atol=1e-13)
    assert abs(got.sum() - 1) < 1e-13


def test_length_distribution_depth_cut_folds_the_tail(oracle):
    """Cutting the walk at D_max leaves shorter lengths alone and puts all deeper mass on D_max."""
    rng, parents, tokens, depths, logits, P = tiny_sampling_case(8, n=12, depth=4)
    full = oracle.accept_length_distribution(logits[None], tokens[None], parents[None])[0]
    for d in range(0, 4):
        cut = oracle.accept_length_distribution(logits[None], tokens[None], parents[None], D_max=d)[0]
        assert cut.shape == (d + 1,)
        assert np.allclose(cut[:d], full[:d], atol=1e-14) and abs(cut[d] - full[d:].sum()) < 1e-13


def test_length_distribution_repeated_sibling_token_and_ragged_batch(oracle):
    """A child that repeats an earlier sibling's token is never reached: the distribution equals
    the one of the tree without that child's subtree.  Rows past n_nodes are ignored."""
    rng = np.random.default_rng(31)
    V = 9
    parents = np.array([-1, 0, 0, 0, 1, 3, 3, 5], np.int32)
    tokens = np.array([0, 4, 2, 4, 1, 6, 7, 3], np.int32)           # node 3 repeats node 1's token
    logits = synth.normal_logits(rng, (8, V), 1.2)
    got = oracle.accept_length_distribution(logits[None], tokens[None], parents[None])[0]
    keep = np.array([0, 1, 2, 4])                                    # drop node 3 and everything under it
    remap = {0: 0, 1: 1, 2: 2, 4: 3}
    p2 = np.array([-1] + [remap[int(parents[v])] for v in keep[1:]], np.int32)
    pad = np.zeros((8, V), np.float32); pad[:4] = logits[keep]
    tp = np.zeros(8, np.int32); tp[:4] = tokens[keep]
    pp = np.full(8, 5, np.int32); pp[:4] = p2                         # junk parents past n_nodes
    want = oracle.accept_length_distribution(pad[None], tp[None], pp[None], n_nodes=np.array([4], np.int32))[0]
    assert np.allclose(got, want, atol=1e-14)
    indep = accept_length_distribution(softmax(pad[:4].astype(np.float64), axis=1), tp[:4], p2, np.array([0, 1, 1, 2]))
    assert np.allclose(want[:3], indep, atol=1e-12)


def test_length_distribution_bad_arguments(oracle):
    from oracle import OracleError
    z = np.zeros((1, 3, 5), np.float32)
    t = np.zeros((1, 3), np.int32)
    with pytest.raises(OracleError):
        oracle.accept_length_distribution(z, t, np.array([[-1, 0, 1]], np.int32), temperature=0.0)
    with pytest.raises(OracleError):
        oracle.accept_length_distribution(z, t, np.array([[-1, 2, 0]], np.int32))      # parent after child
