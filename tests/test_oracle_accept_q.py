"""Pins of the oracle's verification with draft distributions (Sec. 3, Eq. 1-2).

What the paper and the mathematics fix: the emitted tokens are distributed exactly as the
target's (chi-square over many draws, with the drafted tokens themselves drawn from q); on a
chain the accepted length follows the product of Eq. 1's probabilities; after a rejection the
bonus token follows Eq. 2's rectified distribution; a point-mass q reduces to the fixed-token
rule, whose routine is pinned separately; q = p accepts everything.
"""
import numpy as np
import pytest
from scipy.special import softmax
from scipy.stats import chi2

import oracle
from paper_2512_14069_amd import synth


def chi2_ok(counts, probs, alpha=1e-4):
    n = counts.sum()
    keep = probs * n >= 5
    obs = np.append(counts[keep], counts[~keep].sum())
    exp = np.append(probs[keep] * n, probs[~keep].sum() * n)
    if exp[-1] < 1e-9:
        obs, exp = obs[:-1], exp[:-1]
    stat = ((obs - exp) ** 2 / exp).sum()
    return stat <= chi2.ppf(1 - alpha, len(exp) - 1), stat


def batch_of(x, n):
    """The same tree n times (only uniforms, and tokens where given, differ)."""
    return {k: np.repeat(v, n, axis=0) for k, v in x.items()}


@pytest.mark.parametrize("shared_rows", [True, False])
def test_emitted_tokens_follow_the_target_distribution(shared_rows):
    """Losslessness: tokens drawn from q, verified by the oracle; the first emitted token is
    distributed as p_root, and the second, given the accepted child, as that child's row."""
    V, T, n = 9, 6, 60000
    rng = np.random.default_rng(synth.seed_for(31, int(shared_rows)))
    par = np.array([-1, 0, 0, 0, 1, 1], np.int32)
    base = synth.sampled_draft_inputs(rng, [par], V, T, std=1.2, noise=1.0, shared_rows=shared_rows)
    x = batch_of(base, n)
    # fresh token draws and uniforms per repetition
    for c in range(1, T):
        q = softmax(base["draft_logits"][0, base["q_rows"][0, c]].astype(np.float64))
        x["draft_tokens"][:, c] = rng.choice(V, size=n, p=q)
    x["uniforms"] = rng.random((n, T + 1), dtype=np.float32)
    ln, path, bonus = oracle.verify_accept_q(x["target_logits"], x["draft_logits"], x["draft_tokens"], x["parents"],
                                             x["n_nodes"], x["uniforms"], x["q_rows"])
    first = np.where(ln >= 1, x["draft_tokens"][np.arange(n), np.maximum(path[:, 1], 0)], bonus)
    p_root = softmax(base["target_logits"][0, 0].astype(np.float64))
    ok, stat = chi2_ok(np.bincount(first, minlength=V), p_root)
    assert ok, stat
    assert (ln >= 1).mean() > 0.5                      # the drafts are good enough to be accepted often
    # second token after accepting child 1 (which has children 4 and 5)
    sel = (ln >= 1) & (path[:, 1] == 1)
    second = np.where(ln[sel] >= 2, x["draft_tokens"][sel, np.maximum(path[sel, 2], 0)], bonus[sel])
    ok, stat = chi2_ok(np.bincount(second, minlength=V), softmax(base["target_logits"][0, 1].astype(np.float64)))
    assert ok and sel.sum() > 5000, (stat, sel.sum())
    # ... and after accepting leaf 2 or 3: the bonus is a plain draw from that row
    for leaf in (2, 3):
        sel = (ln == 1) & (path[:, 1] == leaf)
        ok, stat = chi2_ok(np.bincount(bonus[sel], minlength=V), softmax(base["target_logits"][0, leaf].astype(np.float64)))
        assert ok and sel.sum() > 300, (leaf, stat, sel.sum())


def test_chain_length_and_bonus_follow_eq1_and_eq2():
    """Fixed tokens on a chain: P(len >= i) = prod_{j<=i} min(1, p_j(x_j)/q_j(x_j)) (Eq. 1), and
    given a rejection at the root the bonus follows max(0, p - q) normalised (Eq. 2)."""
    V, T, n = 7, 4, 80000
    rng = np.random.default_rng(synth.seed_for(31, 7))
    base = synth.sampled_draft_inputs(rng, [synth.chain_tree(T)], V, T, std=1.0, noise=1.5, shared_rows=False)
    x = batch_of(base, n)
    x["uniforms"] = rng.random((n, T + 1), dtype=np.float32)
    ln, path, bonus = oracle.verify_accept_q(x["target_logits"], x["draft_logits"], x["draft_tokens"], x["parents"],
                                             x["n_nodes"], x["uniforms"])
    alpha = []
    for c in range(1, T):
        p = softmax(base["target_logits"][0, c - 1].astype(np.float64))
        q = softmax(base["draft_logits"][0, c].astype(np.float64))
        t = base["draft_tokens"][0, c]
        alpha.append(min(1.0, p[t] / q[t]))
    reach = np.cumprod([1.0] + alpha)
    probs = np.array([reach[i] * (1 - alpha[i]) if i < T - 1 else reach[i] for i in range(T)])
    assert probs.sum() == pytest.approx(1.0, abs=1e-12)
    ok, stat = chi2_ok(np.bincount(ln, minlength=T), probs)
    assert ok, (stat, probs, np.bincount(ln, minlength=T) / n)
    assert 0.02 < alpha[0] < 0.98                      # both branches at the root are exercised
    p0 = softmax(base["target_logits"][0, 0].astype(np.float64))
    q1 = softmax(base["draft_logits"][0, 1].astype(np.float64))
    rect = np.maximum(0.0, p0 - q1)
    ok, stat = chi2_ok(np.bincount(bonus[ln == 0], minlength=V), rect / rect.sum())
    assert ok, stat
    assert np.all(path[ln == 0, 1:] == -1) and np.all(path[:, 0] == 0)
    full = ln == T - 1                                 # everything accepted: plain draw from the last row
    ok, stat = chi2_ok(np.bincount(bonus[full], minlength=V), softmax(base["target_logits"][0, T - 1].astype(np.float64)))
    assert ok, stat


def test_point_mass_drafts_reduce_to_the_fixed_token_rule():
    """A draft distribution concentrated on the drafted token (logit +80) is the fixed-token case:
    lengths, paths and bonus tokens equal verify_accept's sampling mode on the same uniforms."""
    rng = np.random.default_rng(synth.seed_for(31, 3))
    V, T, B = 50, 14, 300
    trees = [synth.make_tree(rng, T, 3, 3, V) for _ in range(B)]
    tl = synth.normal_logits(rng, (B, T, V), 1.5)
    tokens = np.stack([t[1] for t in trees])
    parents = np.stack([t[0] for t in trees])
    for b in range(B):                                  # lift the drafted tokens so that walks go deep
        for c in range(1, T):
            tl[b, parents[b, c], tokens[b, c]] += 2.0
    tokens[5, 3] = tokens[5, 2] if parents[5, 3] == parents[5, 2] else tokens[5, 3]   # a repeated sibling token
    dl = np.zeros((B, T, V), np.float32)
    for b in range(B):
        dl[b, np.arange(T), tokens[b]] = 80.0
    un = rng.random((B, T + 1), dtype=np.float32)
    nn = np.full(B, T, np.int32)
    got = oracle.verify_accept_q(tl, dl, tokens, parents, nn, un, want_margins=True)
    ref = oracle.verify_accept(tl, tokens, parents, nn, un, mode=1)
    sure = (got[3] > 1e-9).all(axis=1)
    assert sure.mean() > 0.99
    for g, r in zip(got[:3], ref):
        assert np.array_equal(g[sure], r[sure])
    assert got[0].max() == 3 and got[0].min() == 0


def test_identical_distributions_accept_everything_and_cuts_apply():
    rng = np.random.default_rng(synth.seed_for(31, 4))
    V, T = 40, 9
    par = np.array([-1, 0, 0, 1, 1, 3, 2, 5, 5], np.int32)      # first-child chain 0-1-3-5-7
    x = synth.sampled_draft_inputs(rng, [par, par[:4]], V, T, std=2.0, shared_rows=True)
    x["draft_logits"] = x["target_logits"].copy()                # q under node v = p_v (rows shared per parent)
    ln, path, bonus = oracle.verify_accept_q(x["target_logits"], x["draft_logits"], x["draft_tokens"], x["parents"],
                                             x["n_nodes"], x["uniforms"], x["q_rows"])
    assert ln.tolist() == [4, 2]
    assert path[0].tolist()[:5] == [0, 1, 3, 5, 7] and path[1].tolist()[:3] == [0, 1, 3]
    assert np.all(path[1, 3:] == -1)
    ln2, path2, _ = oracle.verify_accept_q(x["target_logits"], x["draft_logits"], x["draft_tokens"], x["parents"],
                                           x["n_nodes"], x["uniforms"], x["q_rows"], D_max=2)
    assert ln2.tolist() == [2, 2] and path2.shape == (2, 3) and path2[0].tolist() == [0, 1, 3]
    # q_rows is only an indirection: the same rows copied out per child give the same result
    dl_full = np.zeros_like(x["draft_logits"])
    for b in range(2):
        for c in range(1, int(x["n_nodes"][b])):
            dl_full[b, c] = x["draft_logits"][b, x["q_rows"][b, c]]
    a = oracle.verify_accept_q(x["target_logits"], dl_full, x["draft_tokens"], x["parents"], x["n_nodes"], x["uniforms"])
    assert all(np.array_equal(p, q) for p, q in zip(a, (ln, path, bonus)))


def test_temperatures_scale_logits_and_bad_arguments():
    rng = np.random.default_rng(synth.seed_for(31, 5))
    V, T = 30, 8
    trees = [synth.make_tree(rng, T, 3, 3, V)[0] for _ in range(40)]
    x = synth.sampled_draft_inputs(rng, trees, V, T, std=2.0, noise=1.0)
    args = (x["draft_tokens"], x["parents"], x["n_nodes"], x["uniforms"], x["q_rows"])
    a = oracle.verify_accept_q(x["target_logits"], x["draft_logits"], *args, want_margins=True)
    b = oracle.verify_accept_q(x["target_logits"] * np.float32(2), x["draft_logits"] * np.float32(0.5), *args,
                               temperature=2.0, draft_temperature=0.5)
    sure = (a[3] > 1e-6).all(axis=1)
    assert sure.sum() >= 35
    for p, q in zip(a[:3], b):
        assert np.array_equal(p[sure], q[sure])
    assert len(set(a[0].tolist())) >= 3                 # several accepted lengths occur
    with pytest.raises(oracle.OracleError):
        oracle.verify_accept_q(x["target_logits"], x["draft_logits"], *args, temperature=0.0)
    with pytest.raises(oracle.OracleError):
        oracle.verify_accept_q(x["target_logits"], x["draft_logits"][:, :5], x["draft_tokens"], x["parents"],
                               x["n_nodes"], x["uniforms"])               # no q_rows and Tq != T
    bad = x["q_rows"].copy(); bad[0, 1] = T
    with pytest.raises(oracle.OracleError):
        oracle.verify_accept_q(x["target_logits"], x["draft_logits"], x["draft_tokens"], x["parents"], x["n_nodes"],
                               x["uniforms"], bad)
