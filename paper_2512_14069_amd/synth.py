"""Seeded synthetic inputs for the RADAR hot path (numpy only).

This module serves both the HIP path and the CPU oracle and therefore holds
none of the method's arithmetic: it draws random tensors, lays out draft trees
and names the benchmark configurations.  It imports neither the HIP binding nor
the oracle.

The shapes follow the paper's setting (Sec. 5.1: branching factor k = 10, at
most 8 draft calls, batch 1; LLaMA-3.1-8B-class and 70B-class targets) and the
five configurations of this build's baseline description.  They stand in for
the paper's MT-bench / GSM8K / Alpaca / MBPP runs: no item of those suites is
used.
"""
from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 20251214


def seed_for(config, trial=0):
    return BASE_SEED + 1000 * int(config) + int(trial)


# ----------------------------------------------------------------- bf16 bits

def f32_to_bf16_bits(x):
    """float32 array -> uint16 bf16 bit patterns, round to nearest even."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = ((u + 0x7FFF + lsb) >> 16).astype(np.uint16)
    nan = np.isnan(x)
    if nan.any():
        r = np.where(nan, np.uint16(0x7FC0), r)
    return r


def bf16_bits_to_f32(b):
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32)


def normal_bf16(rng, shape, std=1.0):
    """N(0, std^2) samples rounded to bf16, as uint16 bit patterns."""
    return f32_to_bf16_bits((rng.standard_normal(shape, dtype=np.float32) * np.float32(std)))


# --------------------------------------------------------------------- trees

def level_sizes(rng, n_nodes, depth, k):
    """Split n_nodes-1 non-root nodes over `depth` levels: every level >= 1 node,
    level 1 <= k nodes, level l <= k * min(k, size(l-1)) nodes."""
    n = n_nodes - 1
    if depth < 1 or n < depth:
        raise ValueError("need at least one node per level")
    sizes = [1] * depth
    left = n - depth
    guard = 0
    while left > 0:
        l = int(rng.integers(0, depth))
        cap = k if l == 0 else k * min(k, sizes[l - 1])
        if sizes[l] < cap:
            sizes[l] += 1
            left -= 1
        guard += 1
        if guard > 100000:
            raise ValueError("tree does not fit the level caps")
    return sizes


def make_tree(rng, n_nodes, depth, k, vocab, shuffle=False):
    """A draft tree like the ones dynamic-depth drafting produces.

    Node 0 is the root (parent -1).  Level l nodes pick their parent uniformly
    among at most k "frontier" nodes of level l-1 (the nodes that were expanded),
    each parent getting at most k children; sibling tokens are distinct.  Nodes
    are numbered level by level, or, with shuffle=True, in a random order that
    still puts every parent before its children.

    Returns parents int32[n_nodes], tokens int32[n_nodes], depths int32[n_nodes].
    """
    sizes = level_sizes(rng, n_nodes, depth, k) if n_nodes > 1 else []
    parents = [-1]
    depths = [0]
    prev = [0]
    for l, sz in enumerate(sizes, start=1):
        frontier = list(rng.permutation(prev)[:k])
        # guarantee capacity: at most k children each
        slots = []
        for f in frontier:
            slots += [f] * k
        slots = list(rng.permutation(slots))
        chosen = slots[:sz]
        cur = []
        for p in sorted(chosen):
            parents.append(int(p))
            depths.append(l)
            cur.append(len(parents) - 1)
        prev = cur
    parents = np.asarray(parents, np.int32)
    depths = np.asarray(depths, np.int32)
    n = len(parents)

    if shuffle and n > 2:
        # random topological relabeling: repeatedly emit a random ready node
        children = [[] for _ in range(n)]
        for c in range(1, n):
            children[parents[c]].append(c)
        order, ready = [], [0]
        while ready:
            j = int(rng.integers(0, len(ready)))
            node = ready.pop(j)
            order.append(node)
            ready += children[node]
        new_of = np.empty(n, np.int64)
        new_of[order] = np.arange(n)
        p2 = np.full(n, -1, np.int32)
        d2 = np.zeros(n, np.int32)
        for old in range(n):
            p2[new_of[old]] = -1 if parents[old] < 0 else new_of[parents[old]]
            d2[new_of[old]] = depths[old]
        parents, depths = p2, d2

    tokens = np.zeros(n, np.int32)
    tokens[0] = int(rng.integers(0, vocab))
    for p in range(n):
        kids = np.nonzero(parents == p)[0]
        if len(kids):
            tokens[kids] = rng.choice(vocab, size=len(kids), replace=False).astype(np.int32)
    return parents, tokens, depths


def chain_tree(n_nodes):
    return np.arange(-1, n_nodes - 1, dtype=np.int32)


def star_tree(n_nodes):
    p = np.zeros(n_nodes, np.int32)
    p[0] = -1
    return p


# -------------------------------------------------------------------- logits

def gumbel_logits(rng, shape):
    """N(0,1) + Gumbel(0,1) in fp32: equal maxima have probability ~0."""
    g = rng.standard_normal(shape, dtype=np.float32)
    u = rng.random(shape, dtype=np.float32)
    u = np.clip(u, np.float32(1e-7), np.float32(1.0 - 1e-7))
    return (g - np.log(-np.log(u))).astype(np.float32)


def normal_logits(rng, shape, std):
    return (rng.standard_normal(shape, dtype=np.float32) * np.float32(std)).astype(np.float32)


PLANT_LOGIT = np.float32(64.0)


def plant_greedy_path(rng, logits, parents, tokens, prob=0.75):
    """For each node that has children, with probability `prob` make one child's
    token the clear maximum of that node's logits row (by overwriting that entry
    with a constant far above the noise), so accepted lengths spread over
    0..depth like the paper's acceptance lengths.  In place; returns logits."""
    n = len(parents)
    for p in range(n):
        kids = np.nonzero(parents == p)[0]
        if len(kids) and rng.random() < prob:
            c = int(kids[int(rng.integers(0, len(kids)))])
            logits[p, tokens[c]] = PLANT_LOGIT + np.float32(rng.random())
    return logits


# ------------------------------------------------------------ configurations

@dataclass
class AttnShape:
    B: int
    Hq: int
    Hkv: int
    D: int
    T: int                     # serialized tree rows (root included)
    ctx_lens: tuple            # per sequence
    n_nodes: tuple             # per sequence
    depths: tuple              # per sequence
    k: int = 10

    @property
    def S(self):
        return max(self.ctx_lens) + self.T


@dataclass
class Config:
    cid: int
    name: str
    attn: AttnShape
    vocab: int
    k: int
    N: int                     # nodes kept by rerank
    expand_steps: int
    F: int
    modes: tuple = ("greedy",)
    logit_std: float = 1.0
    extra: dict = field(default_factory=dict)


def config(cid, trial=0):
    """The five configurations; ragged ones draw their lengths from the seed."""
    if cid == 1:
        a = AttnShape(B=1, Hq=4, Hkv=1, D=64, T=16, ctx_lens=(256,), n_nodes=(16,), depths=(4,), k=4)
        return Config(1, "c1_smoke", a, vocab=4096, k=4, N=15, expand_steps=4, F=4, logit_std=2.0)
    if cid == 2:
        a = AttnShape(B=1, Hq=32, Hkv=8, D=128, T=60, ctx_lens=(2048,), n_nodes=(60,), depths=(8,))
        return Config(2, "c2_8b_verify", a, vocab=128256, k=10, N=59, expand_steps=8, F=10)
    if cid == 3:
        a = AttnShape(B=1, Hq=32, Hkv=8, D=128, T=61, ctx_lens=(2048,), n_nodes=(61,), depths=(8,))
        return Config(3, "c3_8b_expand", a, vocab=128256, k=10, N=60, expand_steps=8, F=10,
                      modes=("sampling",), logit_std=3.0)
    if cid == 4:
        rng = np.random.default_rng(seed_for(4, trial))
        B = 16
        ctx = tuple(int(x) for x in rng.integers(512, 8193, size=B))
        dep = tuple(int(x) for x in rng.integers(1, 9, size=B))
        # a depth-d tree of branching 10 holds at most 1 + 10 + (d-1)*100 nodes
        nn = tuple(int(rng.integers(d + 1, min(60, 1 + 10 + (d - 1) * 100) + 1)) for d in dep)
        a = AttnShape(B=B, Hq=32, Hkv=8, D=128, T=60, ctx_lens=ctx, n_nodes=nn, depths=dep)
        return Config(4, "c4_ragged", a, vocab=128256, k=10, N=59, expand_steps=8, F=10)
    if cid == 5:
        a = AttnShape(B=4, Hq=64, Hkv=8, D=128, T=60, ctx_lens=(16384,) * 4, n_nodes=(60,) * 4,
                      depths=(8,) * 4)
        return Config(5, "c5_70b_verify", a, vocab=128256, k=10, N=59, expand_steps=8, F=10,
                      modes=("greedy", "sampling"))
    raise ValueError(f"unknown config {cid}")


def attention_inputs(a, seed, shuffle=False, S=None):
    """q uint16[B,T,Hq,D], k_cache/v_cache uint16[B,Hkv,S,D] (~N(0,1) in bf16),
    parents int32[B,T], ctx_lens int32[B], n_nodes int32[B].  Cache rows past
    ctx_len+n_nodes and tree rows past n_nodes hold noise as well: they must not
    influence any output."""
    rng = np.random.default_rng(seed)
    S = a.S if S is None else S
    q = normal_bf16(rng, (a.B, a.T, a.Hq, a.D))
    kc = normal_bf16(rng, (a.B, a.Hkv, S, a.D))
    vc = normal_bf16(rng, (a.B, a.Hkv, S, a.D))
    parents = np.full((a.B, a.T), -1, np.int32)
    for b in range(a.B):
        nn, dep = a.n_nodes[b], a.depths[b]
        if nn > 1:
            p, _, _ = make_tree(rng, nn, min(dep, nn - 1), a.k, 1 << 20, shuffle=shuffle)
            parents[b, :nn] = p
        # rows >= n_nodes: arbitrary but in-range values that must be ignored
        for i in range(nn, a.T):
            parents[b, i] = int(rng.integers(0, max(i, 1))) if i > 0 else -1
    return dict(q=q, k_cache=kc, v_cache=vc, parents=parents,
                ctx_lens=np.asarray(a.ctx_lens, np.int32), n_nodes=np.asarray(a.n_nodes, np.int32))


def accept_inputs(a, vocab, seed, plant=0.75, shuffle=False):
    """target_logits float32[B,T,V] (N(0,1)+Gumbel, planted argmax path),
    draft_tokens/parents int32[B,T], n_nodes int32[B], uniforms float32[B,T+1]."""
    rng = np.random.default_rng(seed)
    logits = gumbel_logits(rng, (a.B, a.T, vocab))
    parents = np.full((a.B, a.T), -1, np.int32)
    tokens = np.zeros((a.B, a.T), np.int32)
    for b in range(a.B):
        nn, dep = a.n_nodes[b], a.depths[b]
        if nn > 1:
            p, t, _ = make_tree(rng, nn, min(dep, nn - 1), a.k, vocab, shuffle=shuffle)
        else:
            p, t = np.asarray([-1], np.int32), rng.integers(0, vocab, size=1).astype(np.int32)
        parents[b, :nn] = p
        tokens[b, :nn] = t
        plant_greedy_path(rng, logits[b], p, t, prob=plant)
        for i in range(nn, a.T):
            parents[b, i] = int(rng.integers(0, max(i, 1))) if i > 0 else -1
            tokens[b, i] = int(rng.integers(0, vocab))
    uniforms = rng.random((a.B, a.T + 1), dtype=np.float32)
    return dict(target_logits=logits, draft_tokens=tokens, parents=parents,
                n_nodes=np.asarray(a.n_nodes, np.int32), uniforms=uniforms)


def expand_logits(rng, F, vocab, std, normalised=True):
    """F rows of draft logits: N(0, std^2), optionally shifted per row so that the
    row is a log-probability vector (what a draft head hands over after its
    log-softmax).  The shift is input preparation done in fp64 with a library
    routine; the expansion itself never relies on it."""
    x = rng.standard_normal((F, vocab)) * std
    if normalised:
        from scipy.special import log_softmax
        x = log_softmax(x, axis=-1)
    return np.ascontiguousarray(x, dtype=np.float32)


# ------------------------------------------------- prediction-model inputs

POLICY_K = 10        # inputs: the k frontier confidences (Sec. 5.1: k = 10)
POLICY_H = 128       # LSTM hidden size (App. A.3)
POLICY_M = 128       # hidden size of the perceptron head (App. A.3)


def policy_params(rng, k=POLICY_K, H=POLICY_H, M=POLICY_M, gain=1.0):
    """Random parameters of the prediction model's shape (no trained weights
    exist here): every tensor uniform in +-gain/sqrt(fan_in), float32, in the
    row-stacked layout the library documents (gate blocks i, f, g, o)."""
    def u(shape, fan_in):
        b = gain / np.sqrt(fan_in)
        return np.ascontiguousarray(rng.uniform(-b, b, size=shape), dtype=np.float32)
    return dict(w_ih=u((4 * H, k), H), w_hh=u((4 * H, H), H), b_ih=u((4 * H,), H), b_hh=u((4 * H,), H),
                w1=u((M, H + k), H + k), b1=u((M,), H + k), w2=u((2, M), M), b2=u((2,), M))


def policy_conf(rng, B, k=POLICY_K, steps=1):
    """Confidence vectors as the expansion emits them: k values in (0, 1],
    sorted descending, shrinking from draft step to draft step (a path's
    probability only falls as it grows).  float32 [steps, B, k]."""
    c = np.sort(rng.random((steps, B, k)) ** 2.0, axis=-1)[..., ::-1]
    decay = np.cumprod(rng.uniform(0.5, 1.0, size=(steps, B, 1)), axis=0)
    return np.ascontiguousarray(c * decay, dtype=np.float32)


# ------------------------------------------- sampled drafts (general-q verify)

def sampled_draft_inputs(rng, parents_list, vocab, T, std=2.0, noise=1.0, shared_rows=True):
    """Inputs for verification with draft distributions (Sec. 3, Eq. 1-2): a batch of trees whose
    tokens were DRAWN from draft distributions.  Target rows are N(0, std) logits; the draft
    distribution under a node is the target row of that node plus N(0, noise) (a draft model that
    tracks the target loosely).  shared_rows: the children of a node share one draft row (they
    are i.i.d. draws from it; q_rows maps each child to its parent's row), else every child has
    a row of its own.  Token draws use scipy's softmax and numpy's choice: input preparation,
    the draft stage itself is outside the path.

    parents_list: one int32 parent array per sequence (length <= T).
    Returns dict(target_logits [B,T,V], draft_logits [B,T,V], q_rows [B,T], draft_tokens [B,T],
    parents [B,T], n_nodes [B], uniforms [B,T+1])."""
    from scipy.special import softmax
    B = len(parents_list)
    tl = normal_logits(rng, (B, T, vocab), std)
    dl = np.zeros((B, T, vocab), np.float32)
    q_rows = np.zeros((B, T), np.int32)
    tokens = np.zeros((B, T), np.int32)
    parents = np.full((B, T), -1, np.int32)
    n_nodes = np.zeros(B, np.int32)
    for b, par in enumerate(parents_list):
        n = len(par)
        n_nodes[b] = n
        parents[b, :n] = par
        tokens[b, 0] = int(rng.integers(0, vocab))
        for c in range(1, n):
            p = int(par[c])
            row = p if shared_rows else c
            q_rows[b, c] = row
            if not dl[b, row].any():
                dl[b, row] = tl[b, p] + normal_logits(rng, (vocab,), noise)
            q = softmax(dl[b, row].astype(np.float64))
            tokens[b, c] = int(rng.choice(vocab, p=q))
    uniforms = rng.random((B, T + 1), dtype=np.float32)
    return dict(target_logits=tl, draft_logits=dl, q_rows=q_rows, draft_tokens=tokens, parents=parents,
                n_nodes=n_nodes, uniforms=uniforms)
