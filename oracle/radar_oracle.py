"""ctypes wrapper around radar_oracle.c (host only; test infrastructure).

Every function takes numpy arrays, checks shapes and dtypes, and calls the C
routine of the same name.  bf16 tensors travel as uint16 bit patterns.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "radar_oracle.c")
_LIB = os.path.join(_HERE, "libradar_oracle.so")
_lib = None


class OracleError(RuntimeError):
    pass


_SAN_LIB = os.path.join(_HERE, "libradar_oracle_san.so")
# RADAR_ORACLE_SANITIZE=1 in the environment makes this module load the sanitized build (the
# process must then have gcc's libasan preloaded; tests/test_sanitizers.py does that in a child).
_SANITIZE = os.environ.get("RADAR_ORACLE_SANITIZE", "0") == "1"


def build(force=False, sanitize=None):
    """Compile radar_oracle.c with gcc into oracle/libradar_oracle.so, or, with sanitize=True, into
    oracle/libradar_oracle_san.so under AddressSanitizer and UndefinedBehaviorSanitizer."""
    sanitize = _SANITIZE if sanitize is None else sanitize
    lib = _SAN_LIB if sanitize else _LIB
    if (not force and os.path.exists(lib)
            and os.path.getmtime(lib) >= os.path.getmtime(_SRC)):
        return lib
    opt = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
           "-fno-omit-frame-pointer"] if sanitize else ["-O2"]
    cmd = ["gcc"] + opt + ["-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra", "-o", lib, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return lib


def sanitizer_runtime():
    """Path of gcc's address-sanitizer runtime, to preload into a process that loads the sanitized build."""
    return subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.radar_oracle_round_bf16.restype = ctypes.c_uint16
        _lib.radar_oracle_round_bf16.argtypes = [ctypes.c_double]
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _arr(a, dtype, shape=None, name="array"):
    a = np.ascontiguousarray(a, dtype=dtype)
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise OracleError(f"{name}: expected shape {tuple(shape)}, got {tuple(a.shape)}")
    return a


def _check(rc, what):
    if rc != 0:
        raise OracleError(f"{what} failed with status {rc}")


def num_threads():
    return int(_load().radar_oracle_num_threads())


def set_threads(n):
    _load().radar_oracle_set_threads(ctypes.c_int(int(n)))


def round_bf16(x):
    """fp64 -> bf16 bit pattern (round to nearest even)."""
    return int(_load().radar_oracle_round_bf16(ctypes.c_double(float(x))))


def tree_attention(q, k_cache, v_cache, parents, ctx_lens, n_nodes=None, scale=None, want_lse=False):
    """q uint16[B,T,Hq,D]; k_cache, v_cache uint16[B,Hkv,S,D]; parents int32[B,T];
    ctx_lens int32[B]; n_nodes int32[B] or None.  Returns out uint16[B,T,Hq,D]
    (and lse float32[B,T,Hq] when want_lse)."""
    q = _arr(q, np.uint16, name="q")
    B, T, Hq, D = q.shape
    k_cache = _arr(k_cache, np.uint16, name="k_cache")
    _, Hkv, S, _ = k_cache.shape
    v_cache = _arr(v_cache, np.uint16, (B, Hkv, S, D), "v_cache")
    k_cache = _arr(k_cache, np.uint16, (B, Hkv, S, D), "k_cache")
    parents = _arr(parents, np.int32, (B, T), "parents")
    ctx_lens = _arr(ctx_lens, np.int32, (B,), "ctx_lens")
    nn = None if n_nodes is None else _arr(n_nodes, np.int32, (B,), "n_nodes")
    if scale is None:
        scale = 1.0 / np.sqrt(D)
    out = np.zeros((B, T, Hq, D), np.uint16)
    lse = np.zeros((B, T, Hq), np.float32) if want_lse else None
    rc = _load().radar_oracle_tree_attention(
        _p(q), _p(k_cache), _p(v_cache), _p(parents), _p(ctx_lens), _p(nn), _p(out), _p(lse),
        ctypes.c_int(B), ctypes.c_int(T), ctypes.c_int(Hq), ctypes.c_int(Hkv), ctypes.c_int(D),
        ctypes.c_int(S), ctypes.c_float(scale))
    _check(rc, "radar_oracle_tree_attention")
    return (out, lse) if want_lse else out


def draft_expand(logits, parent_scores, parent_pool_idx, k, pool, pool_count):
    """One expansion step.  ``pool`` is a dict of numpy arrays {tokens int32[cap],
    scores float32[cap], parents int32[cap]} that is appended to in place at
    pool_count.  Returns a dict with cand_tokens[F,k], cand_scores[F,k],
    frontier_pool_idx[k], frontier_tokens[k], frontier_scores[k], frontier_conf[k]."""
    logits = _arr(logits, np.float32, name="logits")
    F, V = logits.shape
    parent_scores = _arr(parent_scores, np.float32, (F,), "parent_scores")
    parent_pool_idx = _arr(parent_pool_idx, np.int32, (F,), "parent_pool_idx")
    cap = pool["tokens"].shape[0]
    for key, dt in (("tokens", np.int32), ("scores", np.float32), ("parents", np.int32)):
        a = pool[key]
        if a.dtype != dt or not a.flags["C_CONTIGUOUS"] or a.shape != (cap,):
            raise OracleError(f"pool[{key}] must be contiguous {dt} of shape ({cap},)")
    res = dict(
        cand_tokens=np.zeros((F, k), np.int32), cand_scores=np.zeros((F, k), np.float32),
        frontier_pool_idx=np.zeros(k, np.int32), frontier_tokens=np.zeros(k, np.int32),
        frontier_scores=np.zeros(k, np.float32), frontier_conf=np.zeros(k, np.float32))
    rc = _load().radar_oracle_draft_expand(
        _p(logits), _p(parent_scores), _p(parent_pool_idx),
        ctypes.c_int(F), ctypes.c_int(V), ctypes.c_int(k), ctypes.c_int(pool_count), ctypes.c_int(cap),
        _p(res["cand_tokens"]), _p(res["cand_scores"]), _p(res["frontier_pool_idx"]),
        _p(res["frontier_tokens"]), _p(res["frontier_scores"]), _p(res["frontier_conf"]),
        _p(pool["tokens"]), _p(pool["scores"]), _p(pool["parents"]))
    _check(rc, "radar_oracle_draft_expand")
    return res


def draft_rerank(pool, pool_count, N, root_token):
    """Keep the best N pool entries; returns dict tokens/parents/scores/depth/pool_idx
    (each N+1 long) and n_nodes."""
    res = dict(tokens=np.zeros(N + 1, np.int32), parents=np.zeros(N + 1, np.int32),
               scores=np.zeros(N + 1, np.float32), depth=np.zeros(N + 1, np.int32),
               pool_idx=np.zeros(N + 1, np.int32))
    n_out = ctypes.c_int32(0)
    rc = _load().radar_oracle_draft_rerank(
        _p(pool["tokens"]), _p(pool["scores"]), _p(pool["parents"]),
        ctypes.c_int(pool_count), ctypes.c_int(N), ctypes.c_int32(root_token),
        _p(res["tokens"]), _p(res["parents"]), _p(res["scores"]), _p(res["depth"]), _p(res["pool_idx"]),
        ctypes.byref(n_out))
    _check(rc, "radar_oracle_draft_rerank")
    res["n_nodes"] = int(n_out.value)
    return res


def verify_accept(target_logits, draft_tokens, parents, n_nodes=None, uniforms=None,
                  mode=0, temperature=1.0, D_max=None):
    """target_logits float32[B,T,V]; draft_tokens, parents int32[B,T];
    uniforms float32[B,T+1] for mode 1.  Returns (accept_len[B], path[B,D_max+1], bonus[B])."""
    target_logits = _arr(target_logits, np.float32, name="target_logits")
    B, T, V = target_logits.shape
    draft_tokens = _arr(draft_tokens, np.int32, (B, T), "draft_tokens")
    parents = _arr(parents, np.int32, (B, T), "parents")
    nn = None if n_nodes is None else _arr(n_nodes, np.int32, (B,), "n_nodes")
    un = None if uniforms is None else _arr(uniforms, np.float32, (B, T + 1), "uniforms")
    if D_max is None:
        D_max = T - 1
    accept_len = np.zeros(B, np.int32)
    path = np.zeros((B, D_max + 1), np.int32)
    bonus = np.zeros(B, np.int32)
    rc = _load().radar_oracle_verify_accept(
        _p(target_logits), _p(draft_tokens), _p(parents), _p(nn), _p(un),
        ctypes.c_int(B), ctypes.c_int(T), ctypes.c_int(V), ctypes.c_int(D_max), ctypes.c_int(mode),
        ctypes.c_float(temperature), _p(accept_len), _p(path), _p(bonus))
    _check(rc, "radar_oracle_verify_accept")
    return accept_len, path, bonus


def accept_length_distribution(target_logits, draft_tokens, parents, n_nodes=None, temperature=1.0, D_max=None):
    """Sec. 4.3, Eq. 11-13: float64[B, D_max+1], row b = distribution of the accepted length of tree b."""
    target_logits = _arr(target_logits, np.float32, name="target_logits")
    B, T, V = target_logits.shape
    draft_tokens = _arr(draft_tokens, np.int32, (B, T), "draft_tokens")
    parents = _arr(parents, np.int32, (B, T), "parents")
    nn = None if n_nodes is None else _arr(n_nodes, np.int32, (B,), "n_nodes")
    if D_max is None:
        D_max = T - 1
    dist = np.zeros((B, D_max + 1), np.float64)
    rc = _load().radar_oracle_accept_length_distribution(
        _p(target_logits), _p(draft_tokens), _p(parents), _p(nn),
        ctypes.c_int(B), ctypes.c_int(T), ctypes.c_int(V), ctypes.c_int(D_max), ctypes.c_float(temperature), _p(dist))
    _check(rc, "radar_oracle_accept_length_distribution")
    return dist


def verify_accept_q(target_logits, draft_logits, draft_tokens, parents, n_nodes=None, uniforms=None, q_rows=None,
                    temperature=1.0, draft_temperature=1.0, D_max=None, want_margins=False):
    """Sec. 3, Eq. 1-2 with draft distributions.  target_logits float32[B,T,V]; draft_logits
    float32[B,Tq,V]; q_rows int32[B,T] or None (Tq == T); uniforms float32[B,T+1].
    Returns (accept_len[B], accept_path[B,D_max+1], bonus_token[B]) and, with want_margins,
    margins float64[B,2]."""
    target_logits = _arr(target_logits, np.float32, name="target_logits")
    B, T, V = target_logits.shape
    draft_logits = _arr(draft_logits, np.float32, name="draft_logits")
    Tq = draft_logits.shape[1]
    draft_logits = _arr(draft_logits, np.float32, (B, Tq, V), "draft_logits")
    draft_tokens = _arr(draft_tokens, np.int32, (B, T), "draft_tokens")
    parents = _arr(parents, np.int32, (B, T), "parents")
    nn = None if n_nodes is None else _arr(n_nodes, np.int32, (B,), "n_nodes")
    qr = None if q_rows is None else _arr(q_rows, np.int32, (B, T), "q_rows")
    un = _arr(uniforms, np.float32, (B, T + 1), "uniforms")
    if D_max is None:
        D_max = T - 1
    accept_len = np.zeros(B, np.int32)
    path = np.zeros((B, D_max + 1), np.int32)
    bonus = np.zeros(B, np.int32)
    m = np.zeros((B, 2), np.float64) if want_margins else None
    rc = _load().radar_oracle_verify_accept_q(
        _p(target_logits), _p(draft_logits), _p(qr), _p(draft_tokens), _p(parents), _p(nn), _p(un),
        ctypes.c_int(B), ctypes.c_int(T), ctypes.c_int(Tq), ctypes.c_int(V), ctypes.c_int(D_max),
        ctypes.c_float(temperature), ctypes.c_float(draft_temperature),
        _p(accept_len), _p(path), _p(bonus), _p(m))
    _check(rc, "radar_oracle_verify_accept_q")
    return (accept_len, path, bonus, m) if want_margins else (accept_len, path, bonus)


def policy_step(conf, params, h=None, c=None, uniforms=None):
    """One prediction-model call (Sec. 4.2, App. A.3).  conf float32[B,k]; params a
    dict of float32 arrays w_ih[4H,k], w_hh[4H,H], b_ih[4H], b_hh[4H], w1[M,H+k],
    b1[M], w2[2,M], b2[2]; h, c float32[B,H] or None (zero state); uniforms
    float32[B] or None (argmax action).  Returns a dict of h, c float64[B,H],
    logits, probs float64[B,2], action int32[B]."""
    conf = _arr(conf, np.float32, name="conf")
    B, k = conf.shape
    w_hh = _arr(params["w_hh"], np.float32, name="w_hh")
    H = w_hh.shape[1]
    w_hh = _arr(w_hh, np.float32, (4 * H, H), "w_hh")
    w_ih = _arr(params["w_ih"], np.float32, (4 * H, k), "w_ih")
    b_ih = _arr(params["b_ih"], np.float32, (4 * H,), "b_ih")
    b_hh = _arr(params["b_hh"], np.float32, (4 * H,), "b_hh")
    w1 = _arr(params["w1"], np.float32, name="w1")
    M = w1.shape[0]
    w1 = _arr(w1, np.float32, (M, H + k), "w1")
    b1 = _arr(params["b1"], np.float32, (M,), "b1")
    w2 = _arr(params["w2"], np.float32, (2, M), "w2")
    b2 = _arr(params["b2"], np.float32, (2,), "b2")
    hh = None if h is None else _arr(h, np.float32, (B, H), "h")
    cc = None if c is None else _arr(c, np.float32, (B, H), "c")
    un = None if uniforms is None else _arr(uniforms, np.float32, (B,), "uniforms")
    out = {"h": np.zeros((B, H)), "c": np.zeros((B, H)), "logits": np.zeros((B, 2)),
           "probs": np.zeros((B, 2)), "action": np.zeros(B, np.int32)}
    rc = _load().radar_oracle_policy_step(
        _p(conf), _p(hh), _p(cc), _p(w_ih), _p(w_hh), _p(b_ih), _p(b_hh), _p(w1), _p(b1), _p(w2), _p(b2), _p(un),
        ctypes.c_int(B), ctypes.c_int(k), ctypes.c_int(H), ctypes.c_int(M),
        _p(out["h"]), _p(out["c"]), _p(out["logits"]), _p(out["probs"]), _p(out["action"]))
    _check(rc, "radar_oracle_policy_step")
    return out


def accept_margins(target_logits, draft_tokens, parents, n_nodes, uniforms, temperature=1.0):
    """Distance of every sampling decision from its threshold: float64[B,2]
    (accept tests, residual inverse-CDF)."""
    target_logits = _arr(target_logits, np.float32, name="target_logits")
    B, T, V = target_logits.shape
    draft_tokens = _arr(draft_tokens, np.int32, (B, T), "draft_tokens")
    parents = _arr(parents, np.int32, (B, T), "parents")
    nn = None if n_nodes is None else _arr(n_nodes, np.int32, (B,), "n_nodes")
    un = _arr(uniforms, np.float32, (B, T + 1), "uniforms")
    m = np.zeros((B, 2), np.float64)
    rc = _load().radar_oracle_accept_margins(
        _p(target_logits), _p(draft_tokens), _p(parents), _p(nn), _p(un),
        ctypes.c_int(B), ctypes.c_int(T), ctypes.c_int(V), ctypes.c_float(temperature), _p(m))
    _check(rc, "radar_oracle_accept_margins")
    return m
