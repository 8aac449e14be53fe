"""ctypes binding of libradar.so: argument marshalling only.

Every function has the name of the C entry point it calls (include/radar.h) and
takes torch tensors that already live on the GPU; it passes their device
pointers, a host descriptor and the current HIP stream.  Nothing is computed
here and there is no fallback: if the library is missing, loading fails.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# RADAR_LIB_SANITIZE=1 selects the build whose host code runs under the sanitizers (CPU tests only)
LIB_PATH = os.path.join(_HERE, "libradar_san.so" if os.environ.get("RADAR_LIB_SANITIZE", "0") == "1" else "libradar.so")
_lib = None

RADAR_OK = 0
RADAR_ACCEPT_GREEDY = 0
RADAR_ACCEPT_SAMPLE = 1
RADAR_T_MAX = 64
RADAR_K_MAX = 16
RADAR_F_MAX = 64
RADAR_POOL_MAX = 4096


class RadarError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__(f"{what}: {status_string(status)} ({status})")


class AttnDesc(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("T_max", ctypes.c_int32), ("Hq", ctypes.c_int32),
                ("Hkv", ctypes.c_int32), ("D", ctypes.c_int32), ("S_max", ctypes.c_int32),
                ("q_stride_b", ctypes.c_int64), ("q_stride_t", ctypes.c_int64), ("q_stride_h", ctypes.c_int64),
                ("kv_stride_b", ctypes.c_int64), ("kv_stride_h", ctypes.c_int64), ("kv_stride_s", ctypes.c_int64),
                ("out_stride_b", ctypes.c_int64), ("out_stride_t", ctypes.c_int64), ("out_stride_h", ctypes.c_int64),
                ("softmax_scale", ctypes.c_float), ("keys_per_split", ctypes.c_int32),
]


class ExpandDesc(ctypes.Structure):
    _fields_ = [("F", ctypes.c_int32), ("V", ctypes.c_int32), ("k", ctypes.c_int32),
                ("pool_count", ctypes.c_int32), ("pool_capacity", ctypes.c_int32)]


class KernelTime(ctypes.Structure):
    _fields_ = [("name", ctypes.c_char * 48), ("calls", ctypes.c_int64), ("total_us", ctypes.c_double),
                ("min_us", ctypes.c_double), ("max_us", ctypes.c_double)]


class AcceptDesc(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("T_max", ctypes.c_int32), ("V", ctypes.c_int32),
                ("D_max", ctypes.c_int32), ("mode", ctypes.c_int32), ("temperature", ctypes.c_float)]


class AcceptQDesc(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("T_max", ctypes.c_int32), ("Tq", ctypes.c_int32), ("V", ctypes.c_int32),
                ("D_max", ctypes.c_int32), ("temperature", ctypes.c_float), ("draft_temperature", ctypes.c_float),
                ("walk_spin_limit", ctypes.c_int32)]


class PolicyParams(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in ("w_ih", "w_hh", "b_ih", "b_hh", "w1", "b1", "w2", "b2")] + \
               [("k", ctypes.c_int32), ("H", ctypes.c_int32), ("M", ctypes.c_int32)]


class PolicyIO(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in ("h_in", "c_in", "uniform", "h_out", "c_out", "logits", "probs", "action")]


EXPORTS = [
    "radar_status_string", "radar_version", "radar_workspace_init",
    "radar_tree_attention_workspace_bytes", "radar_tree_attention",
    "radar_draft_expand_workspace_bytes", "radar_draft_expand", "radar_draft_expand_noalloc", "radar_draft_expand_policy",
    "radar_draft_rerank_workspace_bytes", "radar_draft_rerank",
    "radar_cycle_begin", "radar_draft_expand_cycle", "radar_draft_rerank_cycle",
    "radar_draft_expand_batch_workspace_bytes", "radar_draft_expand_batch", "radar_draft_rerank_batch",
    "radar_verify_accept_workspace_bytes", "radar_verify_accept",
    "radar_accept_length_distribution", "radar_policy_step",
    "radar_verify_accept_q_workspace_bytes", "radar_verify_accept_q",
    "radar_debug_validate_tree", "radar_profile_begin", "radar_profile_end", "radar_probe_hbm_read",
]


def load():
    """Load libradar.so (built by paper_2512_14069_amd.build); raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with __graft_entry__.build() "
                           "(python -m paper_2512_14069_amd.build)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, sz, i32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32
    lib.radar_status_string.restype = ctypes.c_char_p
    lib.radar_status_string.argtypes = [i32]
    lib.radar_version.restype = ctypes.c_int
    lib.radar_workspace_init.restype = i32
    lib.radar_workspace_init.argtypes = [vp, sz, vp]
    lib.radar_tree_attention_workspace_bytes.restype = sz
    lib.radar_tree_attention_workspace_bytes.argtypes = [ctypes.POINTER(AttnDesc)]
    lib.radar_tree_attention.restype = i32
    lib.radar_tree_attention.argtypes = [vp] * 8 + [ctypes.POINTER(AttnDesc), vp, sz, vp]
    lib.radar_draft_expand_workspace_bytes.restype = sz
    lib.radar_draft_expand_workspace_bytes.argtypes = [ctypes.POINTER(ExpandDesc)]
    lib.radar_draft_expand.restype = i32
    lib.radar_draft_expand.argtypes = [vp] * 12 + [ctypes.POINTER(ExpandDesc), vp, sz, vp]
    lib.radar_draft_expand_noalloc.restype = i32
    lib.radar_draft_expand_noalloc.argtypes = [vp] * 12 + [ctypes.POINTER(ExpandDesc), vp]
    lib.radar_draft_expand_policy.restype = i32
    lib.radar_draft_expand_policy.argtypes = [vp] * 12 + [ctypes.POINTER(ExpandDesc), ctypes.POINTER(PolicyParams),
                                              ctypes.POINTER(PolicyIO), vp, sz, vp]
    lib.radar_cycle_begin.restype = i32
    lib.radar_cycle_begin.argtypes = [vp, vp]
    lib.radar_draft_expand_cycle.restype = i32
    lib.radar_draft_expand_cycle.argtypes = [vp] * 12 + [ctypes.POINTER(ExpandDesc), ctypes.POINTER(PolicyParams),
                                             ctypes.POINTER(PolicyIO), vp, vp, sz, vp]
    lib.radar_draft_expand_batch_workspace_bytes.restype = sz
    lib.radar_draft_expand_batch_workspace_bytes.argtypes = [ctypes.POINTER(ExpandDesc), i32]
    lib.radar_draft_expand_batch.restype = i32
    lib.radar_draft_expand_batch.argtypes = [vp] * 12 + [ctypes.POINTER(ExpandDesc), i32, ctypes.POINTER(PolicyParams),
                                             ctypes.POINTER(PolicyIO), vp, vp, sz, vp]
    lib.radar_draft_rerank_batch.restype = i32
    lib.radar_draft_rerank_batch.argtypes = [vp] * 4 + [i32, i32, i32, i32] + [vp] * 7 + [vp, sz, vp]
    lib.radar_draft_rerank_cycle.restype = i32
    lib.radar_draft_rerank_cycle.argtypes = [vp] * 4 + [i32, i32, i32] + [vp] * 6 + [vp, sz, vp]
    lib.radar_draft_rerank_workspace_bytes.restype = sz
    lib.radar_draft_rerank_workspace_bytes.argtypes = [i32, i32]
    lib.radar_draft_rerank.restype = i32
    lib.radar_draft_rerank.argtypes = [vp] * 3 + [i32, i32, i32] + [vp] * 6 + [vp, sz, vp]
    lib.radar_verify_accept_workspace_bytes.restype = sz
    lib.radar_verify_accept_workspace_bytes.argtypes = [ctypes.POINTER(AcceptDesc)]
    lib.radar_verify_accept.restype = i32
    lib.radar_verify_accept.argtypes = [vp] * 8 + [ctypes.POINTER(AcceptDesc), vp, sz, vp]
    lib.radar_accept_length_distribution.restype = i32
    lib.radar_accept_length_distribution.argtypes = [vp] * 5 + [ctypes.POINTER(AcceptDesc), vp, sz, vp]
    lib.radar_verify_accept_q_workspace_bytes.restype = sz
    lib.radar_verify_accept_q_workspace_bytes.argtypes = [ctypes.POINTER(AcceptQDesc)]
    lib.radar_verify_accept_q.restype = i32
    lib.radar_verify_accept_q.argtypes = [vp] * 10 + [ctypes.POINTER(AcceptQDesc), vp, sz, vp]
    lib.radar_policy_step.restype = i32
    lib.radar_policy_step.argtypes = [vp] * 3 + [ctypes.POINTER(PolicyParams)] + [vp] * 6 + [i32, vp]
    lib.radar_debug_validate_tree.restype = i32
    lib.radar_debug_validate_tree.argtypes = [vp, vp, i32, i32, vp, vp]
    lib.radar_probe_hbm_read.restype = i32
    lib.radar_probe_hbm_read.argtypes = [vp, sz, vp, vp]
    lib.radar_profile_begin.restype = i32
    lib.radar_profile_begin.argtypes = [i32]
    lib.radar_profile_end.restype = i32
    lib.radar_profile_end.argtypes = [ctypes.POINTER(KernelTime), i32, ctypes.POINTER(i32)]
    _lib = lib
    return lib


def status_string(status):
    return load().radar_status_string(int(status)).decode()


def radar_version():
    return int(load().radar_version())


def _ptr(t, dtype=None, name="tensor"):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must be a GPU tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name} must be {dtype}, got {t.dtype}")
    return ctypes.c_void_p(t.data_ptr())


def _dense(t, name):
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(rc, what):
    if rc != RADAR_OK:
        raise RadarError(rc, what)


class BoundCall:
    """A library call with its arguments already marshalled: calling it again costs one foreign
    call.  It replays exactly the pointers, sizes and stream it was made with (`keep` holds the
    tensors alive); host-side counters such as DraftPool.count are not advanced by a replay.
    `out` is what the plain wrapper would have returned."""
    __slots__ = ("name", "fn", "args", "keep", "out")

    def __init__(self, name, fn, args, keep, out):
        self.name, self.fn, self.args, self.keep, self.out = name, fn, args, keep, out

    def __call__(self):
        rc = self.fn(*self.args)
        if rc != RADAR_OK:
            raise RadarError(rc, self.name)
        return self.out


def _finish(name, fn, args, keep, out, prepared):
    call = BoundCall(name, fn, args, keep, out)
    return call if prepared else call()


def _ws_args(ws):
    if ws is None:
        return None, 0
    return ctypes.c_void_p(ws.data_ptr()), ws.numel() * ws.element_size()


def new_workspace(nbytes, device="cuda"):
    """Device workspace of at least nbytes, passed through radar_workspace_init."""
    nbytes = max(int(nbytes), 4096)
    ws = torch.empty((nbytes + 255) // 256 * 256, dtype=torch.uint8, device=device)
    radar_workspace_init(ws)
    return ws


def radar_workspace_init(ws):
    p, n = _ws_args(ws)
    _check(load().radar_workspace_init(p, n, _stream()), "radar_workspace_init")


# ------------------------------------------------------------ tree attention

def attn_desc(q, k_cache, keys_per_split=0, softmax_scale=0.0):
    B, T, Hq, D = q.shape
    Bk, Hkv, S, Dk = k_cache.shape
    d = AttnDesc()
    d.B, d.T_max, d.Hq, d.Hkv, d.D, d.S_max = B, T, Hq, Hkv, D, S
    d.q_stride_b, d.q_stride_t, d.q_stride_h = q.stride(0), q.stride(1), q.stride(2)
    d.kv_stride_b, d.kv_stride_h, d.kv_stride_s = k_cache.stride(0), k_cache.stride(1), k_cache.stride(2)
    d.out_stride_b = d.out_stride_t = d.out_stride_h = 0
    d.softmax_scale = float(softmax_scale)
    d.keys_per_split = int(keys_per_split)
    return d


def radar_tree_attention_workspace_bytes(desc):
    return int(load().radar_tree_attention_workspace_bytes(ctypes.byref(desc)))


def radar_tree_attention(q, k_cache, v_cache, parents, ctx_lens, n_nodes=None, out=None, lse_out=None,
                         desc=None, workspace=None, keys_per_split=0, softmax_scale=0.0, prepared=False):
    """q bf16 [B,T,Hq,D]; k_cache, v_cache bf16 [B,Hkv,S,D] (same strides, D contiguous);
    parents i32 [B,T]; ctx_lens i32 [B]; n_nodes i32 [B] or None.  Returns out bf16 [B,T,Hq,D]."""
    if q.stride(-1) != 1 or k_cache.stride(-1) != 1 or v_cache.stride() != k_cache.stride():
        raise ValueError("innermost axis must be contiguous and k/v caches must share strides")
    if desc is None:
        desc = attn_desc(q, k_cache, keys_per_split, softmax_scale)
    if out is None:
        out = torch.empty(q.shape, dtype=torch.bfloat16, device=q.device)
    _dense(out, "out")
    if workspace is None:
        workspace = new_workspace(radar_tree_attention_workspace_bytes(desc), q.device)
    wp, wn = _ws_args(workspace)
    args = (
        _ptr(q, torch.bfloat16, "q"), _ptr(k_cache, torch.bfloat16, "k_cache"),
        _ptr(v_cache, torch.bfloat16, "v_cache"), _ptr(_dense(parents, "parents"), torch.int32, "parents"),
        _ptr(_dense(ctx_lens, "ctx_lens"), torch.int32, "ctx_lens"),
        _ptr(None if n_nodes is None else _dense(n_nodes, "n_nodes"), torch.int32, "n_nodes"),
        _ptr(out, torch.bfloat16, "out"), _ptr(lse_out, torch.float32, "lse_out"),
        ctypes.byref(desc), wp, wn, _stream())
    keep = (q, k_cache, v_cache, parents, ctx_lens, n_nodes, out, lse_out, desc, workspace)
    return _finish("radar_tree_attention", load().radar_tree_attention, args, keep, out, prepared)


# ------------------------------------------------------------ draft expansion

class DraftPool:
    """Caller-owned pool arrays (tokens, scores, parents) and the host-side count; with B, the pools of
    B sequences ([B, capacity] arrays, one count for all)."""

    def __init__(self, capacity, device="cuda", B=None):
        self.capacity = int(capacity)
        shape = (self.capacity,) if B is None else (int(B), self.capacity)
        self.tokens = torch.zeros(shape, dtype=torch.int32, device=device)
        self.scores = torch.zeros(shape, dtype=torch.float32, device=device)
        self.parents = torch.zeros(shape, dtype=torch.int32, device=device)
        self.count = 0


class ExpandOut:
    def __init__(self, F, k, device, B=None):
        lead = () if B is None else (int(B),)
        self.cand_tokens = torch.empty(lead + (F * k,), dtype=torch.int32, device=device)
        self.cand_scores = torch.empty(lead + (F * k,), dtype=torch.float32, device=device)
        self.frontier_pool_idx = torch.empty(lead + (k,), dtype=torch.int32, device=device)
        self.frontier_tokens = torch.empty(lead + (k,), dtype=torch.int32, device=device)
        self.frontier_scores = torch.empty(lead + (k,), dtype=torch.float32, device=device)
        self.frontier_conf = torch.empty(lead + (k,), dtype=torch.float32, device=device)


def expand_desc(F, V, k, pool_count, pool_capacity):
    d = ExpandDesc()
    d.F, d.V, d.k, d.pool_count, d.pool_capacity = F, V, k, pool_count, pool_capacity
    return d


def radar_draft_expand_workspace_bytes(desc):
    return int(load().radar_draft_expand_workspace_bytes(ctypes.byref(desc)))


def radar_draft_expand(logits, parent_scores, parent_pool_idx, k, pool, out=None, workspace=None, prepared=False):
    """logits f32 [F,V]; parent_scores f32 [F]; parent_pool_idx i32 [F]; pool: DraftPool
    (appended to; pool.count advances by F*k).  Returns an ExpandOut."""
    F, V = logits.shape
    desc = expand_desc(F, V, k, pool.count, pool.capacity)
    if out is None:
        out = ExpandOut(F, k, logits.device)
    if workspace is None:
        workspace = new_workspace(radar_draft_expand_workspace_bytes(desc), logits.device)
    wp, wn = _ws_args(workspace)
    args = (
        _ptr(_dense(logits, "logits"), torch.float32, "logits"),
        _ptr(_dense(parent_scores, "parent_scores"), torch.float32, "parent_scores"),
        _ptr(_dense(parent_pool_idx, "parent_pool_idx"), torch.int32, "parent_pool_idx"),
        _ptr(out.cand_tokens, torch.int32), _ptr(out.cand_scores, torch.float32),
        _ptr(out.frontier_pool_idx, torch.int32), _ptr(out.frontier_tokens, torch.int32),
        _ptr(out.frontier_scores, torch.float32), _ptr(out.frontier_conf, torch.float32),
        _ptr(pool.tokens, torch.int32), _ptr(pool.scores, torch.float32), _ptr(pool.parents, torch.int32),
        ctypes.byref(desc), wp, wn, _stream())
    keep = (logits, parent_scores, parent_pool_idx, out, pool, desc, workspace)
    pool.count += F * k
    return _finish("radar_draft_expand", load().radar_draft_expand, args, keep, out, prepared)


RADAR_NOALLOC_SCRATCH_BYTES = 1 << 20


def radar_draft_expand_noalloc(logits, parent_scores, parent_pool_idx, k, pool, out=None, prepared=False):
    """radar_draft_expand without a workspace: the library's own device array serves as scratch
    (shapes whose workspace exceeds RADAR_NOALLOC_SCRATCH_BYTES are refused).  `out` is allocated
    here when not given; the library call itself allocates nothing."""
    F, V = logits.shape
    desc = expand_desc(F, V, k, pool.count, pool.capacity)
    if out is None:
        out = ExpandOut(F, k, logits.device)
    args = (
        _ptr(_dense(logits, "logits"), torch.float32, "logits"),
        _ptr(_dense(parent_scores, "parent_scores"), torch.float32, "parent_scores"),
        _ptr(_dense(parent_pool_idx, "parent_pool_idx"), torch.int32, "parent_pool_idx"),
        _ptr(out.cand_tokens, torch.int32), _ptr(out.cand_scores, torch.float32),
        _ptr(out.frontier_pool_idx, torch.int32), _ptr(out.frontier_tokens, torch.int32),
        _ptr(out.frontier_scores, torch.float32), _ptr(out.frontier_conf, torch.float32),
        _ptr(pool.tokens, torch.int32), _ptr(pool.scores, torch.float32), _ptr(pool.parents, torch.int32),
        ctypes.byref(desc), _stream())
    keep = (logits, parent_scores, parent_pool_idx, out, pool, desc)
    call = _finish("radar_draft_expand_noalloc", load().radar_draft_expand_noalloc, args, keep, out, prepared)
    pool.count += F * k
    return call


def radar_draft_expand_policy(logits, parent_scores, parent_pool_idx, k, pool, params, h=None, c=None, uniform=None,
                              out=None, policy_out=None, workspace=None, prepared=False):
    """radar_draft_expand and, in the same launch, radar_policy_step on its frontier_conf.
    params from policy_params(); h, c f32 [1,H] or None; uniform f32 [1] or None.
    Returns (ExpandOut, PolicyOut)."""
    F, V = logits.shape
    pp, held = params
    desc = expand_desc(F, V, k, pool.count, pool.capacity)
    if out is None:
        out = ExpandOut(F, k, logits.device)
    if policy_out is None:
        policy_out = PolicyOut(1, pp.H, logits.device)
    if (h is None) != (c is None):
        raise ValueError("h and c must be given together")
    for n, t in (("h", h), ("c", c)):
        if t is not None and t.numel() != pp.H:
            raise ValueError(f"{n}: expected {pp.H} elements, got {t.numel()}")
    if workspace is None:
        workspace = new_workspace(radar_draft_expand_workspace_bytes(desc), logits.device)
    io = PolicyIO()
    val = lambda t, dt, n: None if t is None else _ptr(_dense(t, n), dt, n).value
    io.h_in, io.c_in = val(h, torch.float32, "h"), val(c, torch.float32, "c")
    io.uniform = val(uniform, torch.float32, "uniform")
    io.h_out, io.c_out = policy_out.h.data_ptr(), policy_out.c.data_ptr()
    io.logits, io.probs, io.action = policy_out.logits.data_ptr(), policy_out.probs.data_ptr(), policy_out.action.data_ptr()
    wp, wn = _ws_args(workspace)
    args = (
        _ptr(_dense(logits, "logits"), torch.float32, "logits"),
        _ptr(_dense(parent_scores, "parent_scores"), torch.float32, "parent_scores"),
        _ptr(_dense(parent_pool_idx, "parent_pool_idx"), torch.int32, "parent_pool_idx"),
        _ptr(out.cand_tokens, torch.int32), _ptr(out.cand_scores, torch.float32),
        _ptr(out.frontier_pool_idx, torch.int32), _ptr(out.frontier_tokens, torch.int32),
        _ptr(out.frontier_scores, torch.float32), _ptr(out.frontier_conf, torch.float32),
        _ptr(pool.tokens, torch.int32), _ptr(pool.scores, torch.float32), _ptr(pool.parents, torch.int32),
        ctypes.byref(desc), ctypes.byref(pp), ctypes.byref(io), wp, wn, _stream())
    keep = (logits, parent_scores, parent_pool_idx, out, pool, desc, workspace, pp, held, io, h, c, uniform, policy_out)
    pool.count += F * k
    return _finish("radar_draft_expand_policy", load().radar_draft_expand_policy, args, keep, (out, policy_out), prepared)


class TreeOut:
    def __init__(self, N, device, B=None):
        shape = (N + 1,) if B is None else (int(B), N + 1)
        self.tokens = torch.empty(shape, dtype=torch.int32, device=device)
        self.parents = torch.empty(shape, dtype=torch.int32, device=device)
        self.scores = torch.empty(shape, dtype=torch.float32, device=device)
        self.depth = torch.empty(shape, dtype=torch.int32, device=device)
        self.pool_idx = torch.empty(shape, dtype=torch.int32, device=device)
        self.n_nodes = torch.empty(1 if B is None else int(B), dtype=torch.int32, device=device)


def radar_draft_rerank_workspace_bytes(pool_count, N):
    return int(load().radar_draft_rerank_workspace_bytes(int(pool_count), int(N)))


def radar_draft_rerank(pool, N, root_token, out=None, workspace=None, prepared=False):
    """Keep the best N pool entries; returns a TreeOut (device tensors)."""
    if out is None:
        out = TreeOut(N, pool.tokens.device)
    wp, wn = _ws_args(workspace)
    args = (
        _ptr(pool.tokens, torch.int32), _ptr(pool.scores, torch.float32), _ptr(pool.parents, torch.int32),
        int(pool.count), int(N), int(root_token),
        _ptr(out.tokens, torch.int32), _ptr(out.parents, torch.int32), _ptr(out.scores, torch.float32),
        _ptr(out.depth, torch.int32), _ptr(out.pool_idx, torch.int32), _ptr(out.n_nodes, torch.int32),
        wp, wn, _stream())
    return _finish("radar_draft_rerank", load().radar_draft_rerank, args, (pool, out, workspace), out, prepared)


# ------------------------------------------------- cycle with device-side stop

def new_cycle_state(device="cuda"):
    """Device-side state of a drafting cycle: int32 [stopped, pool_count, steps_done, last_action]."""
    return torch.zeros(4, dtype=torch.int32, device=device)


def radar_cycle_begin(state, prepared=False):
    args = (_ptr(state, torch.int32, "state"), _stream())
    return _finish("radar_cycle_begin", load().radar_cycle_begin, args, (state,), state, prepared)


def radar_draft_expand_cycle(logits, parent_scores, parent_pool_idx, k, pool, pool_count_max, state, params=None,
                             h=None, c=None, uniform=None, out=None, policy_out=None, workspace=None, prepared=False):
    """One draft call of a cycle whose stop decision stays on the device.  pool_count_max: the pool count
    had every earlier call of the cycle run (host arithmetic); the actual count lives in `state`.
    params None: no decision after this call.  pool.count is not touched.
    Returns (ExpandOut, PolicyOut or None)."""
    F, V = logits.shape
    desc = expand_desc(F, V, k, int(pool_count_max), pool.capacity)
    if out is None:
        out = ExpandOut(F, k, logits.device)
    if workspace is None:
        workspace = new_workspace(radar_draft_expand_workspace_bytes(desc), logits.device)
    pp = held = io = None
    if params is not None:
        pp, held = params
        if policy_out is None:
            policy_out = PolicyOut(1, pp.H, logits.device)
        if (h is None) != (c is None):
            raise ValueError("h and c must be given together")
        io = PolicyIO()
        val = lambda t, dt, n: None if t is None else _ptr(_dense(t, n), dt, n).value
        io.h_in, io.c_in = val(h, torch.float32, "h"), val(c, torch.float32, "c")
        io.uniform = val(uniform, torch.float32, "uniform")
        io.h_out, io.c_out = policy_out.h.data_ptr(), policy_out.c.data_ptr()
        io.logits, io.probs, io.action = policy_out.logits.data_ptr(), policy_out.probs.data_ptr(), policy_out.action.data_ptr()
    wp, wn = _ws_args(workspace)
    args = (
        _ptr(_dense(logits, "logits"), torch.float32, "logits"),
        _ptr(_dense(parent_scores, "parent_scores"), torch.float32, "parent_scores"),
        _ptr(_dense(parent_pool_idx, "parent_pool_idx"), torch.int32, "parent_pool_idx"),
        _ptr(out.cand_tokens, torch.int32), _ptr(out.cand_scores, torch.float32),
        _ptr(out.frontier_pool_idx, torch.int32), _ptr(out.frontier_tokens, torch.int32),
        _ptr(out.frontier_scores, torch.float32), _ptr(out.frontier_conf, torch.float32),
        _ptr(pool.tokens, torch.int32), _ptr(pool.scores, torch.float32), _ptr(pool.parents, torch.int32),
        ctypes.byref(desc), None if pp is None else ctypes.byref(pp), None if io is None else ctypes.byref(io),
        _ptr(state, torch.int32, "state"), wp, wn, _stream())
    keep = (logits, parent_scores, parent_pool_idx, out, pool, desc, workspace, pp, held, io, h, c, uniform, policy_out, state)
    return _finish("radar_draft_expand_cycle", load().radar_draft_expand_cycle, args, keep, (out, policy_out), prepared)


def radar_draft_expand_batch_workspace_bytes(desc, B):
    return int(load().radar_draft_expand_batch_workspace_bytes(ctypes.byref(desc), int(B)))


def radar_draft_expand_batch(logits, parent_scores, parent_pool_idx, k, pool, states=None, pool_count_max=None, params=None,
                             h=None, c=None, uniform=None, out=None, policy_out=None, workspace=None, prepared=False):
    """One draft call for B sequences in one launch.  logits f32 [B,F,V]; parent_scores f32, parent_pool_idx i32
    [B,F]; pool: DraftPool(capacity, B=B).  states None: every sequence's pool holds pool.count candidates
    (pool.count advances by F*k); states i32 [B,4]: per-sequence cycle states as in radar_draft_expand_cycle
    (pool_count_max required, pool.count untouched).  params None: no decision; otherwise h, c f32 [B,H] or
    None, uniform f32 [B] or None.  Returns (ExpandOut, PolicyOut or None), both with a leading B."""
    B, F, V = logits.shape
    if tuple(pool.tokens.shape) != (B, pool.capacity):
        raise ValueError("pool: expected DraftPool(capacity, B=%d)" % B)
    if states is not None and pool_count_max is None:
        raise ValueError("a call with states needs pool_count_max")
    desc = expand_desc(F, V, k, int(pool.count if states is None else pool_count_max), pool.capacity)
    if out is None:
        out = ExpandOut(F, k, logits.device, B=B)
    if workspace is None:
        workspace = new_workspace(radar_draft_expand_batch_workspace_bytes(desc, B), logits.device)
    pp = held = io = None
    if params is not None:
        pp, held = params
        if policy_out is None:
            policy_out = PolicyOut(B, pp.H, logits.device)
        if (h is None) != (c is None):
            raise ValueError("h and c must be given together")
        for n, t, want in (("h", h, B * pp.H), ("c", c, B * pp.H), ("uniform", uniform, B)):
            if t is not None and t.numel() != want:
                raise ValueError(f"{n}: expected {want} elements, got {t.numel()}")
        io = PolicyIO()
        val = lambda t, dt, n: None if t is None else _ptr(_dense(t, n), dt, n).value
        io.h_in, io.c_in = val(h, torch.float32, "h"), val(c, torch.float32, "c")
        io.uniform = val(uniform, torch.float32, "uniform")
        io.h_out, io.c_out = policy_out.h.data_ptr(), policy_out.c.data_ptr()
        io.logits, io.probs, io.action = policy_out.logits.data_ptr(), policy_out.probs.data_ptr(), policy_out.action.data_ptr()
    if states is not None and states.numel() != 4 * B:
        raise ValueError("states: expected [B, 4] int32")
    wp, wn = _ws_args(workspace)
    args = (
        _ptr(_dense(logits, "logits"), torch.float32, "logits"),
        _ptr(_dense(parent_scores, "parent_scores"), torch.float32, "parent_scores"),
        _ptr(_dense(parent_pool_idx, "parent_pool_idx"), torch.int32, "parent_pool_idx"),
        _ptr(out.cand_tokens, torch.int32), _ptr(out.cand_scores, torch.float32),
        _ptr(out.frontier_pool_idx, torch.int32), _ptr(out.frontier_tokens, torch.int32),
        _ptr(out.frontier_scores, torch.float32), _ptr(out.frontier_conf, torch.float32),
        _ptr(pool.tokens, torch.int32), _ptr(pool.scores, torch.float32), _ptr(pool.parents, torch.int32),
        ctypes.byref(desc), int(B), None if pp is None else ctypes.byref(pp), None if io is None else ctypes.byref(io),
        None if states is None else _ptr(_dense(states, "states"), torch.int32, "states"), wp, wn, _stream())
    keep = (logits, parent_scores, parent_pool_idx, out, pool, desc, workspace, pp, held, io, h, c, uniform, policy_out, states)
    if states is None:
        pool.count += F * k
    return _finish("radar_draft_expand_batch", load().radar_draft_expand_batch, args, keep, (out, policy_out), prepared)


def radar_draft_rerank_cycle(pool, state, pool_count_max, N, root_token, out=None, workspace=None, prepared=False):
    """radar_draft_rerank over the candidates `state` counts (at most pool_count_max)."""
    if out is None:
        out = TreeOut(N, pool.tokens.device)
    wp, wn = _ws_args(workspace)
    args = (
        _ptr(pool.tokens, torch.int32), _ptr(pool.scores, torch.float32), _ptr(pool.parents, torch.int32),
        _ptr(state, torch.int32, "state"), int(pool_count_max), int(N), int(root_token),
        _ptr(out.tokens, torch.int32), _ptr(out.parents, torch.int32), _ptr(out.scores, torch.float32),
        _ptr(out.depth, torch.int32), _ptr(out.pool_idx, torch.int32), _ptr(out.n_nodes, torch.int32),
        wp, wn, _stream())
    return _finish("radar_draft_rerank_cycle", load().radar_draft_rerank_cycle, args, (pool, state, out, workspace), out, prepared)


def radar_draft_rerank_batch(pool, N, root_tokens, states=None, pool_count_max=None, out=None, workspace=None, prepared=False):
    """radar_draft_rerank for the B sequences of a DraftPool(capacity, B=B) in one launch.  root_tokens i32 [B];
    states None: every pool holds pool.count candidates; states i32 [B,4]: each its own state's count (at most
    pool_count_max, default the capacity).  Returns a TreeOut with a leading B (what radar_tree_attention and
    radar_verify_accept take as parents / tokens / n_nodes)."""
    B = pool.tokens.shape[0]
    if pool.tokens.dim() != 2 or root_tokens.numel() != B:
        raise ValueError("expected DraftPool(capacity, B=B) and B root tokens")
    if states is not None and states.numel() != 4 * B:
        raise ValueError("states: expected [B, 4] int32")
    if out is None:
        out = TreeOut(N, pool.tokens.device, B=B)
    count = pool.count if states is None else (pool.capacity if pool_count_max is None else pool_count_max)
    wp, wn = _ws_args(workspace)
    args = (
        _ptr(pool.tokens, torch.int32), _ptr(pool.scores, torch.float32), _ptr(pool.parents, torch.int32),
        None if states is None else _ptr(_dense(states, "states"), torch.int32, "states"),
        int(count), int(pool.capacity), int(B), int(N), _ptr(_dense(root_tokens, "root_tokens"), torch.int32, "root_tokens"),
        _ptr(out.tokens, torch.int32), _ptr(out.parents, torch.int32), _ptr(out.scores, torch.float32),
        _ptr(out.depth, torch.int32), _ptr(out.pool_idx, torch.int32), _ptr(out.n_nodes, torch.int32),
        wp, wn, _stream())
    return _finish("radar_draft_rerank_batch", load().radar_draft_rerank_batch, args, (pool, states, root_tokens, out, workspace),
                   out, prepared)


# ------------------------------------------------------------ verification

def accept_desc(B, T, V, D_max, mode, temperature):
    d = AcceptDesc()
    d.B, d.T_max, d.V, d.D_max, d.mode, d.temperature = B, T, V, D_max, mode, temperature
    return d


def radar_verify_accept_workspace_bytes(desc):
    return int(load().radar_verify_accept_workspace_bytes(ctypes.byref(desc)))


def radar_verify_accept(target_logits, draft_tokens, parents, n_nodes=None, uniforms=None, mode=RADAR_ACCEPT_GREEDY,
                        temperature=1.0, D_max=None, out=None, workspace=None, prepared=False):
    """target_logits f32 [B,T,V]; draft_tokens, parents i32 [B,T]; n_nodes i32 [B] or None;
    uniforms f32 [B,T+1] (sampling).  Returns (accept_len [B], accept_path [B,D_max+1], bonus_token [B])."""
    B, T, V = target_logits.shape
    if D_max is None:
        D_max = T - 1
    desc = accept_desc(B, T, V, D_max, mode, temperature)
    dev = target_logits.device
    if out is None:
        out = (torch.empty(B, dtype=torch.int32, device=dev),
               torch.empty((B, D_max + 1), dtype=torch.int32, device=dev),
               torch.empty(B, dtype=torch.int32, device=dev))
    if workspace is None:
        workspace = new_workspace(radar_verify_accept_workspace_bytes(desc), dev)
    wp, wn = _ws_args(workspace)
    args = (
        _ptr(_dense(target_logits, "target_logits"), torch.float32, "target_logits"),
        _ptr(_dense(draft_tokens, "draft_tokens"), torch.int32, "draft_tokens"),
        _ptr(_dense(parents, "parents"), torch.int32, "parents"),
        _ptr(None if n_nodes is None else _dense(n_nodes, "n_nodes"), torch.int32, "n_nodes"),
        _ptr(None if uniforms is None else _dense(uniforms, "uniforms"), torch.float32, "uniforms"),
        _ptr(out[0], torch.int32), _ptr(out[1], torch.int32), _ptr(out[2], torch.int32),
        ctypes.byref(desc), wp, wn, _stream())
    keep = (target_logits, draft_tokens, parents, n_nodes, uniforms, out, desc, workspace)
    return _finish("radar_verify_accept", load().radar_verify_accept, args, keep, out, prepared)


def accept_q_desc(B, T, Tq, V, D_max, temperature=1.0, draft_temperature=1.0, walk_spin_limit=0):
    d = AcceptQDesc()
    d.B, d.T_max, d.Tq, d.V, d.D_max, d.temperature, d.draft_temperature = B, T, Tq, V, D_max, temperature, draft_temperature
    d.walk_spin_limit = walk_spin_limit
    return d


def radar_verify_accept_q_workspace_bytes(desc):
    return int(load().radar_verify_accept_q_workspace_bytes(ctypes.byref(desc)))


def radar_verify_accept_q(target_logits, draft_logits, draft_tokens, parents, n_nodes=None, uniforms=None, q_rows=None,
                          temperature=1.0, draft_temperature=1.0, D_max=None, out=None, workspace=None, prepared=False,
                          walk_spin_limit=0):
    """target_logits f32 [B,T,V]; draft_logits f32 [B,Tq,V]; q_rows i32 [B,T] or None (Tq == T);
    draft_tokens, parents i32 [B,T]; n_nodes i32 [B] or None; uniforms f32 [B,T+1].
    Returns (accept_len [B], accept_path [B,D_max+1], bonus_token [B])."""
    B, T, V = target_logits.shape
    Tq = draft_logits.shape[1]
    if tuple(draft_logits.shape) != (B, Tq, V):
        raise ValueError(f"draft_logits: expected shape {(B, Tq, V)}, got {tuple(draft_logits.shape)}")
    if uniforms is None or tuple(uniforms.shape) != (B, T + 1):
        raise ValueError(f"uniforms: expected shape {(B, T + 1)}")
    if D_max is None:
        D_max = T - 1
    desc = accept_q_desc(B, T, Tq, V, D_max, temperature, draft_temperature, walk_spin_limit)
    dev = target_logits.device
    if out is None:
        out = (torch.empty(B, dtype=torch.int32, device=dev),
               torch.empty((B, D_max + 1), dtype=torch.int32, device=dev),
               torch.empty(B, dtype=torch.int32, device=dev))
    if workspace is None:
        workspace = new_workspace(radar_verify_accept_q_workspace_bytes(desc), dev)
    wp, wn = _ws_args(workspace)
    args = (
        _ptr(_dense(target_logits, "target_logits"), torch.float32, "target_logits"),
        _ptr(_dense(draft_logits, "draft_logits"), torch.float32, "draft_logits"),
        _ptr(None if q_rows is None else _dense(q_rows, "q_rows"), torch.int32, "q_rows"),
        _ptr(_dense(draft_tokens, "draft_tokens"), torch.int32, "draft_tokens"),
        _ptr(_dense(parents, "parents"), torch.int32, "parents"),
        _ptr(None if n_nodes is None else _dense(n_nodes, "n_nodes"), torch.int32, "n_nodes"),
        _ptr(_dense(uniforms, "uniforms"), torch.float32, "uniforms"),
        _ptr(out[0], torch.int32), _ptr(out[1], torch.int32), _ptr(out[2], torch.int32),
        ctypes.byref(desc), wp, wn, _stream())
    keep = (target_logits, draft_logits, q_rows, draft_tokens, parents, n_nodes, uniforms, out, desc, workspace)
    return _finish("radar_verify_accept_q", load().radar_verify_accept_q, args, keep, out, prepared)


def radar_accept_length_distribution(target_logits, draft_tokens, parents, n_nodes=None, temperature=1.0, D_max=None,
                                     out=None, workspace=None, prepared=False):
    """target_logits f32 [B,T,V]; draft_tokens, parents i32 [B,T]; n_nodes i32 [B] or None.
    Returns dist f64 [B, D_max+1]: row b is the distribution of the accepted length of tree b."""
    B, T, V = target_logits.shape
    if D_max is None:
        D_max = T - 1
    desc = accept_desc(B, T, V, D_max, RADAR_ACCEPT_SAMPLE, temperature)
    dev = target_logits.device
    if out is None:
        out = torch.empty((B, D_max + 1), dtype=torch.float64, device=dev)
    if workspace is None:
        workspace = new_workspace(radar_verify_accept_workspace_bytes(desc), dev)
    wp, wn = _ws_args(workspace)
    args = (
        _ptr(_dense(target_logits, "target_logits"), torch.float32, "target_logits"),
        _ptr(_dense(draft_tokens, "draft_tokens"), torch.int32, "draft_tokens"),
        _ptr(_dense(parents, "parents"), torch.int32, "parents"),
        _ptr(None if n_nodes is None else _dense(n_nodes, "n_nodes"), torch.int32, "n_nodes"),
        _ptr(_dense(out, "dist"), torch.float64, "dist"),
        ctypes.byref(desc), wp, wn, _stream())
    keep = (target_logits, draft_tokens, parents, n_nodes, out, desc, workspace)
    return _finish("radar_accept_length_distribution", load().radar_accept_length_distribution, args, keep, out, prepared)


class PolicyOut:
    """Outputs of one prediction-model call: h, c f32 [B,H]; logits, probs f32 [B,2]; action i32 [B]."""
    __slots__ = ("h", "c", "logits", "probs", "action")

    def __init__(self, B, H, device):
        self.h = torch.empty((B, H), dtype=torch.float32, device=device)
        self.c = torch.empty((B, H), dtype=torch.float32, device=device)
        self.logits = torch.empty((B, 2), dtype=torch.float32, device=device)
        self.probs = torch.empty((B, 2), dtype=torch.float32, device=device)
        self.action = torch.empty((B,), dtype=torch.int32, device=device)


def policy_params(tensors):
    """Parameter block from a dict of GPU float32 tensors w_ih [4H,k], w_hh [4H,H], b_ih, b_hh [4H],
    w1 [M,H+k], b1 [M], w2 [2,M], b2 [2].  Returns (struct, tensors kept alive)."""
    w_hh = tensors["w_hh"]
    H = w_hh.shape[1]
    k = tensors["w_ih"].shape[1]
    M = tensors["w1"].shape[0]
    want = {"w_ih": (4 * H, k), "w_hh": (4 * H, H), "b_ih": (4 * H,), "b_hh": (4 * H,),
            "w1": (M, H + k), "b1": (M,), "w2": (2, M), "b2": (2,)}
    pp = PolicyParams()
    for n, shape in want.items():
        t = tensors[n]
        if tuple(t.shape) != shape:
            raise ValueError(f"{n}: expected shape {shape}, got {tuple(t.shape)}")
        setattr(pp, n, _ptr(_dense(t, n), torch.float32, n).value)
    pp.k, pp.H, pp.M = k, H, M
    return pp, dict(tensors)


def radar_policy_step(conf, params, h=None, c=None, uniforms=None, out=None, prepared=False):
    """conf f32 [B,k] (or [k]); params from policy_params(); h, c f32 [B,H] or None (zero state);
    uniforms f32 [B] or None (argmax action).  Returns a PolicyOut."""
    pp, held = params
    if conf.dim() == 1:
        conf = conf[None]
    B, k = conf.shape
    if k != pp.k:
        raise ValueError(f"conf has {k} columns, the parameters expect {pp.k}")
    if (h is None) != (c is None):
        raise ValueError("h and c must be given together")
    if out is None:
        out = PolicyOut(B, pp.H, conf.device)
    for n, t in (("h", h), ("c", c)):
        if t is not None and tuple(t.shape) != (B, pp.H):
            raise ValueError(f"{n}: expected shape {(B, pp.H)}, got {tuple(t.shape)}")
    if uniforms is not None and tuple(uniforms.shape) != (B,):
        raise ValueError(f"uniforms: expected shape {(B,)}")
    args = (
        _ptr(_dense(conf, "conf"), torch.float32, "conf"),
        _ptr(None if h is None else _dense(h, "h"), torch.float32, "h"),
        _ptr(None if c is None else _dense(c, "c"), torch.float32, "c"),
        ctypes.byref(pp),
        _ptr(None if uniforms is None else _dense(uniforms, "uniforms"), torch.float32, "uniforms"),
        _ptr(out.h, torch.float32), _ptr(out.c, torch.float32), _ptr(out.logits, torch.float32),
        _ptr(out.probs, torch.float32), _ptr(out.action, torch.int32), B, _stream())
    keep = (conf, h, c, uniforms, pp, held, out)
    return _finish("radar_policy_step", load().radar_policy_step, args, keep, out, prepared)


def radar_debug_validate_tree(parents, n_nodes=None):
    B, T = parents.shape
    bad = torch.zeros(1, dtype=torch.int32, device=parents.device)
    rc = load().radar_debug_validate_tree(
        _ptr(_dense(parents, "parents"), torch.int32), _ptr(n_nodes, torch.int32), B, T, _ptr(bad), _stream())
    _check(rc, "radar_debug_validate_tree")
    return bad


def radar_probe_hbm_read(buf, nbytes=None, offset=0, prepared=False):
    """One streaming read of nbytes of the uint8 device tensor `buf`, starting at byte `offset`."""
    nbytes = buf.numel() * buf.element_size() - offset if nbytes is None else int(nbytes)
    if offset % 16 or offset + nbytes > buf.numel() * buf.element_size():
        raise ValueError("offset / size outside the buffer or not 16-byte aligned")
    args = (ctypes.c_void_p(buf.data_ptr() + offset), ctypes.c_size_t(nbytes), None, _stream())
    return _finish("radar_probe_hbm_read", load().radar_probe_hbm_read, args, (buf,), None, prepared)


def radar_profile_begin(max_launches):
    _check(load().radar_profile_begin(int(max_launches)), "radar_profile_begin")


def radar_profile_end(capacity=32):
    """Returns {kernel name: dict(calls, total_us, mean_us, min_us, max_us)} for the launches since begin."""
    arr = (KernelTime * capacity)()
    n = ctypes.c_int32(0)
    _check(load().radar_profile_end(arr, capacity, ctypes.byref(n)), "radar_profile_end")
    return {arr[i].name.decode(): dict(calls=int(arr[i].calls), total_us=arr[i].total_us,
                                       mean_us=arr[i].total_us / max(1, arr[i].calls),
                                       min_us=arr[i].min_us, max_us=arr[i].max_us) for i in range(n.value)}
