// Draft-tree expansion and rerank for RADAR's drafting loop (App. A.1, Sec. 2.3,
// Sec. 4.2 Eq. 3), as single-launch HIP kernels for gfx950.
//
// radar_draft_expand: grid (chunks of 4096 logits, frontier rows).  Every
// workgroup streams its chunk once from HBM with 16-byte loads (the whole
// step is one read of F*V*4 bytes), keeps its 16 values per lane in registers,
// and leaves (chunk top-k keys, chunk max, chunk sum of exp) in the workspace.
// The workgroup whose arrival ticket is the last of its row merges that row
// (top-k of the chunk lists, log-sum-exp in fp64, cumulative scores, pool
// append); the workgroup that finishes the last row picks the next frontier.
// There is no second launch and no host round trip.
#include "radar_topk.h"
#include "radar_host.h"

namespace radar {

constexpr int kExpThreads = 256;
constexpr int kExpEPT = 16;
constexpr int kExpChunk = kExpThreads * kExpEPT;      // 4096 logits per workgroup
constexpr int kExpMaxChunks = 256;                    // V <= 1,048,576
constexpr int kCounterStride = 32;                    // arrival counters sit 128 B apart: fetch-adds on one
                                                      // cache line serialise at roughly 10 ns each
constexpr size_t kCounterBytes = 16384;               // leading counter block of the workspace
constexpr float kLog2eF = 1.4426950408889634f;

struct ExpandArgs {
    const float *logits;
    const float *parent_scores;
    const int32_t *parent_pool_idx;
    int32_t *cand_tokens;
    float *cand_scores;
    int32_t *frontier_pool_idx;
    int32_t *frontier_tokens;
    float *frontier_scores;
    float *frontier_conf;
    int32_t *pool_tokens;
    float *pool_scores;
    int32_t *pool_parents;
    int F, V, k, nchunks, pool_count;
    unsigned int *counters;     // [0] rows finished, [(1+f) * kCounterStride] chunks of row f finished
    uint64_t *part_keys;        // [F][nchunks][RADAR_K_MAX]
    double *part_l;             // [F][nchunks] sum of exp(x - part_m) over the chunk
    float *part_m;              // [F][nchunks] chunk maximum
};

struct ExpandSmem {
    TopkSmem topk;
    float wave_m[4];
    double wave_l[4];
    int tok[RADAR_F_MAX * RADAR_K_MAX];
    unsigned int ticket;
};

// sum over the four wavefront entries of l_i * exp(m_i - m): lanes 0..3 of a wavefront take one
// term each (fp64 exp), the terms are then added in a fixed order.  Every lane gets the result.
__device__ __forceinline__ double combine4(const float *wm, const double *wl, float m) {
    const int lane = lane_id();
    double t = 0.0;
    if (lane < 4 && wm[lane] > -INFINITY) t = wl[lane] * exp((double)wm[lane] - (double)m);
    const uint64_t b = (uint64_t)__double_as_longlong(t);
    const double t0 = __longlong_as_double((long long)readlane_u64(b, 0));
    const double t1 = __longlong_as_double((long long)readlane_u64(b, 1));
    const double t2 = __longlong_as_double((long long)readlane_u64(b, 2));
    const double t3 = __longlong_as_double((long long)readlane_u64(b, 3));
    return (t0 + t1) + (t2 + t3);
}

template <bool VEC4>
__global__ __launch_bounds__(kExpThreads, 4) void expand_kernel(ExpandArgs a) {
    __shared__ ExpandSmem s;
    const int tid = threadIdx.x, lane = lane_id(), w = wave_id();
    const int f = blockIdx.y, chunk = blockIdx.x;
    const float *row = a.logits + (size_t)f * a.V;
    const int base = chunk * kExpChunk;

    // ---- stream the chunk: 4 x (256 lanes x 16 B), coalesced
    float x[kExpEPT];
    uint64_t keys[kExpEPT];
#pragma unroll
    for (int g = 0; g < kExpEPT / 4; ++g) {
        const int idx0 = base + g * (kExpThreads * 4) + tid * 4;
        // branch-free: out-of-range lanes read a valid address and are masked afterwards
        float4 v;
        if (VEC4) {
            v = *reinterpret_cast<const float4 *>(row + (idx0 < a.V ? idx0 : 0));
        } else {
            v.x = row[min(idx0 + 0, a.V - 1)];
            v.y = row[min(idx0 + 1, a.V - 1)];
            v.z = row[min(idx0 + 2, a.V - 1)];
            v.w = row[min(idx0 + 3, a.V - 1)];
        }
        if (idx0 + 0 >= a.V) v.x = -INFINITY;
        if (idx0 + 1 >= a.V) v.y = -INFINITY;
        if (idx0 + 2 >= a.V) v.z = -INFINITY;
        if (idx0 + 3 >= a.V) v.w = -INFINITY;
        x[4 * g + 0] = v.x; x[4 * g + 1] = v.y; x[4 * g + 2] = v.z; x[4 * g + 3] = v.w;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            keys[4 * g + j] = (idx0 + j < a.V) ? make_key(x[4 * g + j], uint32_t(idx0 + j)) : 0;
    }

    // ---- chunk log-sum-exp partial per wavefront (exp2 of fp32 differences, sums in fp64)
    float tm = x[0];
#pragma unroll
    for (int e = 1; e < kExpEPT; ++e) tm = fmaxf(tm, x[e]);
    const float wm = wave_max_f32(tm);
    double tl = 0.0;
    if (wm > -INFINITY) {
#pragma unroll
        for (int e = 0; e < kExpEPT; ++e) tl += (double)__builtin_amdgcn_exp2f((x[e] - wm) * kLog2eF);
    }
    const double wl = wave_sum_f64(tl);
    if (lane == 0) { s.wave_m[w] = wm; s.wave_l[w] = wl; }

    // ---- chunk top-k
    block_topk<kExpEPT>(keys, a.k, s.topk);          // synchronises; wave_m / wave_l visible after it

    const size_t pslot = (size_t)f * a.nchunks + chunk;
    if (tid < a.k) store_shared_result(&a.part_keys[pslot * RADAR_K_MAX + tid], s.topk.top[tid]);
    if (w == 1) {                                     // a wavefront that stores no keys
        const float m = fmaxf(fmaxf(s.wave_m[0], s.wave_m[1]), fmaxf(s.wave_m[2], s.wave_m[3]));
        const double l = combine4(s.wave_m, s.wave_l, m);
        if (lane == 0) {
            store_shared_result(&a.part_m[pslot], m);
            store_shared_result(&a.part_l[pslot], l);
        }
    }
    if (publish_then_ticket(&a.counters[(1 + f) * kCounterStride], &s.ticket) != (unsigned int)(a.nchunks - 1)) return;

    // ================= last workgroup of row f: merge the row
    // all loads of the hand-over data are issued together (one round trip)
    const int nk = a.nchunks * a.k;
    uint64_t mk[kExpEPT];
#pragma unroll
    for (int e = 0; e < kExpEPT; ++e) {
        const int i = tid + e * kExpThreads;
        const int ic = min(i, nk - 1);                            // branch-free: clamp, load, mask
        const int c = ic / a.k, r = ic - c * a.k;
        const uint64_t key = load_shared_result(&a.part_keys[((size_t)f * a.nchunks + c) * RADAR_K_MAX + r]);
        mk[e] = (i < nk) ? key : 0;
    }
    const int cc = min(tid, a.nchunks - 1);                       // nchunks <= 256: one chunk per lane
    float cm = load_shared_result(&a.part_m[(size_t)f * a.nchunks + cc]);
    const double cl = load_shared_result(&a.part_l[(size_t)f * a.nchunks + cc]);
    if (tid >= a.nchunks) cm = -INFINITY;
    const float pscore = a.parent_scores[f];
    const int ppool = a.parent_pool_idx[f];
    const float rm = wave_max_f32(cm);
    if (lane == 0) s.wave_m[w] = rm;

    block_topk<kExpEPT>(mk, a.k, s.topk);                         // synchronises

    // row log-sum-exp in fp64 from the chunk partials (fixed association order)
    const float M = fmaxf(fmaxf(s.wave_m[0], s.wave_m[1]), fmaxf(s.wave_m[2], s.wave_m[3]));
    const double term = (cm > -INFINITY) ? cl * exp((double)cm - (double)M) : 0.0;
    const double wsum = wave_sum_f64(term);
    if (lane == 0) s.wave_l[w] = wsum;
    __syncthreads();
    if (tid < a.k) {
        const double L = (s.wave_l[0] + s.wave_l[1]) + (s.wave_l[2] + s.wave_l[3]);
        const double lse = (double)M + log(L);
        const uint64_t key = s.topk.top[tid];
        const int tok = (int)key_index(key);
        const double logp = (double)key_value(key) - lse;
        const float cum = (float)((double)pscore + logp);
        const int c = f * a.k + tid;
        store_shared_result(&a.cand_tokens[c], tok);
        store_shared_result(&a.cand_scores[c], cum);
        a.pool_tokens[a.pool_count + c] = tok;
        a.pool_scores[a.pool_count + c] = cum;
        a.pool_parents[a.pool_count + c] = ppool;
    }
    if (tid == 0) store_shared_result(&a.counters[(1 + f) * kCounterStride], 0u);   // leave the row counter clean
    if (publish_then_ticket(&a.counters[0], &s.ticket) != (unsigned int)(a.F - 1)) return;

    // ================= last workgroup of the call: choose the next frontier
    const int C = a.F * a.k;                                      // <= 64 * 16 = 1024
    uint64_t ck[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int c = tid + e * kExpThreads;
        const int cs = min(c, C - 1);
        const float sc = load_shared_result(&a.cand_scores[cs]);
        s.tok[cs] = load_shared_result(&a.cand_tokens[cs]);
        ck[e] = (c < C) ? make_key(sc, uint32_t(c)) : 0;
    }
    block_topk<4>(ck, a.k, s.topk);                               // synchronises: s.tok visible
    if (tid < a.k) {
        const uint64_t key = s.topk.top[tid];
        int c = (int)key_index(key);
        if (c < 0 || c >= C) c = 0;                               // only reachable with NaN scores
        // candidate scores never are -0.0 results of the sum above unless both terms are zero;
        // the key holds the score exactly otherwise
        const float sc = key_value(key);
        a.frontier_pool_idx[tid] = a.pool_count + c;
        a.frontier_tokens[tid] = s.tok[c];
        a.frontier_scores[tid] = sc;
        a.frontier_conf[tid] = (float)exp((double)sc);
    }
    if (tid == 0) store_shared_result(&a.counters[0], 0u);
}

// ------------------------------------------------------------------ rerank
struct RerankArgs {
    const int32_t *pool_tokens;
    const float *pool_scores;
    const int32_t *pool_parents;
    int pool_count, N, root_token;
    int32_t *tree_tokens;
    int32_t *tree_parents;
    float *tree_scores;
    int32_t *tree_depth;
    int32_t *tree_pool_idx;
    int32_t *n_nodes_out;
};

struct RerankSmem {
    TopkSmem topk;
    int16_t node_of[RADAR_POOL_MAX];     // pool index -> node number, -1 if dropped
    int32_t parent[RADAR_T_MAX];
};

__global__ __launch_bounds__(kTopkThreads) void rerank_kernel(RerankArgs a) {
    __shared__ RerankSmem s;
    const int tid = threadIdx.x;
    const int keep = min(a.N, a.pool_count);

    uint64_t keys[kTopkMaxEPT];
#pragma unroll
    for (int e = 0; e < kTopkMaxEPT; ++e) {
        const int i = tid + e * kTopkThreads;
        const float sc = a.pool_scores[max(0, min(i, a.pool_count - 1))];
        keys[e] = (i < a.pool_count) ? make_key(sc, uint32_t(i)) : 0;
        if (i < RADAR_POOL_MAX) s.node_of[i] = -1;
    }
    if (keep > 0) block_topk<kTopkMaxEPT>(keys, keep, s.topk);
    else __syncthreads();

    int my_pool = -1;
    if (tid >= 1 && tid <= keep) {
        const uint64_t key = s.topk.top[tid - 1];
        my_pool = (int)key_index(key);
        if (key == 0 || my_pool < 0 || my_pool >= a.pool_count) my_pool = 0;   // only reachable with NaN scores
        s.node_of[my_pool] = (int16_t)tid;
    }
    __syncthreads();
    if (tid <= a.N) {
        int tok = -1, par = -1, pidx = -1;
        float sc = 0.f;
        if (tid == 0) { tok = a.root_token; }
        else if (tid <= keep) {
            tok = a.pool_tokens[my_pool];
            sc = a.pool_scores[my_pool];
            pidx = my_pool;
            const int pp = a.pool_parents[my_pool];
            if (pp < 0) par = 0;
            else if (pp < a.pool_count && s.node_of[pp] >= 0 && s.node_of[pp] < tid) par = s.node_of[pp];
            else par = -2;
        }
        s.parent[tid] = par;
        a.tree_tokens[tid] = tok;
        a.tree_parents[tid] = par;
        a.tree_scores[tid] = sc;
        a.tree_pool_idx[tid] = pidx;
    }
    __syncthreads();
    if (tid <= a.N) {
        int depth = 0;
        if (tid >= 1 && tid <= keep && s.parent[tid] >= 0) {
            int cur = tid;
            // parents are strictly smaller node numbers, so this ends within tid steps
            while (cur > 0 && depth < RADAR_T_MAX) {
                const int p = s.parent[cur];
                if (p < 0 || p >= cur) { depth = 0; break; }
                cur = p;
                ++depth;
            }
        }
        a.tree_depth[tid] = depth;
    }
    if (tid == 0) *a.n_nodes_out = 1 + keep;
}

}  // namespace radar

using namespace radar;

extern "C" size_t radar_draft_expand_workspace_bytes(const radar_expand_desc *d) {
    if (!d || d->F < 1 || d->V < 1) return 0;
    const size_t nchunks = ((size_t)d->V + kExpChunk - 1) / kExpChunk;
    size_t bytes = kCounterBytes;
    bytes += (size_t)d->F * nchunks * RADAR_K_MAX * sizeof(uint64_t);
    bytes += (size_t)d->F * nchunks * (sizeof(double) + sizeof(float));
    return (bytes + 255) & ~size_t(255);
}

extern "C" radar_status radar_draft_expand(const float *logits, const float *parent_scores,
                                           const int32_t *parent_pool_idx, int32_t *cand_tokens, float *cand_scores,
                                           int32_t *frontier_pool_idx, int32_t *frontier_tokens,
                                           float *frontier_scores, float *frontier_conf, int32_t *pool_tokens,
                                           float *pool_scores, int32_t *pool_parents, const radar_expand_desc *d,
                                           void *workspace, size_t workspace_bytes, void *stream) {
    if (!d || !logits || !parent_scores || !parent_pool_idx || !cand_tokens || !cand_scores || !frontier_pool_idx ||
        !frontier_tokens || !frontier_scores || !frontier_conf || !pool_tokens || !pool_scores || !pool_parents ||
        !workspace)
        return RADAR_INVALID_ARG;
    if (d->F < 1 || d->V < 1 || d->k < 1 || d->k > d->V || d->pool_count < 0 ||
        (int64_t)d->pool_count + (int64_t)d->F * d->k > (int64_t)d->pool_capacity)
        return RADAR_INVALID_ARG;
    const int64_t nchunks = ((int64_t)d->V + kExpChunk - 1) / kExpChunk;
    if (d->F > RADAR_F_MAX || d->k > RADAR_K_MAX || nchunks > kExpMaxChunks) return RADAR_UNSUPPORTED_SHAPE;
    if (workspace_bytes < radar_draft_expand_workspace_bytes(d)) return RADAR_WORKSPACE_TOO_SMALL;
    if (((uintptr_t)workspace & 255) != 0) return RADAR_INVALID_ARG;

    ExpandArgs a;
    a.logits = logits; a.parent_scores = parent_scores; a.parent_pool_idx = parent_pool_idx;
    a.cand_tokens = cand_tokens; a.cand_scores = cand_scores;
    a.frontier_pool_idx = frontier_pool_idx; a.frontier_tokens = frontier_tokens;
    a.frontier_scores = frontier_scores; a.frontier_conf = frontier_conf;
    a.pool_tokens = pool_tokens; a.pool_scores = pool_scores; a.pool_parents = pool_parents;
    a.F = d->F; a.V = d->V; a.k = d->k; a.nchunks = (int)nchunks; a.pool_count = d->pool_count;
    char *ws = static_cast<char *>(workspace);
    a.counters = reinterpret_cast<unsigned int *>(ws);
    a.part_keys = reinterpret_cast<uint64_t *>(ws + kCounterBytes);
    const size_t nslots = (size_t)d->F * nchunks;
    a.part_l = reinterpret_cast<double *>(ws + kCounterBytes + nslots * RADAR_K_MAX * sizeof(uint64_t));
    a.part_m = reinterpret_cast<float *>(ws + kCounterBytes + nslots * (RADAR_K_MAX * sizeof(uint64_t) + sizeof(double)));

    const dim3 grid((unsigned)nchunks, (unsigned)d->F), block(kExpThreads);
    const bool vec4 = (d->V % 4 == 0) && (((uintptr_t)logits & 15) == 0);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const hipError_t e = vec4 ? launch("expand", expand_kernel<true>, grid, block, 0, st, a)
                              : launch("expand", expand_kernel<false>, grid, block, 0, st, a);
    return e == hipSuccess ? RADAR_OK : RADAR_HIP_ERROR;
}

extern "C" size_t radar_draft_rerank_workspace_bytes(int32_t pool_count, int32_t N) {
    (void)pool_count; (void)N;
    return 256;   // rerank keeps everything in LDS; a minimal workspace keeps the calling convention uniform
}

extern "C" radar_status radar_draft_rerank(const int32_t *pool_tokens, const float *pool_scores,
                                           const int32_t *pool_parents, int32_t pool_count, int32_t N,
                                           int32_t root_token, int32_t *tree_tokens, int32_t *tree_parents,
                                           float *tree_scores, int32_t *tree_depth, int32_t *tree_pool_idx,
                                           int32_t *n_nodes_out, void *workspace, size_t workspace_bytes,
                                           void *stream) {
    (void)workspace; (void)workspace_bytes;
    if (!pool_tokens || !pool_scores || !pool_parents || !tree_tokens || !tree_parents || !tree_scores ||
        !tree_depth || !tree_pool_idx || !n_nodes_out)
        return RADAR_INVALID_ARG;
    if (pool_count < 0 || N < 0) return RADAR_INVALID_ARG;
    if (pool_count > RADAR_POOL_MAX || N >= RADAR_T_MAX) return RADAR_UNSUPPORTED_SHAPE;
    RerankArgs a;
    a.pool_tokens = pool_tokens; a.pool_scores = pool_scores; a.pool_parents = pool_parents;
    a.pool_count = pool_count; a.N = N; a.root_token = root_token;
    a.tree_tokens = tree_tokens; a.tree_parents = tree_parents; a.tree_scores = tree_scores;
    a.tree_depth = tree_depth; a.tree_pool_idx = tree_pool_idx; a.n_nodes_out = n_nodes_out;
    const hipError_t e = launch("rerank", rerank_kernel, dim3(1), dim3(kTopkThreads), 0, static_cast<hipStream_t>(stream), a);
    return e == hipSuccess ? RADAR_OK : RADAR_HIP_ERROR;
}
