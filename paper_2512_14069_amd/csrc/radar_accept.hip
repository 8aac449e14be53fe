// Verification walk of RADAR's speculative-sampling cycle (Sec. 3, Eq. 1-2; tree
// form per Sec. 4.3, Eq. 11-13) as one HIP launch for gfx950.
//
// Phase 1, grid (chunks of 4096 logits, tree rows, sequences): one streaming
// read of the target logits (T*V*4 bytes per sequence) leaves per chunk the
// arg-max key and, in sampling mode, (max, sum exp) of the temperature-scaled
// row.  Phase 2: the workgroup whose arrival ticket is the last of its ROW
// merges that row's chunk partials (one per lane).  Phase 3: the workgroup whose
// ticket is the last of its SEQUENCE walks the tree in a single wavefront (one
// lane per node, sibling sets found with ballots); the residual draw needs one
// more pass over a single 16 KB chunk.  Arrival counters sit 64 B apart.
#include "radar_device.h"
#include "radar_host.h"

namespace radar {

constexpr int kAccThreads = 256;
constexpr int kAccEPT = 16;
constexpr int kAccChunk = kAccThreads * kAccEPT;
constexpr int kAccMaxChunks = 256;
constexpr int kAccCounterStride = 16;   // counters 64 B apart (same-line fetch-adds serialise)

struct AcceptArgs {
    const float *logits;
    const int32_t *tokens;
    const int32_t *parents;
    const int32_t *n_nodes;
    const float *uniforms;
    int32_t *accept_len;
    int32_t *accept_path;
    int32_t *bonus;
    int B, T, V, D_max, mode, nchunks;
    float inv_temp_f;
    double inv_temp;
    unsigned int *counters;     // [(b*T + r) * stride] chunks of a row, [(B*T + b) * stride] rows of a sequence
    uint64_t *row_key;          // [B][T] arg-max key of the row
    double *row_L;              // [B][T] sum of exp(y - row_M)
    float *row_M;               // [B][T]
    uint64_t *part_key;         // [B][T][nchunks] arg-max key of the chunk
    double *part_l;             // [B][T][nchunks] sum of exp(y - part_m) over the chunk, y = logit / temperature
    float *part_m;              // [B][T][nchunks] reference maximum of the chunk
};

struct AcceptSmem {
    uint64_t wave_key[4];
    float wave_m[4];
    double wave_l[4];
    unsigned int ticket;
    // phase 2
    int row_arg[RADAR_T_MAX];
    double row_lse[RADAR_T_MAX];
    float row_M[RADAR_T_MAX];
    double row_L[RADAR_T_MAX];
    int par[RADAR_T_MAX], tok[RADAR_T_MAX];
    double pc[RADAR_T_MAX];
    int rej[RADAR_T_MAX];
    int path[RADAR_T_MAX];
    int nrej, cur, chunk_pick, bonus, owner, last_pos;
    double R, residual_target;
    double mass[kAccMaxChunks];
    double tsum[kAccThreads];
};

template <bool VEC4>
__global__ __launch_bounds__(kAccThreads) void accept_kernel(AcceptArgs a) {
    __shared__ AcceptSmem s;
    const int tid = threadIdx.x, lane = lane_id(), w = wave_id();
    const int chunk = blockIdx.x, r = blockIdx.y, b = blockIdx.z;
    int nn = a.n_nodes ? a.n_nodes[b] : a.T;
    nn = max(1, min(nn, a.T));
    if (r >= nn) return;
    const bool sampling = (a.mode == RADAR_ACCEPT_SAMPLE);
    const float *row = a.logits + ((size_t)b * a.T + r) * a.V;
    const int base = chunk * kAccChunk;

    // ---------------- phase 1: chunk arg-max (and scaled max / sum-exp)
    float x[kAccEPT];
    uint64_t best = 0;
#pragma unroll
    for (int g = 0; g < kAccEPT / 4; ++g) {
        const int idx0 = base + g * (kAccThreads * 4) + tid * 4;
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
            if (idx0 + j < a.V) best = max_u64(best, make_key(x[4 * g + j], uint32_t(idx0 + j)));
    }
    best = wave_max_u64(best);
    if (lane == 0) s.wave_key[w] = best;
    if (sampling) {
        // exponent differences are formed in fp64 and the sums are kept in fp64, so that the
        // only fp32 rounding left is the one inside expf (unbiased, averaging out over a chunk)
        float tm = -INFINITY;
#pragma unroll
        for (int e = 0; e < kAccEPT; ++e) tm = fmaxf(tm, x[e] * a.inv_temp_f);
        const float wm = wave_max_f32(tm);
        double tl = 0.0;
        if (wm > -INFINITY) {
#pragma unroll
            for (int e = 0; e < kAccEPT; ++e)
                tl += (double)expf((float)((double)x[e] * a.inv_temp - (double)wm));
        }
        const double wl = wave_sum_f64(tl);
        if (lane == 0) { s.wave_m[w] = wm; s.wave_l[w] = wl; }
    }
    __syncthreads();
    const size_t pslot = ((size_t)b * a.T + r) * a.nchunks + chunk;
    if (w == 0) {
        const uint64_t bk = max_u64(max_u64(s.wave_key[0], s.wave_key[1]), max_u64(s.wave_key[2], s.wave_key[3]));
        if (lane == 0) store_shared_result(&a.part_key[pslot], bk);
        if (sampling) {
            const float m = fmaxf(fmaxf(s.wave_m[0], s.wave_m[1]), fmaxf(s.wave_m[2], s.wave_m[3]));
            double t = 0.0;                                  // lanes 0..3: one fp64 term each
            if (lane < 4 && s.wave_m[lane] > -INFINITY) t = s.wave_l[lane] * exp((double)s.wave_m[lane] - (double)m);
            const uint64_t tb = (uint64_t)__double_as_longlong(t);
            const double l = (__longlong_as_double((long long)readlane_u64(tb, 0)) +
                              __longlong_as_double((long long)readlane_u64(tb, 1))) +
                             (__longlong_as_double((long long)readlane_u64(tb, 2)) +
                              __longlong_as_double((long long)readlane_u64(tb, 3)));
            if (lane == 0) {
                store_shared_result(&a.part_m[pslot], m);
                store_shared_result(&a.part_l[pslot], l);
            }
        }
    }
    unsigned int *row_counter = &a.counters[((size_t)b * a.T + r) * kAccCounterStride];
    if (publish_then_ticket(row_counter, &s.ticket) != (unsigned int)(a.nchunks - 1)) return;

    // ---------------- phase 2: last workgroup of row r -- merge its chunk partials (one per lane)
    {
        const size_t p0 = ((size_t)b * a.T + r) * a.nchunks;
        const int c = min(tid, a.nchunks - 1);
        uint64_t kb = load_shared_result(&a.part_key[p0 + c]);
        float mc = -INFINITY;
        double lc = 0.0;
        if (sampling) {
            mc = load_shared_result(&a.part_m[p0 + c]);
            lc = load_shared_result(&a.part_l[p0 + c]);
        }
        if (tid >= a.nchunks) { kb = 0; mc = -INFINITY; }
        kb = wave_max_u64(kb);
        const float wmx = wave_max_f32(mc);
        if (lane == 0) { s.wave_key[w] = kb; s.wave_m[w] = wmx; }
        __syncthreads();
        const float M = fmaxf(fmaxf(s.wave_m[0], s.wave_m[1]), fmaxf(s.wave_m[2], s.wave_m[3]));
        const double term = (sampling && mc > -INFINITY) ? lc * exp((double)mc - (double)M) : 0.0;
        const double ws = wave_sum_f64(term);
        if (lane == 0) s.wave_l[w] = ws;
        __syncthreads();
        if (tid == 0) {
            const size_t rs = (size_t)b * a.T + r;
            store_shared_result(&a.row_key[rs],
                                max_u64(max_u64(s.wave_key[0], s.wave_key[1]), max_u64(s.wave_key[2], s.wave_key[3])));
            if (sampling) {
                store_shared_result(&a.row_M[rs], M);
                store_shared_result(&a.row_L[rs], (s.wave_l[0] + s.wave_l[1]) + (s.wave_l[2] + s.wave_l[3]));
            }
            store_shared_result(row_counter, 0u);            // leave the row counter clean for the next call
        }
    }
    unsigned int *seq_counter = &a.counters[((size_t)a.B * a.T + b) * kAccCounterStride];
    if (publish_then_ticket(seq_counter, &s.ticket) != (unsigned int)(nn - 1)) return;
    if (tid == 0) store_shared_result(seq_counter, 0u);

    // ---------------- phase 3: last workgroup of sequence b
    if (tid < RADAR_T_MAX) {
        const size_t rs = (size_t)b * a.T + min(tid, nn - 1);
        const uint64_t kb = load_shared_result(&a.row_key[rs]);
        s.row_arg[tid] = (int)key_index(kb);
        if (sampling) {
            const float M = load_shared_result(&a.row_M[rs]);
            const double L = load_shared_result(&a.row_L[rs]);
            s.row_M[tid] = M; s.row_L[tid] = L; s.row_lse[tid] = (double)M + log(L);
        }
    }
    if (tid < RADAR_T_MAX) {
        int p = -1, t = -1;
        if (tid < nn) { p = a.parents[(size_t)b * a.T + tid]; t = a.tokens[(size_t)b * a.T + tid]; }
        s.par[tid] = p; s.tok[tid] = t;
    }
    __syncthreads();

    int32_t *path = a.accept_path + (size_t)b * (a.D_max + 1);
    if (w == 0) {
        const int c = lane;
        const int p = s.par[c], t = s.tok[c];
        const bool valid = (c > 0 && c < nn && p >= 0 && p < c);
        int cur = 0, len = 0;
        if (lane == 0) s.path[0] = 0;
        if (!sampling) {
            const bool match = valid && s.row_arg[p] == t;
            while (len < a.D_max) {
                const uint64_t m = __ballot(match && p == cur);
                if (!m) break;
                cur = __ffsll((long long)m) - 1;
                ++len;
                if (lane == 0) s.path[len] = cur;
            }
            if (lane == 0) { a.accept_len[b] = len; a.bonus[b] = s.row_arg[cur]; }
        } else {
            // probability of each node's token under its parent's row
            double pcv = 0.0;
            if (valid && t >= 0 && t < a.V) {
                const float xv = a.logits[((size_t)b * a.T + p) * a.V + t];
                pcv = exp((double)xv * a.inv_temp - s.row_lse[p]);
            }
            s.pc[c] = pcv;
            wave_lds_sync();
            bool dup = false;                         // same token as an earlier sibling
            for (int o = 1; o < c; ++o) dup = dup || (valid && o > p && s.par[o] == p && s.tok[o] == t);
            const float *u = a.uniforms + (size_t)b * (a.T + 1);
            double R = 0.0;
            int nrej = 0;
            for (;;) {
                uint64_t kids = (len < a.D_max) ? __ballot(valid && !dup && p == cur) : 0ull;
                R = 0.0; nrej = 0;
                int next = -1;
                while (kids) {
                    const int cc = __ffsll((long long)kids) - 1;
                    kids &= kids - 1;
                    const double pcc = s.pc[cc];
                    if ((double)u[cc] * (1.0 - R) < pcc) { next = cc; break; }
                    R += pcc;
                    if (lane == 0) s.rej[nrej] = s.tok[cc];
                    ++nrej;
                }
                if (next < 0) break;
                cur = next;
                ++len;
                if (lane == 0) s.path[len] = cur;
            }
            wave_lds_sync();
            // residual draw: find the chunk that holds the target mass
            const float M = s.row_M[cur];
            const size_t p0 = ((size_t)b * a.T + cur) * a.nchunks;
            const float *xr = a.logits + ((size_t)b * a.T + cur) * a.V;
            for (int cch = lane; cch < a.nchunks; cch += kWave) {
                const float mc = load_shared_result(&a.part_m[p0 + cch]);
                const double lc = load_shared_result(&a.part_l[p0 + cch]);
                double mass = (mc > -INFINITY) ? lc * exp((double)mc - (double)M) : 0.0;
                for (int j = 0; j < nrej; ++j) {
                    const int tj = s.rej[j];
                    if (tj >= 0 && tj < a.V && tj / kAccChunk == cch)
                        mass -= exp((double)xr[tj] * a.inv_temp - (double)M);
                }
                s.mass[cch] = mass > 0.0 ? mass : 0.0;
            }
            wave_lds_sync();
            const double target = (double)u[a.T] * (1.0 - R) * s.row_L[cur];
            double cum = 0.0;
            int pick = -1;
            for (int cch = 0; cch < a.nchunks; ++cch) {
                const double mcc = s.mass[cch];
                if (cum + mcc > target) { pick = cch; break; }
                cum += mcc;
            }
            if (pick < 0) {                            // rounding pushed the target past the total
                for (int cch = a.nchunks - 1; cch >= 0; --cch)
                    if (s.mass[cch] > 0.0) { pick = cch; break; }
                if (pick < 0) pick = 0;
                cum = target;                          // nothing will exceed it: fall back to the last token with mass
            }
            if (lane == 0) {
                a.accept_len[b] = len;
                s.cur = cur; s.nrej = nrej; s.R = R; s.chunk_pick = pick; s.residual_target = target - cum;
                s.owner = kAccThreads; s.last_pos = -1; s.bonus = -1;
            }
        }
        wave_lds_sync();
        if (c <= a.D_max) path[c] = (c <= len) ? s.path[c] : -1;
    }
    if (!sampling) return;
    __syncthreads();

    // (b) residual draw inside the chosen chunk: every lane owns 16 consecutive tokens
    {
        const int cur = s.cur, nrej = s.nrej;
        const float M = s.row_M[cur];
        const float *xr = a.logits + ((size_t)b * a.T + cur) * a.V;
        const int i0 = s.chunk_pick * kAccChunk + tid * kAccEPT;
        double pv[kAccEPT];
        double sum = 0.0;
        int lastpos = -1;
#pragma unroll
        for (int e = 0; e < kAccEPT; ++e) {
            const int i = i0 + e;
            double v = 0.0;
            if (i < a.V) {
                v = exp((double)xr[i] * a.inv_temp - (double)M);
                for (int j = 0; j < nrej; ++j) if (s.rej[j] == i) v = 0.0;
            }
            pv[e] = v;
            sum += v;
            if (v > 0.0) lastpos = i;
        }
        s.tsum[tid] = sum;
        __syncthreads();
        double prefix = 0.0;
        for (int j = 0; j < tid; ++j) prefix += s.tsum[j];
        const double target = s.residual_target;
        if (prefix + sum > target) atomicMin(&s.owner, tid);
        if (lastpos >= 0) atomicMax(&s.last_pos, lastpos);
        __syncthreads();
        if (s.owner == tid) {
            double cdf = prefix;
            int pick = -1;
#pragma unroll
            for (int e = 0; e < kAccEPT; ++e) {
                cdf += pv[e];
                if (pick < 0 && pv[e] > 0.0 && cdf > target) pick = i0 + e;
            }
            s.bonus = pick >= 0 ? pick : lastpos;
        }
        __syncthreads();
        if (tid == 0) a.bonus[b] = (s.owner < kAccThreads && s.bonus >= 0) ? s.bonus : s.last_pos;
    }
}

__global__ void validate_tree_kernel(const int32_t *parents, const int32_t *n_nodes, int B, int T, int32_t *bad) {
    __shared__ int count;
    if (threadIdx.x == 0) count = 0;
    __syncthreads();
    for (int i = threadIdx.x; i < B * T; i += blockDim.x) {
        const int b = i / T, n = i % T;
        int nn = n_nodes ? n_nodes[b] : T;
        nn = max(1, min(nn, T));
        if (n < nn) {
            const int p = parents[i];
            const bool ok = (n == 0) ? (p == -1) : (p >= 0 && p < n);
            if (!ok) atomicAdd(&count, 1);
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) *bad = count;
}

}  // namespace radar

using namespace radar;

// Workspace layout: arrival counters (one 64-byte slot per row and per sequence), row results,
// chunk partials.  Returns the total size; fills the pointers when `ws` is given.
static size_t accept_layout(int B, int T, size_t nchunks, char *ws, AcceptArgs *a) {
    const size_t rows = (size_t)B * T, slots = rows * nchunks;
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t o = off; off += (bytes + 255) & ~size_t(255); return o; };
    const size_t o_cnt = take((rows + B) * kAccCounterStride * sizeof(unsigned int));
    const size_t o_rk = take(rows * sizeof(uint64_t)), o_rl = take(rows * sizeof(double)), o_rm = take(rows * sizeof(float));
    const size_t o_pk = take(slots * sizeof(uint64_t)), o_pl = take(slots * sizeof(double)), o_pm = take(slots * sizeof(float));
    if (ws) {
        a->counters = reinterpret_cast<unsigned int *>(ws + o_cnt);
        a->row_key = reinterpret_cast<uint64_t *>(ws + o_rk);
        a->row_L = reinterpret_cast<double *>(ws + o_rl);
        a->row_M = reinterpret_cast<float *>(ws + o_rm);
        a->part_key = reinterpret_cast<uint64_t *>(ws + o_pk);
        a->part_l = reinterpret_cast<double *>(ws + o_pl);
        a->part_m = reinterpret_cast<float *>(ws + o_pm);
    }
    return off;
}

extern "C" size_t radar_verify_accept_workspace_bytes(const radar_accept_desc *d) {
    if (!d || d->B < 1 || d->T_max < 1 || d->V < 1) return 0;
    const size_t nchunks = ((size_t)d->V + kAccChunk - 1) / kAccChunk;
    return accept_layout(d->B, d->T_max, nchunks, nullptr, nullptr);
}

extern "C" radar_status radar_verify_accept(const float *target_logits, const int32_t *draft_tokens,
                                            const int32_t *parents, const int32_t *n_nodes, const float *uniforms,
                                            int32_t *accept_len, int32_t *accept_path, int32_t *bonus_token,
                                            const radar_accept_desc *d, void *workspace, size_t workspace_bytes,
                                            void *stream) {
    if (!d || !target_logits || !draft_tokens || !parents || !accept_len || !accept_path || !bonus_token || !workspace)
        return RADAR_INVALID_ARG;
    if (d->B < 1 || d->T_max < 1 || d->V < 1 || d->D_max < 0) return RADAR_INVALID_ARG;
    if (d->mode != RADAR_ACCEPT_GREEDY && d->mode != RADAR_ACCEPT_SAMPLE) return RADAR_INVALID_ARG;
    if (d->mode == RADAR_ACCEPT_SAMPLE && (!(d->temperature > 0.0f) || !uniforms)) return RADAR_INVALID_ARG;
    const int64_t nchunks = ((int64_t)d->V + kAccChunk - 1) / kAccChunk;
    if (d->T_max > RADAR_T_MAX || d->D_max >= RADAR_T_MAX || d->B > 65535 || nchunks > kAccMaxChunks)
        return RADAR_UNSUPPORTED_SHAPE;
    if (workspace_bytes < radar_verify_accept_workspace_bytes(d)) return RADAR_WORKSPACE_TOO_SMALL;
    if (((uintptr_t)workspace & 255) != 0) return RADAR_INVALID_ARG;

    AcceptArgs a;
    a.logits = target_logits; a.tokens = draft_tokens; a.parents = parents; a.n_nodes = n_nodes; a.uniforms = uniforms;
    a.accept_len = accept_len; a.accept_path = accept_path; a.bonus = bonus_token;
    a.B = d->B; a.T = d->T_max; a.V = d->V; a.D_max = d->D_max; a.mode = d->mode; a.nchunks = (int)nchunks;
    a.inv_temp = d->mode == RADAR_ACCEPT_SAMPLE ? 1.0 / (double)d->temperature : 1.0;
    a.inv_temp_f = (float)a.inv_temp;
    accept_layout(d->B, d->T_max, (size_t)nchunks, static_cast<char *>(workspace), &a);

    const dim3 grid((unsigned)nchunks, (unsigned)d->T_max, (unsigned)d->B), block(kAccThreads);
    const bool vec4 = (d->V % 4 == 0) && (((uintptr_t)target_logits & 15) == 0);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const hipError_t e = vec4 ? launch("accept", accept_kernel<true>, grid, block, 0, st, a)
                              : launch("accept", accept_kernel<false>, grid, block, 0, st, a);
    return e == hipSuccess ? RADAR_OK : RADAR_HIP_ERROR;
}

extern "C" radar_status radar_debug_validate_tree(const int32_t *parents, const int32_t *n_nodes, int32_t B,
                                                  int32_t T_max, int32_t *bad_count_out, void *stream) {
    if (!parents || !bad_count_out || B < 1 || T_max < 1) return RADAR_INVALID_ARG;
    const hipError_t e = launch("validate_tree", validate_tree_kernel, dim3(1), dim3(256), 0,
                                static_cast<hipStream_t>(stream), parents, n_nodes, (int)B, (int)T_max, bad_count_out);
    return e == hipSuccess ? RADAR_OK : RADAR_HIP_ERROR;
}
