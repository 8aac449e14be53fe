// radar_verify_accept_q: verification with draft distributions (Sec. 3, Eq. 1-2), for trees
// whose tokens were drawn from the draft model's distributions.
//
// Two launches.  (1) Row statistics, spread over the whole chip: one workgroup per 16384
// logits of every target row and every draft row streams its chunk once and leaves (max, sum
// of exp) partials; the workgroup that completes a row (arrival ticket) merges them into the
// row's normaliser.  This is the HBM-bound part: it reads every logit once.  (2) The walk, one
// workgroup per sequence: sequential by nature (Eq. 1 is applied child by child, Eq. 2 changes
// the distribution every later test sees).  Every rejection is one vocabulary-wide pass of the
// workgroup that turns the unnormalised residual u into max(0, u - W q) (W = sum u), keeps it
// in a workspace row and leaves sums per 256 tokens in LDS; the bonus token is then found from
// those sums without another pass.  A walk that ends without a rejection draws the bonus from
// the row's chunk partials and one 16384-token chunk.
#include "radar_device.h"
#include "radar_host.h"

namespace radar {

constexpr int kAqThreads = 1024;
constexpr int kAqWaves = kAqThreads / kWave;
constexpr int kAqChunk = 16 * kAqThreads;             // logits per workgroup in the statistics launch
constexpr int kAqMaxChunks = 64;                      // V <= 1,048,576
constexpr int kAqGran = 4 * kWave;                    // tokens per partial sum in the walk (one wavefront x 16 B)
constexpr int kAqMaxGran = kAqMaxChunks * kAqChunk / kAqGran;   // 4096
constexpr int kAqCounterStride = 8;                   // arrival counters 32 B apart

struct AqArgs {
    const float *target;        // [B][T][V]
    const float *draft;         // [B][Tq][V]
    const int32_t *q_rows;      // [B][T] or null
    const int32_t *tokens, *parents, *n_nodes;
    const float *uniforms;      // [B][T+1]
    int32_t *accept_len, *accept_path, *bonus;
    int B, T, Tq, V, D_max, nchunks;
    double inv_t, inv_td;
    unsigned int *counters;     // one per row of the statistics launch
    float *part_m;              // [rows][nchunks] chunk maximum (raw logit)
    double *part_l;             // [rows][nchunks] sum of exp((x - part_m) * inv_temperature)
    float *row_m;               // [rows]
    double *row_l;              // [rows]
    float *ubuf;                // [B][V] unnormalised residual of the node being verified
};

// exp((x - m) * inv_temp) with the difference formed in fp64, rounded to fp32 once, and the fp32
// hardware exponential; the sums that use it are fp64.
__device__ __forceinline__ double exp_rel(float x, float m, double inv_temp) {
    return (double)__expf((float)(((double)x - (double)m) * inv_temp));
}

// the same in fp32 throughout (relative error about 1e-7 per unit of |x - m| * inv_temp)
__device__ __forceinline__ float exp_rel_f32(float x, float m, float inv_temp) { return __expf((x - m) * inv_temp); }

// sum over the workgroup of one double per thread, fixed order; every thread gets it
__device__ __forceinline__ double block_sum_f64(double v, double *wred) {
    const double ws = wave_sum_f64(v);
    __syncthreads();
    if (lane_id() == 0) wred[wave_id()] = ws;
    __syncthreads();
    double t = 0.0;
#pragma unroll
    for (int i = 0; i < kAqWaves; ++i) t += wred[i];
    return t;
}

// rows of the statistics launch: b * (T + Tq) + r, r < T a target row, else draft row r - T
template <bool VEC4>
__global__ __launch_bounds__(kAqThreads) void accept_q_stats_kernel(AqArgs a) {
    __shared__ float wmax[kAqWaves];
    __shared__ double wred[kAqWaves];
    __shared__ unsigned int ticket;
    const int tid = threadIdx.x, lane = lane_id(), w = wave_id();
    const int R = blockIdx.y, rows_per_seq = a.T + a.Tq;
    const int b = R / rows_per_seq, r = R - b * rows_per_seq;
    const int nn = a.n_nodes ? min(max(a.n_nodes[b], 0), a.T) : a.T;
    const bool is_target = r < a.T;
    // rows nothing will read: target rows past the tree, and, when nodes use their own draft
    // row, the root's and those past the tree
    if (is_target ? r >= nn : (a.q_rows == nullptr && (r - a.T == 0 || r - a.T >= nn))) return;
    const float *row = is_target ? a.target + ((size_t)b * a.T + r) * a.V : a.draft + ((size_t)b * a.Tq + (r - a.T)) * a.V;
    const double inv = is_target ? a.inv_t : a.inv_td;
    const int base = blockIdx.x * kAqChunk;

    float x[16];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const int i0 = base + g * (kAqThreads * 4) + tid * 4;
        if (VEC4) {
            const float4 v = *reinterpret_cast<const float4 *>(row + (i0 < a.V ? i0 : 0));
            x[4 * g] = v.x; x[4 * g + 1] = v.y; x[4 * g + 2] = v.z; x[4 * g + 3] = v.w;
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) x[4 * g + j] = row[min(i0 + j, a.V - 1)];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (i0 + j >= a.V) x[4 * g + j] = -INFINITY;
    }
    float m = x[0];
#pragma unroll
    for (int e = 1; e < 16; ++e) m = fmaxf(m, x[e]);
    m = wave_max_f32(m);
    if (lane == 0) wmax[w] = m;
    __syncthreads();
    m = wmax[0];
#pragma unroll
    for (int i = 1; i < kAqWaves; ++i) m = fmaxf(m, wmax[i]);
    double l = 0.0;
    if (m > -INFINITY) {
#pragma unroll
        for (int e = 0; e < 16; ++e) l += exp_rel(x[e], m, inv);
    }
    l = block_sum_f64(l, wred);
    const size_t slot = (size_t)R * a.nchunks + blockIdx.x;
    if (tid == 0) {
        store_shared_result(&a.part_m[slot], m);
        store_shared_result(&a.part_l[slot], l);
    }
    unsigned int *counter = &a.counters[(size_t)R * kAqCounterStride];
    if (publish_then_ticket(counter, &ticket) != (unsigned int)(a.nchunks - 1)) return;
    if (w != 0) return;
    // last chunk of the row: merge the partials (the counter goes back to zero for the next call)
    float mr = -INFINITY;
    for (int c = lane; c < a.nchunks; c += kWave) mr = fmaxf(mr, load_shared_result(&a.part_m[(size_t)R * a.nchunks + c]));
    mr = wave_max_f32(mr);
    double lr = 0.0;
    for (int c = lane; c < a.nchunks; c += kWave) {
        const float mc = load_shared_result(&a.part_m[(size_t)R * a.nchunks + c]);
        const double lc = load_shared_result(&a.part_l[(size_t)R * a.nchunks + c]);
        if (mc > -INFINITY) lr += lc * exp(((double)mc - (double)mr) * inv);
    }
    lr = wave_sum_f64(lr);
    if (lane == 0) {
        a.row_m[R] = mr;
        a.row_l[R] = lr;
        store_shared_result(counter, 0u);
    }
}

// ------------------------------------------------------------------------------------ walk
struct AqSmem {
    double gsum[kAqMaxGran];     // residual mass per 256 tokens (of the last pass)
    double wred[kAqWaves];
    double px[kWave], qx[kWave]; // per node: residual at its token under its parent, draft probability of its token
    int par[kWave], tok[kWave], qrow[kWave];
    float uni[kWave + 1];
    double W;                    // mass of the residual
    unsigned long long kids;     // untried children of the current node
    int cur, len, next, have_u, pick, gran;
    double before;               // residual mass in front of the chosen granule
};

// One pass over tokens [lo, hi) (lo a multiple of 4096) of sequence b:
//   u(i) = have_u ? ubuf[i] : softmax(target row)[i];   u(i) <- max(0, u(i) - W * q(i)) when q is given;
// u is written to ubuf (as fp32), its sums per 256 tokens to s.gsum[(i - lo) / 256]; returns the total
// of the stored values.  All threads call it.
template <bool VEC4>
__device__ __forceinline__ double residual_pass(const AqArgs &a, AqSmem &s, int b, const float *prow, float pm, double pinv_l,
                                                const float *qrow, float qm, double qinv_l, double W, int lo, int hi) {
    const int tid = threadIdx.x, lane = lane_id(), w = wave_id();
    float *ub = a.ubuf + (size_t)b * a.V;
    const int ngran = (hi - lo + kAqGran - 1) / kAqGran;
    const float it_f = (float)a.inv_t, itd_f = (float)a.inv_td, pinv_l_f = (float)pinv_l, qinv_l_f = (float)qinv_l, W_f = (float)W;
    constexpr int U = 4;                                             // 4096-token steps whose loads are in flight together
    for (int base0 = lo + tid * 4; base0 - lane * 4 < hi; base0 += U * kAqThreads * 4) {
        float u4[U][4], q4[U][4];
#pragma unroll
        for (int k = 0; k < U; ++k) {
            const int base = base0 + k * kAqThreads * 4;
            if (VEC4) {                                              // V % 4 == 0: a float4 is all in or all out
                const int i0 = base < hi ? base : lo;                // out of range: any legal address, masked below
                const float4 v = *reinterpret_cast<const float4 *>((prow ? prow : ub) + i0);
                u4[k][0] = v.x; u4[k][1] = v.y; u4[k][2] = v.z; u4[k][3] = v.w;
                if (qrow) {
                    const float4 y = *reinterpret_cast<const float4 *>(qrow + i0);
                    q4[k][0] = y.x; q4[k][1] = y.y; q4[k][2] = y.z; q4[k][3] = y.w;
                }
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int i = min(base + j, hi - 1);
                    u4[k][j] = (prow ? prow : ub)[i];
                    if (qrow) q4[k][j] = qrow[i];
                }
            }
        }
#pragma unroll
        for (int k = 0; k < U; ++k) {
            const int base = base0 + k * kAqThreads * 4;
            if (base - lane * 4 >= hi) break;                        // wave-uniform
            // fp32 per token (one workgroup's vector ALUs, not its memory path, bound this loop), fp64 sums
            float out[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float u = prow ? exp_rel_f32(u4[k][j], pm, it_f) * pinv_l_f : u4[k][j];
                if (qrow) u = fmaxf(0.f, fmaf(-W_f, exp_rel_f32(q4[k][j], qm, itd_f) * qinv_l_f, u));
                out[j] = (base + j < hi) ? u : 0.f;
            }
            double sum = ((double)out[0] + (double)out[1]) + ((double)out[2] + (double)out[3]);
            if (VEC4) {
                if (base < hi) *reinterpret_cast<float4 *>(ub + base) = make_float4(out[0], out[1], out[2], out[3]);
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (base + j < hi) ub[base + j] = out[j];
            }
            sum = wave_sum_f64(sum);
            if (lane == 0) s.gsum[(base - lo) / kAqGran] = sum;
        }
    }
    __syncthreads();
    double part = 0.0;
    for (int g = tid; g < ngran; g += kAqThreads) part += s.gsum[g];
    return block_sum_f64(part, s.wred);
}

// Inverse CDF by wavefront 0: first token i in [lo, hi) with before0 + sum_{lo..i} u > target, or, if
// the sums never get there (rounding), the last token with u > 0; -1 if there is none.  The sums per
// 256 tokens are in s.gsum, u itself in ubuf.  Returns the token to every lane of wavefront 0.
template <bool VEC4>
__device__ __forceinline__ int pick_token(const AqArgs &a, AqSmem &s, int b, double before0, double target, int lo, int hi) {
    const int lane = lane_id();
    const float *ub = a.ubuf + (size_t)b * a.V;
    const int ngran = (hi - lo + kAqGran - 1) / kAqGran;
    const int per = (ngran + kWave - 1) / kWave;
    // each lane owns `per` consecutive granules
    double mine = 0.0;
    int last_pos = -1;
    for (int g = lane * per; g < min((lane + 1) * per, ngran); ++g) {
        mine += s.gsum[g];
        if (s.gsum[g] > 0.0) last_pos = g;
    }
    const double incl = wave_scan_f64(mine);
    const uint64_t cross = __ballot(before0 + incl > target);
    int g_pick;
    double before;
    if (cross != 0) {
        const int owner = __ffsll((long long)cross) - 1;
        // the owner walks its granules
        int g_loc = -1;
        double acc = before0 + incl - mine, bef = acc;
        for (int g = lane * per; g < min((lane + 1) * per, ngran); ++g) {
            if (g_loc < 0) {
                bef = acc;
                acc += s.gsum[g];
                if (acc > target) g_loc = g;
            }
        }
        if (g_loc < 0) {                                             // the lane's own running sum was rounded differently: its last granule
            g_loc = min((lane + 1) * per, ngran) - 1;
            bef = acc - s.gsum[g_loc];
        }
        g_pick = __shfl(g_loc, owner);
        before = readlane_f64(bef, owner);
    } else {
        // no crossing: the last granule with mass
        int lp = last_pos;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) lp = max(lp, __shfl_xor(lp, off));
        if (lp < 0) return -1;
        g_pick = lp;
        before = -1.0;                                               // marks "take the last positive token"
    }
    // the 256 tokens of the granule, 4 per lane in token order
    const int i0 = lo + g_pick * kAqGran + lane * 4;
    double v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = (i0 + j < hi) ? (double)ub[i0 + j] : 0.0;
    if (before < 0.0) {
        int lastj = -1;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (v[j] > 0.0) lastj = i0 + j;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) lastj = max(lastj, __shfl_xor(lastj, off));
        return lastj;
    }
    const double lsum = (v[0] + v[1]) + (v[2] + v[3]);
    const double linc = wave_scan_f64(lsum);
    const uint64_t c2 = __ballot(before + linc > target);
    if (c2 == 0) {                                                   // the granule's own sum was rounded differently: its last positive token
        int lastj = -1;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (v[j] > 0.0) lastj = i0 + j;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) lastj = max(lastj, __shfl_xor(lastj, off));
        return lastj;
    }
    const int owner2 = __ffsll((long long)c2) - 1;
    double acc = before + linc - lsum;
    int pick = -1;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        acc += v[j];
        if (pick < 0 && acc > target) pick = i0 + j;
    }
    return __shfl(pick, owner2);
}

template <bool VEC4>
__global__ __launch_bounds__(kAqThreads) void accept_q_walk_kernel(AqArgs a) {
    __shared__ AqSmem s;
    const int tid = threadIdx.x, lane = lane_id(), w = wave_id();
    const int b = blockIdx.x;
    const int rows_per_seq = a.T + a.Tq;
    const int nn = a.n_nodes ? min(max(a.n_nodes[b], 0), a.T) : a.T;
    int32_t *path = a.accept_path + (size_t)b * (a.D_max + 1);
    for (int d = tid; d <= a.D_max; d += kAqThreads) path[d] = d == 0 && nn >= 1 ? 0 : -1;
    if (nn < 1) {
        if (tid == 0) { a.accept_len[b] = 0; a.bonus[b] = -1; }
        return;
    }
    if (tid < kWave) {
        const bool live = tid < nn;
        s.par[tid] = live ? a.parents[(size_t)b * a.T + tid] : -2;
        s.tok[tid] = live ? a.tokens[(size_t)b * a.T + tid] : -1;
        s.qrow[tid] = !live ? -1 : a.q_rows ? a.q_rows[(size_t)b * a.T + tid] : tid;
        s.uni[tid] = tid <= a.T ? a.uniforms[(size_t)b * (a.T + 1) + tid] : 0.f;
        if (tid == 0) { s.uni[kWave] = a.T == kWave ? a.uniforms[(size_t)b * (a.T + 1) + kWave] : 0.f; s.cur = 0; s.len = 0; }
    }
    __syncthreads();

    for (;;) {                                                       // one iteration per visited node; at most T of them
        const int cur = s.cur, len = s.len;
        const int prow_id = b * rows_per_seq + cur;
        const float *prow = a.target + ((size_t)b * a.T + cur) * a.V;
        const float pm = a.row_m[prow_id];
        const double pinv_l = 1.0 / a.row_l[prow_id];
        // ---- children of cur (ascending node index) and, for each, p(token) and q(token)
        if (w == 0) {
            const int x = s.tok[lane], qr = s.qrow[lane];
            const bool kid = lane > cur && lane < nn && s.par[lane] == cur && len < a.D_max && x >= 0 && x < a.V && qr >= 0 && qr < a.Tq;
            if (kid) {
                const int qid = b * rows_per_seq + a.T + qr;
                s.px[lane] = exp_rel(prow[x], pm, a.inv_t) * pinv_l;
                s.qx[lane] = exp_rel(a.draft[((size_t)b * a.Tq + qr) * a.V + x], a.row_m[qid], a.inv_td) / a.row_l[qid];
            }
            const unsigned long long kids = __ballot(kid);
            if (lane == 0) { s.kids = kids; s.W = 1.0; s.have_u = 0; s.next = -1; }
        }
        __syncthreads();
        // ---- Eq. 1 child by child; Eq. 2 after every rejection
        while (s.kids != 0 && s.next < 0 && s.W > 0.0) {
            const int c = __ffsll((long long)s.kids) - 1;
            const double W = s.W;
            const bool accept = (double)s.uni[c] * W * s.qx[c] < s.px[c];
            __syncthreads();                                         // everyone has read the state of this test
            if (accept) {
                if (tid == 0) s.next = c;
            } else {
                const int qr = s.qrow[c], qid = b * rows_per_seq + a.T + qr;
                const double total = residual_pass<VEC4>(a, s, b, s.have_u ? nullptr : prow, pm, pinv_l,
                                                         a.draft + ((size_t)b * a.Tq + qr) * a.V, a.row_m[qid], 1.0 / a.row_l[qid],
                                                         W, 0, a.V);
                // the residual at the tokens of the children still to be tried (written by this workgroup)
                const unsigned long long rest = s.kids & ~(1ull << c);
                if (w == 0 && ((rest >> lane) & 1)) s.px[lane] = (double)a.ubuf[(size_t)b * a.V + s.tok[lane]];
                if (tid == 0) { s.kids = rest; s.W = total; s.have_u = 1; }
            }
            __syncthreads();
        }
        if (s.next >= 0) {
            if (tid == 0) {
                const int c = s.next;
                s.cur = c;
                s.len = len + 1;
                path[len + 1] = c;
            }
            __syncthreads();
            continue;
        }
        // ---- bonus token from the residual (or from p itself when nothing was rejected, or when
        // the residual vanished)
        const bool use_u = s.have_u && s.W > 0.0;
        int lo = 0, hi = a.V;
        double before0 = 0.0, W = s.W;
        __syncthreads();
        if (!use_u) {
            // find the 16384-token chunk from the row's partials, then make u = p on that chunk only
            W = 1.0;
            const double target = (double)s.uni[a.T] * W;
            if (w == 0) {
                double mass = 0.0;
                if (lane < a.nchunks) {
                    const float mc = a.part_m[(size_t)prow_id * a.nchunks + lane];
                    if (mc > -INFINITY) mass = a.part_l[(size_t)prow_id * a.nchunks + lane] * exp(((double)mc - (double)pm) * a.inv_t) * pinv_l;
                }
                const double incl = wave_scan_f64(mass);
                const uint64_t cross = __ballot(lane < a.nchunks && incl > target);
                const uint64_t has = __ballot(mass > 0.0);
                const int ch = cross ? __ffsll((long long)cross) - 1 : (has ? 63 - __clzll((long long)has) : 0);
                const double bef = readlane_f64(incl - mass, ch);
                if (lane == 0) { s.gran = ch; s.before = bef; }
            }
            __syncthreads();
            lo = s.gran * kAqChunk;
            hi = min(a.V, lo + kAqChunk);
            before0 = s.before;
            residual_pass<VEC4>(a, s, b, prow, pm, pinv_l, nullptr, 0.f, 0.0, 0.0, lo, hi);
        }
        if (w == 0) {
            const double target = (double)s.uni[a.T] * W;
            const int pick = pick_token<VEC4>(a, s, b, before0, target, lo, hi);
            if (lane == 0) {
                a.bonus[b] = pick;
                a.accept_len[b] = len;
            }
        }
        return;
    }
}

}  // namespace radar

using namespace radar;

static int aq_chunks(int V) { return (V + kAqChunk - 1) / kAqChunk; }

extern "C" size_t radar_verify_accept_q_workspace_bytes(const radar_accept_q_desc *d) {
    if (!d || d->B < 1 || d->T_max < 1 || d->Tq < 1 || d->V < 1) return 0;
    const size_t rows = (size_t)d->B * ((size_t)d->T_max + d->Tq), nch = aq_chunks(d->V);
    size_t bytes = (rows * kAqCounterStride * sizeof(unsigned int) + 255) & ~size_t(255);
    bytes += (rows * nch * sizeof(double) + 255) & ~size_t(255);
    bytes += (rows * nch * sizeof(float) + 255) & ~size_t(255);
    bytes += (rows * sizeof(double) + 255) & ~size_t(255);
    bytes += (rows * sizeof(float) + 255) & ~size_t(255);
    bytes += ((size_t)d->B * d->V * sizeof(float) + 255) & ~size_t(255);
    return bytes;
}

extern "C" radar_status radar_verify_accept_q(const float *target_logits, const float *draft_logits, const int32_t *q_rows,
                                              const int32_t *draft_tokens, const int32_t *parents, const int32_t *n_nodes,
                                              const float *uniforms, int32_t *accept_len, int32_t *accept_path,
                                              int32_t *bonus_token, const radar_accept_q_desc *d, void *workspace,
                                              size_t workspace_bytes, void *stream) {
    if (!d || !target_logits || !draft_logits || !draft_tokens || !parents || !uniforms || !accept_len || !accept_path ||
        !bonus_token || !workspace)
        return RADAR_INVALID_ARG;
    if (d->B < 1 || d->T_max < 1 || d->Tq < 1 || d->V < 1 || d->D_max < 0 || !(d->temperature > 0.f) ||
        !(d->draft_temperature > 0.f))
        return RADAR_INVALID_ARG;
    if (!q_rows && d->Tq != d->T_max) return RADAR_INVALID_ARG;
    if (d->T_max > RADAR_T_MAX || d->D_max >= RADAR_T_MAX || aq_chunks(d->V) > kAqMaxChunks) return RADAR_UNSUPPORTED_SHAPE;
    if ((int64_t)d->B * ((int64_t)d->T_max + d->Tq) > 65535) return RADAR_UNSUPPORTED_SHAPE;      // rows ride on gridDim.y
    if (workspace_bytes < radar_verify_accept_q_workspace_bytes(d)) return RADAR_WORKSPACE_TOO_SMALL;
    if (((uintptr_t)workspace & 255) != 0) return RADAR_INVALID_ARG;

    AqArgs a{};
    a.target = target_logits; a.draft = draft_logits; a.q_rows = q_rows;
    a.tokens = draft_tokens; a.parents = parents; a.n_nodes = n_nodes; a.uniforms = uniforms;
    a.accept_len = accept_len; a.accept_path = accept_path; a.bonus = bonus_token;
    a.B = d->B; a.T = d->T_max; a.Tq = d->Tq; a.V = d->V; a.D_max = d->D_max; a.nchunks = aq_chunks(d->V);
    a.inv_t = 1.0 / (double)d->temperature; a.inv_td = 1.0 / (double)d->draft_temperature;
    const size_t rows = (size_t)d->B * ((size_t)d->T_max + d->Tq), nch = a.nchunks;
    char *ws = static_cast<char *>(workspace);
    auto take = [&](size_t bytes) { char *p = ws; ws += (bytes + 255) & ~size_t(255); return p; };
    a.counters = reinterpret_cast<unsigned int *>(take(rows * kAqCounterStride * sizeof(unsigned int)));
    a.part_l = reinterpret_cast<double *>(take(rows * nch * sizeof(double)));
    a.part_m = reinterpret_cast<float *>(take(rows * nch * sizeof(float)));
    a.row_l = reinterpret_cast<double *>(take(rows * sizeof(double)));
    a.row_m = reinterpret_cast<float *>(take(rows * sizeof(float)));
    a.ubuf = reinterpret_cast<float *>(take((size_t)d->B * d->V * sizeof(float)));

    const bool vec4 = (d->V % 4 == 0) && (((uintptr_t)target_logits & 15) == 0) && (((uintptr_t)draft_logits & 15) == 0);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 g1((unsigned)a.nchunks, (unsigned)rows), g2((unsigned)d->B), block(kAqThreads);
    hipError_t e = vec4 ? launch("accept_q_stats", accept_q_stats_kernel<true>, g1, block, 0, st, a)
                        : launch("accept_q_stats", accept_q_stats_kernel<false>, g1, block, 0, st, a);
    if (e != hipSuccess) return RADAR_HIP_ERROR;
    e = vec4 ? launch("accept_q_walk", accept_q_walk_kernel<true>, g2, block, 0, st, a)
             : launch("accept_q_walk", accept_q_walk_kernel<false>, g2, block, 0, st, a);
    return e == hipSuccess ? RADAR_OK : RADAR_HIP_ERROR;
}
