// radar_verify_accept_q: verification with draft distributions (Sec. 3, Eq. 1-2), for trees
// whose tokens were drawn from the draft model's distributions.
//
// Two launches, or three when the walk is shared.  (1) Row statistics, spread over the whole chip: one workgroup per 16384
// logits of every target row and every draft row streams its chunk once and leaves (max, sum
// of exp) partials; the workgroup that completes a row (arrival ticket) merges them into the
// row's normaliser.  This is the HBM-bound part: it reads every logit once.  (2) The walk, one
// workgroup per sequence: sequential by nature (Eq. 1 is applied child by child, Eq. 2 changes
// the distribution every later test sees).  Every rejection is one vocabulary-wide pass of the
// workgroup that turns the unnormalised residual u into max(0, u - W q) (W = sum u), keeps it
// in a workspace row and leaves sums per 256 tokens in LDS; the bonus token is then found from
// those sums without another pass.  A walk that ends without a rejection draws the bonus from
// the row's chunk partials and one 16384-token chunk.  Where the chip has room the walk of a
// sequence is shared by up to 32 workgroups instead (further down), followed by a launch that
// redoes, with one workgroup, any sequence whose workgroups could not meet.
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
    // walk by several workgroups per sequence
    unsigned int *co_ctl;       // [B][32]: arrival counter, leave counter, abort flag (each on its own 32 bytes)
    double *co_psum;            // [B][2][32] slice sums of the last two meetings
    float *co_sib;              // [B][2][64] residual at the tokens of untried children
    int co_R;                   // float4 per lane
    unsigned int co_spin_limit; // polls of the arrival counter before a workgroup gives up
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

// The whole walk of sequence b by one workgroup (every thread calls it).
template <bool VEC4>
__device__ __forceinline__ void walk_single(const AqArgs &a, AqSmem &s, int b) {
    const int tid = threadIdx.x, lane = lane_id(), w = wave_id();
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

// only_marked: the launch that follows the shared walk; it redoes the sequences that walk marked
// (and clears the mark), and leaves the others alone.
template <bool VEC4>
__global__ __launch_bounds__(kAqThreads) void accept_q_walk_kernel(AqArgs a, int only_marked) {
    __shared__ AqSmem s;
    if (only_marked) {
        unsigned int *mark = &a.co_ctl[(size_t)blockIdx.x * 32 + 24];
        const unsigned int m = *mark;                     // written by the previous launch
        __syncthreads();                                  // everyone has read it
        if (m == 0u) return;
        if (threadIdx.x == 0) *mark = 0u;
    }
    walk_single<VEC4>(a, s, blockIdx.x);
}

// ------------------------------------------------------------------- walk by several workgroups
// G workgroups per sequence; workgroup g keeps the residual of tokens [g * slice, (g + 1) * slice) in
// registers (R float4 per lane) for as long as the walk stays at a node, so a rejection costs each
// of them one 16-byte load per float4 (its part of the draft row) instead of a vocabulary-wide pass
// by a single CU.  Every workgroup takes the same decisions from the same numbers: after a
// rejection each publishes the sum of its slice and the residual at the tokens of the children
// still to be tried, all meet at an arrival counter, and all add the G sums in the same order.
// The wait at the counter is bounded: a workgroup that gives up (the workgroups of a sequence
// were not all resident, which the host avoids by keeping G * B within the chip) raises the
// sequence's abort flag, everyone leaves, and the last one to leave redoes the sequence alone.
constexpr int kCoG = 32;                     // most workgroups per sequence
constexpr int kCoR = 4;                      // most float4 per lane (V <= 32 * 4 * 4096; larger vocabularies walk with one workgroup)
constexpr int kCoCtl = 32;                   // uints per sequence in the control block: arrive, leave, abort, redo mark at 0, 8, 16, 24

struct CoSmem {
    double wred[kAqWaves];
    double psum[kCoG];
    double px[kWave], qx[kWave];
    int par[kWave], tok[kWave], qrow[kWave];
    float uni[kWave + 1];
    double W;
    unsigned long long kids;
    int wlast[kAqWaves];
    int cur, len, next, aborted, pick;
};

template <bool VEC4>
__global__ __launch_bounds__(kAqThreads) void accept_q_coop_kernel(AqArgs a) {
    __shared__ CoSmem s;
    const int tid = threadIdx.x, lane = lane_id(), w = wave_id();
    const int g = blockIdx.x, G = gridDim.x, b = blockIdx.y;
    const int R = a.co_R, slice = R * kAqThreads * 4, lo = g * slice;
    const int rows_per_seq = a.T + a.Tq;
    const int nn = a.n_nodes ? min(max(a.n_nodes[b], 0), a.T) : a.T;
    unsigned int *ctl = a.co_ctl + (size_t)b * kCoCtl;
    double *psum_g = a.co_psum + (size_t)b * 2 * kCoG;    // [2][kCoG]
    float *sib_g = a.co_sib + (size_t)b * 2 * kWave;      // [2][64]
    int32_t *path = a.accept_path + (size_t)b * (a.D_max + 1);
    unsigned int nsync = 0;

    // leave: every workgroup of the sequence ends here.  The last one to arrive clears the control
    // block for the next call and learns whether anybody gave up on the way (all their stores are
    // complete by then); if so it marks the sequence for the launch that follows, in which a single
    // workgroup redoes it.  (Calling that code from here would give this kernel a stack, which
    // costs every launch 8 us.)
    auto leave = [&]() {
        __syncthreads();
        if (tid == 0) {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            const unsigned int before = __hip_atomic_fetch_add(&ctl[8], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (before == (unsigned int)(G - 1)) {
                store_shared_result(&ctl[24], load_shared_result(&ctl[16]));
                store_shared_result(&ctl[0], 0u);
                store_shared_result(&ctl[8], 0u);
                store_shared_result(&ctl[16], 0u);
            }
        }
    };
    // meet: publish this workgroup's sum (and whatever the caller stored before), wait for all G,
    // return the total.  Sets s.aborted when the wait gave up or somebody else did.
    auto meet = [&](double mine) -> double {
        const int par = nsync & 1;
        ++nsync;
        if (tid == 0) store_shared_result(&psum_g[par * kCoG + g], mine);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (tid == 0) {
            __hip_atomic_fetch_add(&ctl[0], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const unsigned int want = nsync * (unsigned int)G;
            unsigned int spins = 0;
            int bad = 0;
            while (__hip_atomic_load(&ctl[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < want) {
                if (++spins > a.co_spin_limit || load_shared_result(&ctl[16]) != 0u) { bad = 1; break; }
                __builtin_amdgcn_s_sleep(4);
            }
            if (bad) store_shared_result(&ctl[16], 1u);
            s.aborted = bad;
        }
        __syncthreads();
        if (s.aborted) return 0.0;
        if (tid < G) s.psum[tid] = load_shared_result(&psum_g[par * kCoG + tid]);
        __syncthreads();
        double t = 0.0;
        for (int i = 0; i < G; ++i) t += s.psum[i];
        return t;
    };

    if (tid == 0) s.aborted = load_shared_result(&ctl[16]) != 0u;   // somebody gave up before this workgroup even started
    if (tid < kWave) {
        const bool live = tid < nn;
        s.par[tid] = live ? a.parents[(size_t)b * a.T + tid] : -2;
        s.tok[tid] = live ? a.tokens[(size_t)b * a.T + tid] : -1;
        s.qrow[tid] = !live ? -1 : a.q_rows ? a.q_rows[(size_t)b * a.T + tid] : tid;
        s.uni[tid] = tid <= a.T ? a.uniforms[(size_t)b * (a.T + 1) + tid] : 0.f;
        if (tid == 0) { s.uni[kWave] = a.T == kWave ? a.uniforms[(size_t)b * (a.T + 1) + kWave] : 0.f; s.cur = 0; s.len = 0; }
    }
    // Outputs are written through (agent-scope stores): should the sequence be redone by another
    // workgroup, on another die, no older copy of them may linger in this die's L2 to be written back later.
    if (g == 0) for (int d = tid; d <= a.D_max; d += kAqThreads) store_shared_result(&path[d], d == 0 && nn >= 1 ? 0 : -1);
    __syncthreads();
    bool fall_back = s.aborted != 0;
    if (nn < 1) {
        if (g == 0 && tid == 0) { store_shared_result(&a.accept_len[b], 0); store_shared_result(&a.bonus[b], -1); }
        leave();                                          // nobody meets on this path, so nobody can have given up
        return;
    }

    const float it_f = (float)a.inv_t, itd_f = (float)a.inv_td;
    float u4[kCoR][4];
    // this lane's tokens: float4 r covers lo + (r * 1024 + tid) * 4 .. + 3
    auto load_row = [&](const float *row, float m, float inv_l, float inv_temp, float (&out)[kCoR][4]) {
#pragma unroll
        for (int r = 0; r < kCoR; ++r) {
            if (r < R) {
                const int i0 = lo + (r * kAqThreads + tid) * 4;
                float x[4];
                if (VEC4) {
                    const float4 v = *reinterpret_cast<const float4 *>(row + (i0 < a.V ? i0 : 0));
                    x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) x[j] = row[min(i0 + j, a.V - 1)];
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) out[r][j] = (i0 + j < a.V) ? exp_rel_f32(x[j], m, inv_temp) * inv_l : 0.f;
            }
        }
    };
    auto my_sum = [&]() -> double {
        double t = 0.0;
#pragma unroll
        for (int r = 0; r < kCoR; ++r)
            if (r < R) t += ((double)u4[r][0] + (double)u4[r][1]) + ((double)u4[r][2] + (double)u4[r][3]);
        return block_sum_f64(t, s.wred);
    };

    while (!fall_back) {                                  // one iteration per visited node
        const int cur = s.cur, len = s.len;
        const int prow_id = b * rows_per_seq + cur;
        const float *prow = a.target + ((size_t)b * a.T + cur) * a.V;
        const float pm = a.row_m[prow_id];
        const double pinv_l = 1.0 / a.row_l[prow_id];
        if (w == 0) {
            const int x = s.tok[lane], qr = s.qrow[lane];
            const bool kid = lane > cur && lane < nn && s.par[lane] == cur && len < a.D_max && x >= 0 && x < a.V && qr >= 0 && qr < a.Tq;
            if (kid) {
                const int qid = b * rows_per_seq + a.T + qr;
                s.px[lane] = exp_rel(prow[x], pm, a.inv_t) * pinv_l;
                s.qx[lane] = exp_rel(a.draft[((size_t)b * a.Tq + qr) * a.V + x], a.row_m[qid], a.inv_td) / a.row_l[qid];
            }
            const unsigned long long kids = __ballot(kid);
            if (lane == 0) { s.kids = kids; s.W = 1.0; s.next = -1; }
        }
        load_row(prow, pm, (float)pinv_l, it_f, u4);      // u = p_cur on this workgroup's slice
        __syncthreads();
        bool rejected_here = false;
        while (s.kids != 0 && s.next < 0 && s.W > 0.0) {
            const int c = __ffsll((long long)s.kids) - 1;
            const double W = s.W;
            const bool accept = (double)s.uni[c] * W * s.qx[c] < s.px[c];
            __syncthreads();
            if (accept) {
                if (tid == 0) s.next = c;
            } else {
                const int qr = s.qrow[c], qid = b * rows_per_seq + a.T + qr;
                float q4[kCoR][4];
                load_row(a.draft + ((size_t)b * a.Tq + qr) * a.V, a.row_m[qid], (float)(1.0 / a.row_l[qid]), itd_f, q4);
                const float W_f = (float)W;
#pragma unroll
                for (int r = 0; r < kCoR; ++r)
                    if (r < R) {
#pragma unroll
                        for (int j = 0; j < 4; ++j) u4[r][j] = fmaxf(0.f, fmaf(-W_f, q4[r][j], u4[r][j]));
                    }
                // the residual at the tokens of the children still to be tried: their owners publish it
                const unsigned long long rest = s.kids & ~(1ull << c);
                const int par = nsync & 1;
                for (unsigned long long m = rest; m != 0; m &= m - 1) {
                    const int c2 = __ffsll((long long)m) - 1;
                    const int off = s.tok[c2] - lo;
                    if (off >= 0 && off < slice && ((off >> 2) & (kAqThreads - 1)) == tid) {
                        const int r2 = off >> 12, j2 = off & 3;                 // float4 index, element
                        float val = 0.f;
#pragma unroll
                        for (int r = 0; r < kCoR; ++r)
#pragma unroll
                            for (int j = 0; j < 4; ++j)
                                if (r == r2 && j == j2) val = u4[r][j];
                        store_shared_result(&sib_g[par * kWave + c2], val);
                    }
                }
                const double total = meet(my_sum());
                if (s.aborted) break;
                if (w == 0 && ((rest >> lane) & 1)) s.px[lane] = (double)load_shared_result(&sib_g[par * kWave + lane]);
                if (tid == 0) { s.kids = rest; s.W = total; }
                rejected_here = true;
            }
            __syncthreads();
        }
        if (s.aborted) { fall_back = true; break; }
        if (s.next >= 0) {
            if (tid == 0) {
                const int c = s.next;
                s.cur = c;
                s.len = len + 1;
                if (g == 0) store_shared_result(&path[len + 1], c);
            }
            __syncthreads();
            continue;
        }
        // ---- bonus token.  Everybody needs the G slice sums of what the bonus is drawn from.
        double W = s.W;
        __syncthreads();
        if (!rejected_here || !(W > 0.0)) {               // nothing rejected here, or the residual vanished: draw from p_cur
            if (rejected_here) load_row(prow, pm, (float)pinv_l, it_f, u4);
            W = meet(my_sum());
            if (s.aborted) { fall_back = true; break; }
        }
        // (after a rejection s.psum still holds the sums of the last meeting)
        const double target = (double)s.uni[a.T] * W;
        int owner = -1, last_pos = -1;
        double before = 0.0, acc = 0.0;
        for (int i = 0; i < G; ++i) {
            if (s.psum[i] > 0.0) last_pos = i;
            if (owner < 0 && acc + s.psum[i] > target) { owner = i; before = acc; }
            acc += s.psum[i];
        }
        const bool take_last = owner < 0;                 // rounding: the sums never exceed the target
        if (take_last) owner = last_pos;
        if (g == 0 && tid == 0) store_shared_result(&a.accept_len[b], len);
        if (owner < 0) { if (g == 0 && tid == 0) store_shared_result(&a.bonus[b], -1); break; }
        if (g == owner) {
            // token order inside the slice: float4 row r, then thread, then element
            if (tid == 0) s.pick = 0x7fffffff;
            __syncthreads();
            double run = before;
            int lastp = -1;
            for (int r = 0; r < R; ++r) {                 // uniform; the row is picked by comparison (r is not a constant here)
                float v[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int rr = 0; rr < kCoR; ++rr)
                    if (rr == r) { v[0] = u4[rr][0]; v[1] = u4[rr][1]; v[2] = u4[rr][2]; v[3] = u4[rr][3]; }
                const double lsum = ((double)v[0] + (double)v[1]) + ((double)v[2] + (double)v[3]);
                const double linc = wave_scan_f64(lsum);
                if (lane == kWave - 1) s.wred[w] = linc;
                __syncthreads();
                double wbefore = run, rtot = 0.0;
                for (int i = 0; i < kAqWaves; ++i) {
                    if (i < w) wbefore += s.wred[i];
                    rtot += s.wred[i];
                }
                const int i0 = lo + (r * kAqThreads + tid) * 4;
                double accl = wbefore + linc - lsum;
                int pick = -1;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    if (v[j] > 0.f) lastp = i0 + j;
                    accl += (double)v[j];
                    if (pick < 0 && accl > target) pick = i0 + j;
                }
                if (pick >= 0 && !take_last) atomicMin(&s.pick, pick);
                run += rtot;
                __syncthreads();
            }
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) lastp = max(lastp, __shfl_xor(lastp, off));
            if (lane == 0) s.wlast[w] = lastp;
            __syncthreads();
            if (tid == 0) {
                int lp = -1;
                for (int i = 0; i < kAqWaves; ++i) lp = max(lp, s.wlast[i]);
                store_shared_result(&a.bonus[b], s.pick != 0x7fffffff ? s.pick : lp);
            }
        }
        break;
    }
    (void)fall_back;
    leave();
}

}  // namespace radar

using namespace radar;

static int aq_chunks(int V) { return (V + kAqChunk - 1) / kAqChunk; }

// How many 1024-lane workgroups of the shared walk the current device can hold at once: the
// occupancy the runtime reports for the kernel times the number of CUs (queried once; 0 if the
// queries fail, which selects the single-workgroup walk).
static int aq_resident_capacity() {
    static const int capacity = [] {
        int dev = 0, per_cu = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void *>(&accept_q_coop_kernel<true>),
                                                         kAqThreads, 0) != hipSuccess)
            return 0;
        return per_cu * prop.multiProcessorCount;
    }();
    return capacity;
}

// Workgroups per sequence (G) and float4 per lane (R) of the walk; G = 1 means the single-workgroup
// walk.  The G * B workgroups of the shared walk meet at arrival counters, which only makes progress
// while all of them are resident, so their number stays within what the device holds at once (on a
// GPU that other work shares, the bounded wait turns a missing workgroup into the fall-back).
static void aq_coop_plan(const radar_accept_q_desc *d, int *G, int *R) {
    *G = 1; *R = 1;
    const int cap = aq_resident_capacity();
    if (d->walk_spin_limit < 0 || cap < 2 || d->B > cap / 2) return;
    const int gcap = cap / d->B < kCoG ? cap / d->B : kCoG;
    const int per_wg = kAqThreads * 4;
    int r = ((d->V + per_wg - 1) / per_wg + gcap - 1) / gcap;              // float4 per lane needed with gcap workgroups
    if (r > kCoR) return;
    if (r < 1) r = 1;
    const int g = (d->V + per_wg * r - 1) / (per_wg * r);
    if (g < 2) return;                                                    // one workgroup would cover it anyway
    *G = g; *R = r;
}

extern "C" size_t radar_verify_accept_q_workspace_bytes(const radar_accept_q_desc *d) {
    if (!d || d->B < 1 || d->T_max < 1 || d->Tq < 1 || d->V < 1) return 0;
    const size_t rows = (size_t)d->B * ((size_t)d->T_max + d->Tq), nch = aq_chunks(d->V);
    size_t bytes = (rows * kAqCounterStride * sizeof(unsigned int) + 255) & ~size_t(255);
    bytes += (rows * nch * sizeof(double) + 255) & ~size_t(255);
    bytes += (rows * nch * sizeof(float) + 255) & ~size_t(255);
    bytes += (rows * sizeof(double) + 255) & ~size_t(255);
    bytes += (rows * sizeof(float) + 255) & ~size_t(255);
    bytes += ((size_t)d->B * d->V * sizeof(float) + 255) & ~size_t(255);
    bytes += ((size_t)d->B * kCoCtl * sizeof(unsigned int) + 255) & ~size_t(255);
    bytes += ((size_t)d->B * 2 * kCoG * sizeof(double) + 255) & ~size_t(255);
    bytes += ((size_t)d->B * 2 * kWave * sizeof(float) + 255) & ~size_t(255);
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
    a.co_ctl = reinterpret_cast<unsigned int *>(take((size_t)d->B * kCoCtl * sizeof(unsigned int)));
    a.co_psum = reinterpret_cast<double *>(take((size_t)d->B * 2 * kCoG * sizeof(double)));
    a.co_sib = reinterpret_cast<float *>(take((size_t)d->B * 2 * kWave * sizeof(float)));
    int G = 1, R = 1;
    aq_coop_plan(d, &G, &R);
    a.co_R = R;
    // default: 256 polls of about 0.4 us (an atomic load and a short sleep): the workgroups of a walk reach a
    // meeting within microseconds of each other, so 100 us without progress means one of them is not running
    a.co_spin_limit = d->walk_spin_limit > 0 ? (unsigned int)d->walk_spin_limit : 256u;

    const bool vec4 = (d->V % 4 == 0) && (((uintptr_t)target_logits & 15) == 0) && (((uintptr_t)draft_logits & 15) == 0);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 g1((unsigned)a.nchunks, (unsigned)rows), g2((unsigned)d->B), block(kAqThreads);
    hipError_t e = vec4 ? launch("accept_q_stats", accept_q_stats_kernel<true>, g1, block, 0, st, a)
                        : launch("accept_q_stats", accept_q_stats_kernel<false>, g1, block, 0, st, a);
    if (e != hipSuccess) return RADAR_HIP_ERROR;
    if (G > 1) {
        const dim3 g3((unsigned)G, (unsigned)d->B);
        e = vec4 ? launch("accept_q_walk_shared", accept_q_coop_kernel<true>, g3, block, 0, st, a)
                 : launch("accept_q_walk_shared", accept_q_coop_kernel<false>, g3, block, 0, st, a);
        if (e != hipSuccess) return RADAR_HIP_ERROR;
        e = vec4 ? launch("accept_q_walk_redo", accept_q_walk_kernel<true>, g2, block, 0, st, a, 1)
                 : launch("accept_q_walk_redo", accept_q_walk_kernel<false>, g2, block, 0, st, a, 1);
    } else {
        e = vec4 ? launch("accept_q_walk", accept_q_walk_kernel<true>, g2, block, 0, st, a, 0)
                 : launch("accept_q_walk", accept_q_walk_kernel<false>, g2, block, 0, st, a, 0);
    }
    return e == hipSuccess ? RADAR_OK : RADAR_HIP_ERROR;
}
