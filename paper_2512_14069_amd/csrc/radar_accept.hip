// Verification walk of RADAR's speculative-sampling cycle (Sec. 3, Eq. 1-2; tree
// form per Sec. 4.3, Eq. 11-13) as one HIP launch for gfx950.
//
// Phase 1, grid (blocks of the vocabulary, tree rows, sequences): one streaming
// read of the target logits (T*V*4 bytes per sequence).  Every wavefront owns
// 1024 consecutive logits and leaves their arg-max key and, in sampling mode,
// (max, sum exp) of the temperature-scaled values; nothing is combined inside a
// workgroup.  Phase 2: the workgroup whose arrival ticket is the last of its ROW
// merges that row's partials in one wavefront and turns the sums into masses
// relative to the row maximum.  Phase 3: the workgroup whose ticket is the last
// of its SEQUENCE walks the tree in one wavefront, one lane per node: sibling
// sets come from ballots, everything the walk compares sits in registers and is
// passed between lanes by lane reads or DPP scans.  The residual draw scans the
// 1024-logit masses across lanes and then re-reads one such block (4 KB).
#include "radar_device.h"
#include "radar_host.h"

namespace radar {

constexpr int kAccThreads = 256;
constexpr int kAccWaves = kAccThreads / kWave;
constexpr int kAccEPT = 16;
constexpr int kAccSub = kWave * kAccEPT;              // 1024 logits per wavefront = one partial
constexpr int kAccChunk = kAccThreads * kAccEPT;      // logits per workgroup
constexpr int kAccMaxSubs = 4096;                     // V <= 4,194,304
constexpr int kAccCounterStride = 16;   // counters 64 B apart (same-line fetch-adds serialise)
constexpr float kAccLog2e = 1.4426950408889634f;
constexpr int kAccDistribution = 2;     // internal mode: acceptance-length distribution instead of a walk

struct AcceptArgs {
    const float *logits;
    const int32_t *tokens;
    const int32_t *parents;
    const int32_t *n_nodes;
    const float *uniforms;
    int32_t *accept_len;
    int32_t *accept_path;
    int32_t *bonus;
    double *dist;               // mode kAccDistribution: [B][D_max+1]
    int B, T, V, D_max, mode, nwg, nsub;   // nwg workgroups and nsub 1024-logit blocks per row
    int exact_scale;            // 1/temperature is exactly representable in fp32
    float inv_temp_f;
    double inv_temp;
    unsigned int *counters;     // [(b*T + r) * stride] workgroups of a row, [(B*T + b) * stride] rows of a sequence
    uint64_t *row_key;          // [B][T] arg-max key of the row
    double *row_L;              // [B][T] sum of exp(y - row_M), y = logit / temperature
    float *row_M;               // [B][T]
    uint64_t *part_key;         // [B][T][nsub] arg-max key of the block
    double *part_l;             // [B][T][nsub] sum of exp(y - part_m) over the block; once the row is merged:
                                //              sum of exp(y - row_M) over the block
    float *part_m;              // [B][T][nsub] reference maximum of the block
};

struct AcceptSmem {
    unsigned int ticket;
    double row_lse[RADAR_T_MAX];
    int row_arg[RADAR_T_MAX];
    double rej_e[RADAR_T_MAX];                    // what each rejected token carries, and the block it lies in
    int rej_sub[RADAR_T_MAX];
    unsigned int rej_bits[kWave];                 // pass (b): which of a lane's 16 tokens are rejected ones
    unsigned char seen[4096];                     // sibling tokens, hashed
};

// exp(x / temperature - ref) for one logit, as a double.  The exponent difference is rounded to
// fp32 once (an fp32 FMA does that when the scale is exact in fp32, else it is formed in fp64);
// the exponential itself is the fp32 one.  The sums that use it are kept in fp64.
__device__ __forceinline__ double scaled_exp(float x, const AcceptArgs &a, float ref) {
    if (a.exact_scale) return (double)__builtin_amdgcn_exp2f(__builtin_fmaf(x, a.inv_temp_f, -ref) * kAccLog2e);
    return (double)expf((float)((double)x * a.inv_temp - (double)ref));
}

// 16 logits per lane of one 1024-logit block: lane l takes [16 * l, 16 * l + 16) when CONTIG (pass
// (b) needs token order inside a lane), else 4 x (64 lanes x 16 B) interleaved (widest requests).
template <bool VEC4, bool CONTIG>
__device__ __forceinline__ void load_block(const float *row, int i_block, int V, float (&x)[kAccEPT], int (&first)[kAccEPT / 4]) {
    const int lane = lane_id();
    float4 raw[kAccEPT / 4];
#pragma unroll
    for (int g = 0; g < kAccEPT / 4; ++g) {
        const int i = i_block + (CONTIG ? lane * kAccEPT + 4 * g : g * (kWave * 4) + lane * 4);
        first[g] = i;
        // branch-free: out-of-range lanes read a valid address and are masked afterwards
        if (VEC4) {
            raw[g] = *reinterpret_cast<const float4 *>(row + (i < V ? i : 0));
        } else {
            raw[g].x = row[min(i + 0, V - 1)];
            raw[g].y = row[min(i + 1, V - 1)];
            raw[g].z = row[min(i + 2, V - 1)];
            raw[g].w = row[min(i + 3, V - 1)];
        }
    }
    const bool tail = i_block + kAccSub > V;                  // wave-uniform: only a row's last block needs masking
#pragma unroll
    for (int g = 0; g < kAccEPT / 4; ++g) {
        const float v[4] = {raw[g].x, raw[g].y, raw[g].z, raw[g].w};
        if (tail) {
#pragma unroll
            for (int j = 0; j < 4; ++j) x[4 * g + j] = (first[g] + j < V) ? v[j] : -INFINITY;
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) x[4 * g + j] = v[j];
        }
    }
}

template <bool VEC4>
__global__ __launch_bounds__(kAccThreads) void accept_kernel(AcceptArgs a) {
    __shared__ AcceptSmem s;
    const int tid = threadIdx.x, lane = lane_id(), w = wave_id();
    const int r = blockIdx.y, b = blockIdx.z;
    int nn = a.n_nodes ? a.n_nodes[b] : a.T;
    nn = max(1, min(nn, a.T));
    if (r >= nn) return;
    const bool sampling = (a.mode != RADAR_ACCEPT_GREEDY);      // row statistics are needed
    const float *row = a.logits + ((size_t)b * a.T + r) * a.V;
    const int sub = blockIdx.x * kAccWaves + w;              // this wavefront's 1024-logit block

    // ---------------- phase 1: per-wavefront arg-max (and scaled max / sum-exp)
    if (sub < a.nsub) {
        float x[kAccEPT];
        int first[kAccEPT / 4];
        load_block<VEC4, false>(row, sub * kAccSub, a.V, x, first);
        // Largest logit of the block first (lane, then wavefront); only the lanes that hold it look for
        // its position, lowest index first (-0.0 equals +0.0 here, as in the key order).
        float tmx = x[0];
#pragma unroll
        for (int e = 1; e < kAccEPT; ++e) tmx = fmaxf(tmx, x[e]);
        const float wmx = wave_max_f32(tmx);
        uint32_t bi = 0xffffffffu;
        if (tmx == wmx) {
#pragma unroll
            for (int e = kAccEPT - 1; e >= 0; --e) bi = (x[e] == wmx) ? uint32_t(first[e / 4] + (e & 3)) : bi;
        }
        bi = ~wave_max_u32(~bi);                                  // lowest index over the wavefront
        const uint64_t best = bi < (uint32_t)a.V ? make_key(wmx, bi) : 0;
        const size_t pslot = ((size_t)b * a.T + r) * a.nsub + sub;
        if (sampling) {
            // 1 / temperature > 0 and rounding is monotone, so the largest scaled logit is the scaled largest
            const float wm = wmx * a.inv_temp_f;
            double tl = 0.0;
            if (wm > -INFINITY) {
#pragma unroll
                for (int e = 0; e < kAccEPT; ++e) tl += scaled_exp(x[e], a, wm);
            }
            const double wl = wave_sum_f64(tl);
            if (lane == 0) {
                store_shared_result(&a.part_m[pslot], wm);
                store_shared_result(&a.part_l[pslot], wl);
            }
        }
        if (lane == 0) store_shared_result(&a.part_key[pslot], best);
    }
    unsigned int *row_counter = &a.counters[((size_t)b * a.T + r) * kAccCounterStride];
    if (publish_then_ticket(row_counter, &s.ticket) != (unsigned int)(a.nwg - 1)) return;
    if (w != 0) {                                            // one wavefront does the rest; the others only
        __syncthreads();                                     // take part in the next ticket's barriers
        __syncthreads();
        return;
    }

    // ---------------- phase 2: last workgroup of row r -- merge the row's partials.
    // What only the walk needs (lane c is tree node c) is fetched here, so that it has arrived by
    // the time the walk starts.
    int p = -1, t = -1;
    float xg = 0.f, uc = 0.f, ubonus = 0.f;
    bool tree_ok = false;
    {
        const int c = lane;
        if (c < nn) { p = a.parents[(size_t)b * a.T + c]; t = a.tokens[(size_t)b * a.T + c]; }
        tree_ok = (c > 0 && c < nn && p >= 0 && p < c);
        if (sampling) {
            if (a.uniforms) {                                // none in distribution mode
                const float *u = a.uniforms + (size_t)b * (a.T + 1);
                uc = u[min(c, a.T)];
                ubonus = u[a.T];
            }
            if (tree_ok && t >= 0 && t < a.V) xg = a.logits[((size_t)b * a.T + p) * a.V + t];
        }
        const size_t p0 = ((size_t)b * a.T + r) * a.nsub;
        // the first 128 partials (all of them up to V = 131072) are taken in one round trip
        uint64_t kb = 0;
        float m_[2];
        double l_[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int c0 = i * kWave + lane;
            const int cc = min(c0, a.nsub - 1);                  // branch-free: clamp, load, mask
            const uint64_t k2 = load_shared_result(&a.part_key[p0 + cc]);
            kb = max_u64(kb, c0 < a.nsub ? k2 : 0);
            m_[i] = -INFINITY; l_[i] = 0.0;
            if (sampling) {
                const float m2 = load_shared_result(&a.part_m[p0 + cc]);
                const double l2 = load_shared_result(&a.part_l[p0 + cc]);
                if (c0 < a.nsub) { m_[i] = m2; l_[i] = l2; }
            }
        }
        float mmax = fmaxf(m_[0], m_[1]);
        for (int c0 = 2 * kWave + lane; c0 < a.nsub; c0 += kWave) {
            kb = max_u64(kb, load_shared_result(&a.part_key[p0 + c0]));
            if (sampling) mmax = fmaxf(mmax, load_shared_result(&a.part_m[p0 + c0]));
        }
        kb = wave_max_u64(kb);
        const float M = wave_max_f32(mmax);
        double lsum = 0.0;
        if (sampling) {
            // each block's mass relative to the row maximum: summed for the row, and left in part_l
            // for the residual draw
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int c0 = i * kWave + lane;
                const double mass = m_[i] > -INFINITY ? l_[i] * exp((double)m_[i] - (double)M) : 0.0;
                if (c0 < a.nsub) store_shared_result(&a.part_l[p0 + c0], mass);
                lsum += mass;
            }
            for (int c0 = 2 * kWave + lane; c0 < a.nsub; c0 += kWave) {
                const float m2 = load_shared_result(&a.part_m[p0 + c0]);
                const double l2 = load_shared_result(&a.part_l[p0 + c0]);
                const double mass = m2 > -INFINITY ? l2 * exp((double)m2 - (double)M) : 0.0;
                store_shared_result(&a.part_l[p0 + c0], mass);
                lsum += mass;
            }
        }
        const double L = wave_sum_f64(lsum);
        if (lane == 0) {
            const size_t rs = (size_t)b * a.T + r;
            store_shared_result(&a.row_key[rs], kb);
            if (sampling) {
                store_shared_result(&a.row_M[rs], M);
                store_shared_result(&a.row_L[rs], L);
            }
            store_shared_result(row_counter, 0u);            // leave the row counter clean for the next call
        }
    }
    unsigned int *seq_counter = &a.counters[((size_t)a.B * a.T + b) * kAccCounterStride];
    if (publish_then_ticket(seq_counter, &s.ticket) != (unsigned int)(nn - 1)) return;
    if (lane == 0) store_shared_result(seq_counter, 0u);

    // ---------------- phase 3: last workgroup of sequence b, one wavefront
    const int c = lane;
    const size_t rs = (size_t)b * a.T + min(c, nn - 1);
    const int arg = (int)key_index(load_shared_result(&a.row_key[rs]));
    float Mc = 0.f;
    double Lc = 1.0;
    if (sampling) {
        Mc = load_shared_result(&a.row_M[rs]);
        Lc = load_shared_result(&a.row_L[rs]);
        s.row_lse[c] = (double)Mc + log(Lc);
    }
    s.row_arg[c] = arg;
    wave_lds_sync();

    int cur = 0, len = 0, mypath = 0;                        // lane i keeps path[i]
    int32_t *path = a.accept_path + (size_t)b * (a.D_max + 1);
    if (!sampling) {
        const bool match = tree_ok && s.row_arg[p] == t;
        while (len < a.D_max) {
            const uint64_t m = __ballot(match && p == cur);
            if (!m) break;
            cur = __ffsll((long long)m) - 1;
            ++len;
            if (lane == len) mypath = cur;
        }
        if (lane == 0) { a.accept_len[b] = len; a.bonus[b] = s.row_arg[cur]; }
        if (c <= a.D_max) path[c] = (c <= len) ? mypath : -1;
        return;
    }

    // probability of each node's token under its parent's row
    double pc = 0.0;
    if (tree_ok && t >= 0 && t < a.V) pc = exp((double)xg * a.inv_temp - s.row_lse[p]);

    if (a.mode == kAccDistribution) {
        // Sec. 4.3, Eq. 11-13.  Nodes are visited in index order (parents come first), one lane per
        // node, values passed between lanes by lane reads; sums run in node order.
        bool dup = false;                                    // same token as an earlier sibling: never reached
        for (int o = 1; o < nn; ++o) {
            const int po = (int)readlane_u32((uint32_t)p, o), to = (int)readlane_u32((uint32_t)t, o);
            dup = dup || (o < c && po == p && to == t);
        }
        if (dup) pc = 0.0;
        // depth and reach level by level: a lane whose parent is settled takes depth(parent) + 1 and
        // reach(parent) * its own probability (two lane gathers); as many rounds as the tree is deep.
        // Nodes with a broken parent count as settled with depth 0 and reach 0.
        int depth = 0;
        double reach = c == 0 ? 1.0 : 0.0, kids = 0.0;       // mass that arrives here / that goes on to children
        bool settled = !tree_ok;                             // the root and everything outside the tree
        for (int round = 0; round < nn; ++round) {
            if (__ballot(!settled) == 0ull) break;
            const int src = max(p, 0);
            const int pd = __shfl(depth, src);
            const bool ps = __shfl((int)settled, src) != 0;
            const double pr = __longlong_as_double(__shfl((long long)__double_as_longlong(reach), src));
            if (!settled && ps) {
                depth = pd + 1;
                if (depth > a.D_max) pc = 0.0;               // cut: nothing is handed below D_max
                reach = pr * pc;
                settled = true;
            }
        }
        for (int v = 1; v < nn; ++v) {                       // children's mass per parent, summed in node order
            const int pv = (int)readlane_u32((uint32_t)p, v);
            const double pcv = readlane_f64(pc, v);
            if (lane == pv) kids += pcv;
        }
        double stay = 1.0 - kids;
        stay = stay > 0.0 ? stay : 0.0;
        const double pstop = (c < nn && depth <= a.D_max) ? reach * stay : 0.0;
        double acc = 0.0;
        for (int v = 0; v < nn; ++v) {
            const int dv = (int)readlane_u32((uint32_t)depth, v);
            const double sv = readlane_f64(pstop, v);
            if (lane == dv) acc += sv;
        }
        for (int d = lane; d <= a.D_max; d += kWave) a.dist[(size_t)b * (a.D_max + 1) + d] = d == lane ? acc : 0.0;
        return;
    }
    double R = 0.0;
    int nrej = 0, rejtok = -1;                               // lane j keeps the j-th rejected token
    for (;;) {
        uint64_t kids = (len < a.D_max) ? __ballot(tree_ok && p == cur) : 0ull;
        R = 0.0; nrej = 0;
        int next = -1;
        if (__popcll(kids) > 4) {
            // wide level: all children at once.  A child is reached only if every earlier sibling was
            // rejected, so its residual is the sum of the earlier siblings' probabilities.
            const bool kid = (kids >> lane) & 1;
            // same token as an earlier sibling?  Tokens are hashed into a byte table; a lane that does
            // not read its own number back shares a bucket, and only then are tokens compared.
            const uint32_t h = ((uint32_t)t * 2654435761u) >> 20;
            if (kid) s.seen[h] = (unsigned char)lane;
            wave_lds_sync();
            const bool shared = kid && s.seen[h] != (unsigned char)lane;
            wave_lds_sync();
            bool dup = false;
            if (__ballot(shared)) {
                for (uint64_t m = kids; m; m &= m - 1) {
                    const int cc = __ffsll((long long)m) - 1;
                    const int tcc = (int)readlane_u32((uint32_t)t, cc);
                    dup = dup || (kid && lane > cc && t == tcc);
                }
            }
            const bool live = kid && !dup;
            const double mine = live ? pc : 0.0;
            const double before = wave_scan_f64(mine) - mine;
            const uint64_t acc = __ballot(live && (double)uc * (1.0 - before) < pc);
            uint64_t rejected = __ballot(live);
            if (acc) {
                next = __ffsll((long long)acc) - 1;
                rejected &= (1ull << next) - 1;
            }
            nrej = __popcll(rejected);
            R = nrej ? readlane_f64(before + mine, 63 - __clzll((long long)rejected)) : 0.0;
            // lane j takes the token of the j-th rejected child
            if ((rejected >> lane) & 1) s.row_arg[lanes_below(rejected)] = t;      // row_arg is free by now
            wave_lds_sync();
            rejtok = lane < nrej ? s.row_arg[lane] : -1;
            wave_lds_sync();
        } else {
            while (kids) {
                const int cc = __ffsll((long long)kids) - 1;
                kids &= kids - 1;
                const int tcc = (int)readlane_u32((uint32_t)t, cc);
                if (__ballot(lane < nrej && rejtok == tcc)) continue;   // same token as an earlier sibling
                const double pcc = readlane_f64(pc, cc);
                const float ucc = readlane_f32(uc, cc);
                if ((double)ucc * (1.0 - R) < pcc) { next = cc; break; }
                R += pcc;
                if (lane == nrej) rejtok = tcc;
                ++nrej;
            }
        }
        if (next < 0) break;
        cur = next;
        ++len;
        if (lane == len) mypath = cur;
    }
    if (c <= a.D_max) path[c] = (c <= len) ? mypath : -1;
    if (lane == 0) a.accept_len[b] = len;

    // ---- residual draw, (a): the 1024-logit block that holds the target mass
    const float M = readlane_f32(Mc, cur);
    const double L = readlane_f64(Lc, cur);
    const size_t p0 = ((size_t)b * a.T + cur) * a.nsub;
    const float *xr = a.logits + ((size_t)b * a.T + cur) * a.V;
    // masses of the first 128 blocks: requested together with the rejected tokens' logits
    double mass0 = (lane < a.nsub) ? load_shared_result(&a.part_l[p0 + lane]) : 0.0;
    double mass1 = (kWave + lane < a.nsub) ? load_shared_result(&a.part_l[p0 + kWave + lane]) : 0.0;
    {   // what the rejected children's tokens carry (the same arithmetic as pass (b) uses)
        float xj = -INFINITY;
        int sj = -1;
        if (lane < nrej && rejtok >= 0 && rejtok < a.V) {
            xj = xr[rejtok];
            sj = rejtok / kAccSub;
        }
        s.rej_e[lane] = sj >= 0 ? scaled_exp(xj, a, M) : 0.0;
        s.rej_sub[lane] = sj;
        wave_lds_sync();
    }
    const double target = (double)ubonus * (1.0 - R) * L;
    double before = 0.0;                                     // mass of the blocks before this group of 64
    int pick = -1, lastc = -1;
    double resid = 0.0;
    for (int c0 = 0; c0 < a.nsub && pick < 0; c0 += kWave) {
        const int cs = c0 + lane;
        double mass = c0 == 0 ? mass0 : mass1;
        if (c0 >= 2 * kWave) mass = (cs < a.nsub) ? load_shared_result(&a.part_l[p0 + cs]) : 0.0;
        for (int j0 = 0; j0 < nrej; j0 += 8) {                // broadcast LDS reads, eight in flight; entries
#pragma unroll                                                 // past nrej name no block
            for (int j = j0; j < j0 + 8; ++j) {
                const double e = s.rej_e[j];                 // read unconditionally: no branch per entry
                mass -= (s.rej_sub[j] == cs) ? e : 0.0;
            }
        }
        mass = mass > 0.0 ? mass : 0.0;
        const double incl = before + wave_scan_f64(mass);
        const uint64_t hit = __ballot(cs < a.nsub && incl > target);
        const uint64_t pos = __ballot(cs < a.nsub && mass > 0.0);
        if (pos) lastc = c0 + 63 - __clzll((long long)pos);
        if (hit) {
            const int hl = __ffsll((long long)hit) - 1;
            pick = c0 + hl;
            resid = target - (readlane_f64(incl, hl) - readlane_f64(mass, hl));
        }
        before = readlane_f64(incl, kWave - 1);
    }
    if (pick < 0) {                                          // rounding pushed the target past the total:
        pick = lastc >= 0 ? lastc : 0;                       // the last token with mass is taken
        resid = INFINITY;
    }

    // ---- residual draw, (b): inside the chosen block every lane owns 16 consecutive tokens
    s.rej_bits[lane] = 0;
    wave_lds_sync();
    if (lane < nrej && rejtok >= 0 && rejtok / kAccSub == pick) {
        const int off = rejtok - pick * kAccSub;
        atomicOr(&s.rej_bits[off / kAccEPT], 1u << (off % kAccEPT));
    }
    float xv[kAccEPT];
    int first[kAccEPT / 4];
    load_block<VEC4, true>(xr, pick * kAccSub, a.V, xv, first);
    wave_lds_sync();
    const unsigned int rejected = s.rej_bits[lane];
    const int i0 = pick * kAccSub + lane * kAccEPT;
    double pv[kAccEPT];
    double sum = 0.0;
    int lastpos = -1;
#pragma unroll
    for (int e = 0; e < kAccEPT; ++e) {
        const int i = i0 + e;
        const double v = (i < a.V && !((rejected >> e) & 1)) ? scaled_exp(xv[e], a, M) : 0.0;
        pv[e] = v;
        sum += v;
        if (v > 0.0) lastpos = i;
    }
    const double incl = wave_scan_f64(sum);
    const uint64_t hit = __ballot(incl > resid);
    const int lp = (int)wave_max_u32((uint32_t)(lastpos + 1)) - 1;      // last token of the block with mass
    int bonus = lp;
    if (hit) {
        const int owner = __ffsll((long long)hit) - 1;
        int mine = -1;
        double cdf = incl - sum;
#pragma unroll
        for (int e = 0; e < kAccEPT; ++e) {
            cdf += pv[e];
            if (mine < 0 && pv[e] > 0.0 && cdf > resid) mine = i0 + e;
        }
        if (mine < 0) mine = lastpos;
        const int got = (int)readlane_u32((uint32_t)mine, owner);
        if (got >= 0) bonus = got;
    }
    if (lane == 0) a.bonus[b] = bonus;
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
// per-wavefront partials.  Returns the total size; fills the pointers when `ws` is given.
static size_t accept_layout(int B, int T, size_t nsub, char *ws, AcceptArgs *a) {
    const size_t rows = (size_t)B * T, slots = rows * nsub;
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
    const size_t nsub = ((size_t)d->V + kAccSub - 1) / kAccSub;
    return accept_layout(d->B, d->T_max, nsub, nullptr, nullptr);
}

static radar_status launch_accept(const float *target_logits, const int32_t *draft_tokens, const int32_t *parents,
                                  const int32_t *n_nodes, const float *uniforms, int32_t *accept_len,
                                  int32_t *accept_path, int32_t *bonus_token, double *dist, int mode,
                                  const radar_accept_desc *d, void *workspace, size_t workspace_bytes, void *stream) {
    if (d->B < 1 || d->T_max < 1 || d->V < 1 || d->D_max < 0) return RADAR_INVALID_ARG;
    if (mode != RADAR_ACCEPT_GREEDY && !(d->temperature > 0.0f)) return RADAR_INVALID_ARG;
    const int64_t nsub = ((int64_t)d->V + kAccSub - 1) / kAccSub;
    const int64_t nwg = (nsub + kAccWaves - 1) / kAccWaves;
    if (d->T_max > RADAR_T_MAX || d->D_max >= RADAR_T_MAX || d->B > 65535 || nsub > kAccMaxSubs)
        return RADAR_UNSUPPORTED_SHAPE;
    if (workspace_bytes < radar_verify_accept_workspace_bytes(d)) return RADAR_WORKSPACE_TOO_SMALL;
    if (((uintptr_t)workspace & 255) != 0) return RADAR_INVALID_ARG;

    AcceptArgs a;
    a.logits = target_logits; a.tokens = draft_tokens; a.parents = parents; a.n_nodes = n_nodes; a.uniforms = uniforms;
    a.accept_len = accept_len; a.accept_path = accept_path; a.bonus = bonus_token; a.dist = dist;
    a.B = d->B; a.T = d->T_max; a.V = d->V; a.D_max = d->D_max; a.mode = mode;
    a.nsub = (int)nsub; a.nwg = (int)nwg;
    a.inv_temp = mode != RADAR_ACCEPT_GREEDY ? 1.0 / (double)d->temperature : 1.0;
    a.inv_temp_f = (float)a.inv_temp;
    a.exact_scale = ((double)a.inv_temp_f == a.inv_temp) ? 1 : 0;
    accept_layout(d->B, d->T_max, (size_t)nsub, static_cast<char *>(workspace), &a);

    const dim3 grid((unsigned)nwg, (unsigned)d->T_max, (unsigned)d->B), block(kAccThreads);
    const bool vec4 = (d->V % 4 == 0) && (((uintptr_t)target_logits & 15) == 0);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const char *name = mode == kAccDistribution ? "accept_length_distribution" : "accept";
    const hipError_t e = vec4 ? launch(name, accept_kernel<true>, grid, block, 0, st, a)
                              : launch(name, accept_kernel<false>, grid, block, 0, st, a);
    return e == hipSuccess ? RADAR_OK : RADAR_HIP_ERROR;
}

extern "C" radar_status radar_verify_accept(const float *target_logits, const int32_t *draft_tokens,
                                            const int32_t *parents, const int32_t *n_nodes, const float *uniforms,
                                            int32_t *accept_len, int32_t *accept_path, int32_t *bonus_token,
                                            const radar_accept_desc *d, void *workspace, size_t workspace_bytes,
                                            void *stream) {
    if (!d || !target_logits || !draft_tokens || !parents || !accept_len || !accept_path || !bonus_token || !workspace)
        return RADAR_INVALID_ARG;
    if (d->mode != RADAR_ACCEPT_GREEDY && d->mode != RADAR_ACCEPT_SAMPLE) return RADAR_INVALID_ARG;
    if (d->mode == RADAR_ACCEPT_SAMPLE && !uniforms) return RADAR_INVALID_ARG;
    return launch_accept(target_logits, draft_tokens, parents, n_nodes, uniforms, accept_len, accept_path, bonus_token,
                         nullptr, d->mode, d, workspace, workspace_bytes, stream);
}

extern "C" radar_status radar_accept_length_distribution(const float *target_logits, const int32_t *draft_tokens,
                                                         const int32_t *parents, const int32_t *n_nodes, double *dist,
                                                         const radar_accept_desc *d, void *workspace,
                                                         size_t workspace_bytes, void *stream) {
    if (!d || !target_logits || !draft_tokens || !parents || !dist || !workspace) return RADAR_INVALID_ARG;
    return launch_accept(target_logits, draft_tokens, parents, n_nodes, nullptr, nullptr, nullptr, nullptr, dist,
                         kAccDistribution, d, workspace, workspace_bytes, stream);
}

extern "C" radar_status radar_debug_validate_tree(const int32_t *parents, const int32_t *n_nodes, int32_t B,
                                                  int32_t T_max, int32_t *bad_count_out, void *stream) {
    if (!parents || !bad_count_out || B < 1 || T_max < 1) return RADAR_INVALID_ARG;
    const hipError_t e = launch("validate_tree", validate_tree_kernel, dim3(1), dim3(256), 0,
                                static_cast<hipStream_t>(stream), parents, n_nodes, (int)B, (int)T_max, bad_count_out);
    return e == hipSuccess ? RADAR_OK : RADAR_HIP_ERROR;
}
