// Draft-tree expansion and rerank for RADAR's drafting loop (App. A.1, Sec. 2.3,
// Sec. 4.2 Eq. 3), as single-launch HIP kernels for gfx950.
//
// radar_draft_expand: grid (chunks of 4096, 8192 or 16384 logits, frontier rows).
// Every workgroup streams its chunk once from HBM with 16-byte loads (the whole
// step is one read of F*V*4 bytes), keeps its 4, 8 or 16 values per lane in registers,
// and leaves (chunk top-k keys, chunk max, chunk sum of exp) in the workspace.
// Arrival tickets (one counter per row, then one per call) single out the
// workgroup that finishes last; it merges every row, one wavefront per row
// (top-k of the chunk lists, log-sum-exp in fp64, cumulative scores, pool
// append), and picks the next frontier.  There is no second launch and no
// host round trip.  radar_draft_expand_policy lets the same workgroup go on to
// the prediction model's step on the k confidences it has just produced
// (Sec. 4.2), so the continue / stop decision costs no launch of its own.
// radar_draft_expand_batch adds a grid dimension: one such call per sequence,
// B sequences in one launch, each with its own arrays, tickets and last workgroup.
#include <algorithm>
#include <mutex>

#include "radar_topk.h"
#include "radar_policy.h"
#include "radar_host.h"

namespace radar {

constexpr int kExpThreads = 1024;
constexpr int kExpWaves = kExpThreads / kWave;
constexpr int kExpMinEPT = 4;                         // logits per lane: 4, 8 or 16 (chosen per call)
constexpr int kExpMaxChunks = 256;                    // V <= 1,048,576
constexpr int kCounterStride = 32;                    // arrival counters sit 128 B apart: fetch-adds on one
                                                      // cache line serialise at roughly 10 ns each
constexpr size_t kCounterBytes = 16384;               // leading counter block of the workspace
constexpr float kLog2eF = 1.4426950408889634f;
constexpr int kDumpCap = 64;                          // hot lanes (largest logit reaches the threshold) whose logits go through LDS
constexpr int kFastCap = 512;                         // chunk candidates ranked by the short path; more (runs of equal values) rank per wavefront
constexpr int64_t kStreamMinLogits = 4 << 20;         // batched calls of at least 16 MB of logits take the streaming path

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
    int pool_capacity;          // length of one sequence's pool arrays (their stride in a batched call)
    unsigned int *counters;     // [0] rows finished, [(1+f) * kCounterStride] chunks of row f finished
    uint64_t *part_keys;        // [F][nchunks][RADAR_K_MAX] best first, 0 where a chunk has fewer
    double *part_l;             // [F][nchunks] sum of exp(x - part_m) over the chunk
    float *part_m;              // [F][nchunks] chunk maximum
    PolicyArgs pol;             // prediction model run by the last workgroup when has_policy != 0
    float *gate_pre;            // [4H] w_hh h of that model, computed by the first workgroups of the launch
    radar_cycle_state *cycle;   // device-side state of the drafting cycle, or null: when set, pool_count above is
                                // only the largest value the state's own count may have
    int has_policy, pol_has_state;
};

struct alignas(16) ExpandSmem {
    WaveTopkSmem wtk[kExpWaves];                  // one scratch per wavefront
    uint64_t wlist[kExpWaves * kWaveListSlots];   // the wavefronts' candidates of a chunk (0 = none; many ties only)
    float gmax[16];                               // maxima of the sixteen 16-lane rows of the streaming wavefronts
    float wave_l[4];                              // sum of exp(x - chunk maximum) over each streaming wavefront
    unsigned int nsurv;                           // candidates of the chunk that reached the threshold
    unsigned int ndump;                           // lanes whose largest logit reached it
    float tau;                                    // the threshold
    unsigned short dump_lane[kDumpCap];           // which lane left each block of logits
    // last workgroup only: candidate (row f, rank r) at f * 16 + r
    float cand_sc[RADAR_F_MAX * 16];
    int cand_tok[RADAR_F_MAX * 16];
    unsigned int ticket, ticket2;
};

// 512 slots, starting at c0, of one row's chunk lists in the workspace (device-scope loads)
__device__ __forceinline__ void load_key_block(const uint64_t *pk, int nslot, int c0, int K, uint64_t (&kk)[9]) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int i = c0 + topk_slot_of(e);
        const uint64_t key = load_shared_result(pk + min(i, nslot - 1));     // branch-free: clamp, load, mask
        kk[e] = (i < nslot && (i & 15) < K) ? key : 0;
    }
    kk[8] = 0;
}

// top-K of one row's chunk lists by one wavefront; kk holds the first 512 slots already
__device__ __forceinline__ uint64_t row_topk(uint64_t (&kk)[9], const uint64_t *pk, int nslot, int K, WaveTopkSmem &scratch) {
    uint64_t top = wave_topk<9>(kk, K, scratch);
    for (int c0 = 8 * kWave; c0 < nslot; c0 += 8 * kWave) {        // V > 131072 only
        load_key_block(pk, nslot, c0, K, kk);
        kk[8] = top;                                                 // the running selection rides along
        top = wave_topk<9>(kk, K, scratch);
    }
    return top;
}

// Next frontier: top-k of the F*k candidates in s.cand_sc by cumulative score (candidate index
// breaks ties), by one wavefront.  conf_lds, when given, also receives the k confidences.
__device__ __forceinline__ void select_frontier(const ExpandArgs &a, ExpandSmem &s, float *conf_lds) {
    const int lane = lane_id();
    const int K = a.k;
    // ---- next frontier: top-k of the candidates by cumulative score (candidate index breaks ties)
    const int nfs = a.F * 16;
    uint64_t top;
    if (nfs <= 4 * kWave) {                                    // F <= 16 rows: four slots per lane
        uint64_t kk[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int i = topk_slot_of(e);
            const float sc = s.cand_sc[min(i, nfs - 1)];
            kk[e] = (i < nfs && (i & 15) < K) ? make_key(sc, uint32_t((i >> 4) * K + (i & 15))) : 0;
        }
        top = wave_topk<4>(kk, K, s.wtk[0]);
    } else {
        top = 0;
        for (int c0 = 0; c0 < nfs; c0 += 8 * kWave) {
            uint64_t kk[9];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int i = c0 + topk_slot_of(e);
                const float sc = s.cand_sc[min(i, nfs - 1)];
                kk[e] = (i < nfs && (i & 15) < K) ? make_key(sc, uint32_t((i >> 4) * K + (i & 15))) : 0;
            }
            kk[8] = top;
            top = wave_topk<9>(kk, K, s.wtk[0]);
        }
    }
    if (lane < K) {
        const int C = a.F * K;
        int c = (int)key_index(top);
        if (c < 0 || c >= C) c = 0;                               // only reachable with NaN scores
        const int fr = c / K, r = c - fr * K;
        const float sc = s.cand_sc[fr * 16 + r];
        a.frontier_pool_idx[lane] = a.pool_count + c;
        a.frontier_tokens[lane] = s.cand_tok[fr * 16 + r];
        a.frontier_scores[lane] = sc;
        const float conf = expf(sc);
        a.frontier_conf[lane] = conf;
        if (conf_lds) conf_lds[lane] = conf;
    }
}

// Sequence bz of a batched call: every array of the call, the workspace parts and the cycle states
// have a leading batch dimension; after this the workgroup sees its own sequence only.
__device__ __forceinline__ void sequence_view(ExpandArgs &a, int bz) {
    const size_t b = (size_t)bz, fk = (size_t)a.F * a.k, fc = (size_t)a.F * a.nchunks;
    a.logits += b * a.F * a.V;
    a.parent_scores += b * a.F; a.parent_pool_idx += b * a.F;
    a.cand_tokens += b * fk; a.cand_scores += b * fk;
    a.frontier_pool_idx += b * a.k; a.frontier_tokens += b * a.k;
    a.frontier_scores += b * a.k; a.frontier_conf += b * a.k;
    a.pool_tokens += b * a.pool_capacity; a.pool_scores += b * a.pool_capacity; a.pool_parents += b * a.pool_capacity;
    a.counters += b * (kCounterBytes / sizeof(unsigned int));
    a.part_keys += b * fc * RADAR_K_MAX; a.part_l += b * fc; a.part_m += b * fc;
    a.gate_pre += b * (4 * kPolH);
    if (a.cycle) a.cycle += b;
}

// What the last workgroup of a sequence's call does once every chunk list and partial sum of the
// sequence is in the workspace (all 1024 lanes must call): rows are merged, candidates scored and
// pooled, the next frontier chosen; with a prediction model its step follows, with a cycle state
// its update.  `a` is already the sequence's own view of the call (bz = its index in the batch).
// hidden(row) returns row `row` of w_hh h (complete before the call; only used with a prediction
// model that has a state).
template <bool EXT, typename Hidden>
__device__ __forceinline__ void expand_finish(const ExpandArgs &a, ExpandSmem &s, int bz, radar_cycle_state *cycle,
                                              bool cycle_first, Hidden &&hidden) {
    const bool has_policy = EXT && a.has_policy != 0;
    const int lane = lane_id(), w = wave_id();
    const int K = a.k;
    // One wavefront per row (rows w, w+16, ...):
    // top-k of the row's chunk lists, log-sum-exp of the row, cumulative scores, pool append.
    const int nslot = a.nchunks * RADAR_K_MAX;
    for (int fr = w; fr < a.F; fr += kExpWaves) {
        const uint64_t *pk = a.part_keys + (size_t)fr * nslot;
        const bool few = nslot <= 4 * kWave;                       // up to 16 chunks per row (V <= 131072 at 8 per lane)
        uint64_t kk[9];
        if (few) {                                                 // four slots per lane: half the loads, a shorter selection
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int i = topk_slot_of(e);
                const uint64_t key = load_shared_result(pk + min(i, nslot - 1));
                kk[e] = (i < nslot && (i & 15) < K) ? key : 0;
            }
        } else {
            load_key_block(pk, nslot, 0, K, kk);
        }
        float ml;
        double ll;
        const bool few_chunks = a.nchunks <= 16;                   // every 16-lane row of the wavefront takes all chunks
        {                                                          // chunk partials, one chunk per lane first
            const int cl = few_chunks ? (lane & 15) : lane;
            const int c = min(cl, a.nchunks - 1);
            ml = load_shared_result(&a.part_m[(size_t)fr * a.nchunks + c]);
            ll = load_shared_result(&a.part_l[(size_t)fr * a.nchunks + c]);
            if (cl >= a.nchunks) { ml = -INFINITY; ll = 0.0; }
        }
        const float pscore = a.parent_scores[fr];
        const int ppool = a.parent_pool_idx[fr];
        uint64_t top;
        if (few) {
            const uint64_t k4[4] = {kk[0], kk[1], kk[2], kk[3]};
            top = wave_topk<4>(k4, K, s.wtk[w]);
        } else {
            top = row_topk(kk, pk, nslot, K, s.wtk[w]);
        }
        for (int c = lane + kWave; c < a.nchunks; c += kWave) {        // V > 262144 only
            const float m2 = load_shared_result(&a.part_m[(size_t)fr * a.nchunks + c]);
            const double l2 = load_shared_result(&a.part_l[(size_t)fr * a.nchunks + c]);
            const float mn = fmaxf(ml, m2);
            if (mn > -INFINITY)
                ll = ll * (double)__builtin_amdgcn_exp2f((ml - mn) * kLog2eF) + l2 * (double)__builtin_amdgcn_exp2f((m2 - mn) * kLog2eF);
            ml = mn;
        }
        float M;
        double L;
        if (few_chunks) {
            // maximum and sum inside each 16-lane row by DPP steps alone (no lane reads: those cost a
            // scalar round trip each); fixed order of addition, every lane ends up with the result
            M = ml;
            M = fmaxf(M, dpp_f32<0xB1>(M));
            M = fmaxf(M, dpp_f32<0x4E>(M));
            M = fmaxf(M, dpp_f32<0x141>(M));
            M = fmaxf(M, dpp_f32<0x140>(M));
            L = ml > -INFINITY ? ll * (double)__builtin_amdgcn_exp2f((ml - M) * kLog2eF) : 0.0;
            auto add = [](double x, uint64_t moved) { return x + __longlong_as_double((long long)moved); };
            L = add(L, dpp_u64<0xB1>((uint64_t)__double_as_longlong(L)));
            L = add(L, dpp_u64<0x4E>((uint64_t)__double_as_longlong(L)));
            L = add(L, dpp_u64<0x141>((uint64_t)__double_as_longlong(L)));
            L = add(L, dpp_u64<0x140>((uint64_t)__double_as_longlong(L)));
        } else {
            M = wave_max_f32(ml);
            L = wave_sum_f64(ml > -INFINITY ? ll * (double)__builtin_amdgcn_exp2f((ml - M) * kLog2eF) : 0.0);
        }
        // log in fp32 (1 ulp of a value below 14: 1e-6, a tenth of the tolerance on log-probabilities); the
        // fp64 routine costs 0.3 us on this serial path
        const double lse = (double)M + (double)logf((float)L);
        if (lane < K) {
            const int tok = (int)key_index(top);
            const double logp = (double)key_value(top) - lse;
            const float cum = (float)((double)pscore + logp);
            const int c = fr * K + lane;
            a.cand_tokens[c] = tok;
            a.cand_scores[c] = cum;
            a.pool_tokens[a.pool_count + c] = tok;
            a.pool_scores[a.pool_count + c] = cum;
            a.pool_parents[a.pool_count + c] = ppool;
            s.cand_sc[fr * 16 + lane] = cum;
            s.cand_tok[fr * 16 + lane] = tok;
        }
    }
    __syncthreads();
    if (!has_policy) {
        if (w == 0) {
            select_frontier(a, s, nullptr);
            if (cycle && lane == 0) {
                cycle->pool_count = a.pool_count + a.F * a.k;
                cycle->steps_done = cycle_first ? 1 : cycle->steps_done + 1;
                if (cycle_first) { cycle->stopped = 0; cycle->last_action = -1; }
            }
        }
        return;
    }
    // ---- prediction-model step on the new frontier's confidences.  Its LDS reuses the
    // selection scratch of wavefronts 1.., idle since the barrier above; the other wavefronts
    // fetch the model's operands while wavefront 0 still selects the frontier.
    static_assert(sizeof(PolicySmem) <= (kExpWaves - 1) * sizeof(WaveTopkSmem) && sizeof(WaveTopkSmem) % 16 == 0, "policy LDS overlay");
    PolicySmem &ps = *reinterpret_cast<PolicySmem *>(&s.wtk[1]);
    policy_step_block<true>(
        a.pol, bz, a.pol_has_state != 0, ps, hidden,
        [&] { select_frontier(a, s, ps.x); },
        [&](int action) {
            if (cycle) {
                cycle->pool_count = a.pool_count + a.F * a.k;
                cycle->steps_done = cycle_first ? 1 : cycle->steps_done + 1;
                cycle->last_action = action;
                if (action == 0) cycle->stopped = 1;
                else if (cycle_first) cycle->stopped = 0;
            }
        });
}

// EXT: the launch may carry a prediction model and / or a device-side cycle state; the plain
// expansion is compiled without any of that code.
template <bool VEC4, int EPT, bool EXT>
__global__ __launch_bounds__(kExpThreads, 1) void expand_kernel(ExpandArgs a) {
    const bool has_policy = EXT && a.has_policy != 0;
    static_assert(EPT == 4 || EPT == 8 || EPT == 16, "EPT");
    static_assert(kFastCap + 8 <= kWave * kWaveTopkMaxEPL + 8 && kExpWaves == 16, "candidate list inside the selection scratch");
    constexpr int kChunk = kExpThreads * EPT;
    __shared__ ExpandSmem s;
    const int tid = threadIdx.x, lane = lane_id(), w = wave_id();
    const int f = blockIdx.y, chunk = blockIdx.x;
    const int bz = EXT ? (int)blockIdx.z : 0;
    if (EXT && bz != 0) sequence_view(a, bz);
    radar_cycle_state *const cycle = EXT ? a.cycle : nullptr;
    // The first draft call of a cycle (the host says so: the largest count the state may hold is 0)
    // never reads the state; its last workgroup writes all of it.
    const bool cycle_first = cycle != nullptr && a.pool_count == 0;
    if (cycle && !cycle_first) {
        // A drafting cycle that has stopped skips its remaining draft calls: every workgroup leaves
        // before touching anything.  (The state is only written by the last workgroup of a launch,
        // after every other workgroup has handed over its results, i.e. long after this read.)
        const int pc = cycle->pool_count;
        if (cycle->stopped != 0 || pc < 0 || pc > a.pool_count) return;
        a.pool_count = pc;
    }
    const float *row = a.logits + (size_t)f * a.V;
    const int base = chunk * kChunk;
    const int K = a.k;

    // ---- stream the chunk.  Only the first four wavefronts (one per SIMD) stream and select: a
    // 64-wide vector instruction occupies its SIMD for four cycles whichever wavefront issues it, so
    // four wavefronts with 4 * EPT logits per lane do the per-logit work in the same time as sixteen
    // with EPT each, and what a wavefront does once (reductions, threshold, list bookkeeping) is
    // done four times per workgroup instead of sixteen.  The other wavefronts only serve the end of
    // the call (one row each, the prediction model).  NE/4 x (256 lanes x 16 B) coalesced loads, all
    // issued before anything is computed from them (out-of-range lanes read a valid address and are
    // masked).
    constexpr int kStreamers = 4;                                  // wavefronts that stream
    constexpr int kSLanes = kStreamers * kWave;
    constexpr int NE = EPT * (kExpThreads / kSLanes);              // logits per streaming lane
    const bool streamer = w < kStreamers;
    const bool tail = base + kChunk > a.V;                         // the row ends inside this chunk
    float x[NE];
    if (streamer) {
        float4 raw[NE / 4];
#pragma unroll
        for (int g = 0; g < NE / 4; ++g) {
            const int idx0 = base + g * (kSLanes * 4) + tid * 4;
            if (VEC4) {
                raw[g] = *reinterpret_cast<const float4 *>(row + (idx0 < a.V ? idx0 : 0));
            } else {
                raw[g].x = row[min(idx0 + 0, a.V - 1)];
                raw[g].y = row[min(idx0 + 1, a.V - 1)];
                raw[g].z = row[min(idx0 + 2, a.V - 1)];
                raw[g].w = row[min(idx0 + 3, a.V - 1)];
            }
        }
#pragma unroll
        for (int g = 0; g < NE / 4; ++g) {
            x[4 * g + 0] = raw[g].x; x[4 * g + 1] = raw[g].y; x[4 * g + 2] = raw[g].z; x[4 * g + 3] = raw[g].w;
        }
        if (tail) {
#pragma unroll
            for (int e = 0; e < NE; ++e) {
                const int idx = base + (e >> 2) * (kSLanes * 4) + tid * 4 + (e & 3);
                x[e] = idx < a.V ? x[e] : -INFINITY;
            }
        }
    }
    // The prediction model's input-free part (w_hh h) is shared out over the workgroups of the
    // launch: its loads travel with the logits', its results are handed to the last workgroup
    // through the workspace like the chunk partials.
    if (has_policy && a.pol_has_state)
        policy_hidden_rows<4>(a.pol, bz, blockIdx.y * gridDim.x + blockIdx.x, gridDim.x * gridDim.y,
                              [&](int r, float v) { store_shared_result(&a.gate_pre[r], v); });

    // ---- the chunk's maximum, and the threshold of its top-k: the k-th largest of the maxima of the
    // sixteen 16-lane rows of the streaming wavefronts.  At least k logits of the chunk reach it (one
    // per row whose maximum does), and on untied data only about 1.6 k do.  Everything here is a
    // chain of latencies (a ballot whose count a scalar instruction needs costs ~30 cycles, a lane
    // read with a compare ~40, an LDS round trip ~120), so the steps are laid out to run side by
    // side: a wavefront that does not stream ranks the sixteen maxima while the streaming ones take
    // their exponentials, and logits are compared with the threshold only where they can reach it.
    float lmax = -INFINITY;                                        // the lane's largest logit
    if (streamer) {
        lmax = x[0];
#pragma unroll
        for (int e = 1; e < NE; ++e) lmax = fmaxf(lmax, x[e]);
        float rm = lmax;
        rm = fmaxf(rm, dpp_f32<0xB1>(rm));
        rm = fmaxf(rm, dpp_f32<0x4E>(rm));
        rm = fmaxf(rm, dpp_f32<0x141>(rm));
        rm = fmaxf(rm, dpp_f32<0x140>(rm));                        // every lane: the maximum of its 16-lane row
        if ((lane & 15) == 0) s.gmax[w * 4 + (lane >> 4)] = rm;
    }
    if (tid == 0) { s.nsurv = 0; s.ndump = 0; }
    __syncthreads();
    float cm = 0.f;                                                // chunk maximum (streamers, and wavefront 1 below)
    if (w == kStreamers) {
        // threshold: the k-th largest of the sixteen maxima (ties: lower row first), by one wavefront
        const uint32_t ov = ord_of(s.gmax[lane & 15]);             // every 16-lane row holds the 16 maxima
        int larger = 0;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const uint32_t oj = readlane_u32(ov, j);
            larger += (oj > ov || (oj == ov && j < (lane & 15))) ? 1 : 0;
        }
        const uint64_t sel = __ballot(larger == K - 1) & 0xffffull; // ranks are a permutation of 0..15: exactly one lane
        if (lane == 0) s.tau = float_of_ord(readlane_u32(ov, __ffsll((long long)sel) - 1));
    } else if (streamer) {
        cm = s.gmax[lane & 15];
        cm = fmaxf(cm, dpp_f32<0xB1>(cm));
        cm = fmaxf(cm, dpp_f32<0x4E>(cm));
        cm = fmaxf(cm, dpp_f32<0x141>(cm));
        cm = fmaxf(cm, dpp_f32<0x140>(cm));
        // ---- sum of exp(x - chunk maximum): fp32 exponentials; a lane adds its terms in four fp32 chains,
        // the wavefront's 64 lanes as a fixed fp32 tree (relative error below 1e-6), the rest is fp64.
        // (x - cm) first: folding the scale into one fused multiply-add would round cm * log2(e), an
        // absolute error in the exponent that grows with |cm|.
        float tl[4] = {0.f, 0.f, 0.f, 0.f};
        if (cm > -INFINITY) {
#pragma unroll
            for (int e = 0; e < NE; ++e) tl[e & 3] += __builtin_amdgcn_exp2f((x[e] - cm) * kLog2eF);
        }
        const float wl = wave_sum_f32((tl[0] + tl[1]) + (tl[2] + tl[3]));
        if (lane == 0) s.wave_l[w] = wl;
    }
    __syncthreads();
    // Lanes whose largest logit reaches the threshold (about 1.6 k of the 256) leave all their logits
    // in LDS; only those are compared one by one afterwards.
    float *const dump = reinterpret_cast<float *>(&s.wtk[1]);      // [kDumpCap][NE], inside the selection scratch
    uint64_t *const surv = s.wtk[0].surv;                          // kFastCap + 8 slots
    static_assert(kDumpCap * NE * sizeof(float) <= (kExpWaves - 1) * sizeof(WaveTopkSmem), "dump inside the scratch");
    const float tau_f = s.tau;
    if (streamer) {
        const bool hot = lmax >= tau_f && base + tid * 4 < a.V;    // (a lane wholly past the row holds -inf only)
        const uint64_t hm = __ballot(hot);
        if (hm != 0) {
            int at = 0;
            if (lane == 0) at = (int)atomicAdd(&s.ndump, (unsigned int)__popcll(hm));
            at = (int)readlane_u32((uint32_t)at, 0) + lanes_below(hm);
            if (hot && at < kDumpCap) {
                float4 *d4 = reinterpret_cast<float4 *>(dump + (size_t)at * NE);
#pragma unroll
                for (int g = 0; g < NE / 4; ++g) d4[g] = make_float4(x[4 * g], x[4 * g + 1], x[4 * g + 2], x[4 * g + 3]);
                s.dump_lane[at] = (unsigned short)tid;
            }
        }
    }
    __syncthreads();
    const int ndump = (int)s.ndump;
    if (ndump <= kDumpCap) {
        // The logits of the hot lanes against the threshold, all sixteen wavefronts side by side: a lane
        // takes one logit of one block; what passes goes to the workgroup's candidate list (its order is
        // immaterial, the ranking below is by key).
        constexpr int kPerWave = NE <= kWave ? kWave / NE : 1;     // blocks a wavefront takes at a time
        for (int d0 = w * kPerWave; d0 < ndump; d0 += kExpWaves * kPerWave) {
#pragma unroll
            for (int e1 = 0; e1 < NE; e1 += kWave) {               // (one round unless a lane streams more than 64 logits)
                const int d = d0 + (NE <= kWave ? lane / NE : 0);
                const int e = NE <= kWave ? lane % NE : e1 + lane;
                const bool live = d < ndump;
                const float v = dump[(size_t)min(d, ndump - 1) * NE + e];
                const int src = (int)s.dump_lane[min(d, ndump - 1)];
                const int idx = base + (e >> 2) * (kSLanes * 4) + src * 4 + (e & 3);
                const uint64_t m = __ballot(live && v >= tau_f && idx < a.V);
                if (m != 0) {
                    int at = 0;
                    if (lane == 0) at = (int)atomicAdd(&s.nsurv, (unsigned int)__popcll(m));
                    at = (int)readlane_u32((uint32_t)at, 0) + lanes_below(m);
                    if (((m >> lane) & 1) && at < kFastCap) surv[at] = make_key(v, uint32_t(idx));
                }
            }
        }
    }
    // more hot lanes or candidates than the lists hold means long runs of equal values (every
    // wavefront reads the same counts after the barrier and takes the same path)
    if (ndump > kDumpCap && tid == 0) s.nsurv = kFastCap + 1;
    __syncthreads();
    const size_t pslot = (size_t)f * a.nchunks + chunk;
    const int nsurv = (int)s.nsurv;
    if (nsurv > kFastCap) {
        // Long runs of equal values (more candidates than the list holds): every streaming wavefront
        // ranks its own logits exactly, eight per lane at a time with the selection so far riding
        // along, then one wavefront ranks the four lists.  The logits are read again (a rolled loop
        // over registers would index them dynamically); this path only runs on heavily tied rows.
        if (streamer) {
            uint64_t wt = 0;
#pragma unroll 1
            for (int g0 = 0; g0 < NE / 4; g0 += 2) {
                uint64_t kk[9];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int idx = base + (g0 + (u >> 2)) * (kSLanes * 4) + tid * 4 + (u & 3);
                    const float v = row[min(idx, a.V - 1)];
                    kk[u] = idx < a.V ? make_key(v, uint32_t(idx)) : 0;
                }
                kk[8] = wt;
                wt = wave_topk<9>(kk, K, s.wtk[w]);
            }
            if (lane < kWaveListSlots) s.wlist[w * kWaveListSlots + lane] = wt;   // lanes 16.. hold 0
        }
        __syncthreads();
        if (w == 0) {
            constexpr int NS = kStreamers * kWaveListSlots / kWave;   // four lists of 32 slots, two slots per lane
            uint64_t k2[NS];
#pragma unroll
            for (int e = 0; e < NS; ++e) k2[e] = s.wlist[e * kWave + lane];
            const uint64_t top = wave_topk<NS>(k2, K, s.wtk[0]);
            if (lane < K) store_shared_result(a.part_keys + pslot * RADAR_K_MAX + lane, top);
        }
    } else if (w == 0) {
        // exact ranks among the chunk's candidates: every lane counts the larger keys with broadcast reads
        if (lane < 8) surv[nsurv + lane] = 0;                      // padding for the grouped reads
        wave_lds_sync();
        for (int i0 = 0; i0 < nsurv; i0 += kWave) {                // one pass unless there are many ties
            const int i = i0 + lane;
            const uint64_t key = surv[min(i, nsurv - 1)];
            int rank = 0;
            for (int j = 0; j < nsurv; j += 8) {
                uint64_t kj[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) kj[u] = surv[j + u];
#pragma unroll
                for (int u = 0; u < 8; ++u) rank += (kj[u] > key) ? 1 : 0;
            }
            if (i < nsurv && rank < K) store_shared_result(a.part_keys + pslot * RADAR_K_MAX + rank, key);   // ranks are distinct
        }
        if (lane >= nsurv && lane < K) store_shared_result(a.part_keys + pslot * RADAR_K_MAX + lane, (uint64_t)0);   // fewer than K in the chunk
    }
    if (w == 1) {
        double l = 0.0;                                            // fixed order of addition
#pragma unroll
        for (int i = 0; i < kStreamers; ++i) l += (double)s.wave_l[i];
        if (lane == 0) {
            store_shared_result(&a.part_m[pslot], cm);
            store_shared_result(&a.part_l[pslot], l);
        }
    }
    unsigned int *row_counter = &a.counters[(1 + f) * kCounterStride];
    if (publish_then_ticket(row_counter, &s.ticket) != (unsigned int)(a.nchunks - 1)) return;

    // ---- last chunk of row f: the row is complete; count it.  Only the workgroup that completes
    // the last row goes on (its predecessors' partials were all acknowledged before their tickets).
    if (tid == 0) {
        store_shared_result(row_counter, 0u);                      // leave the row counter clean
        s.ticket2 = __hip_atomic_fetch_add(&a.counters[0], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (s.ticket2 != (unsigned int)(a.F - 1)) return;
    if (tid == 0) store_shared_result(&a.counters[0], 0u);

    // ================= last workgroup of the call
    expand_finish<EXT>(a, s, bz, cycle, cycle_first, [&](int row) { return load_shared_result(&a.gate_pre[row]); });
}

// ------------------------------------------------------------------ rerank
struct RerankArgs {
    const int32_t *pool_tokens;
    const float *pool_scores;
    const int32_t *pool_parents;
    int pool_count, N, root_token;
    const radar_cycle_state *cycle;   // or null; when set, pool_count is the state's, clamped to the value above
    const int32_t *root_tokens;       // batched call: one root token per sequence (else null: root_token)
    int pool_capacity;                // batched call: stride of the pool arrays
    int32_t *tree_tokens;
    int32_t *tree_parents;
    float *tree_scores;
    int32_t *tree_depth;
    int32_t *tree_pool_idx;
    int32_t *n_nodes_out;
};

constexpr int kRerankStaged = 4 * kTopkThreads;       // pools up to this size are copied to LDS whole

struct RerankSmem {
    TopkSmem topk;
    int16_t node_of[RADAR_POOL_MAX];     // pool index -> node number, -1 if dropped
    int32_t parent[RADAR_T_MAX];
    // small pools: tokens, parents and scores ride along with the first loads, so that the kept
    // entries are read from LDS instead of a second round trip to memory
    int32_t tok[kRerankStaged], par[kRerankStaged];
    float sc[kRerankStaged];
};

template <int EPT>                       // pool entries per lane: 4 (pools up to 1024) or 16
__global__ __launch_bounds__(kTopkThreads) void rerank_kernel(RerankArgs a) {
    __shared__ RerankSmem s;
    const int tid = threadIdx.x;
    if (blockIdx.x != 0) {                               // sequence b of a batched call: every array has a leading batch dimension
        const size_t b = blockIdx.x, n1 = (size_t)a.N + 1;
        a.pool_tokens += b * a.pool_capacity; a.pool_scores += b * a.pool_capacity; a.pool_parents += b * a.pool_capacity;
        a.tree_tokens += b * n1; a.tree_parents += b * n1; a.tree_scores += b * n1;
        a.tree_depth += b * n1; a.tree_pool_idx += b * n1;
        a.n_nodes_out += b;
        if (a.cycle) a.cycle += b;
    }
    if (a.root_tokens) a.root_token = a.root_tokens[blockIdx.x];
    if (a.cycle) a.pool_count = min(max(a.cycle->pool_count, 0), a.pool_count);
    const int keep = min(a.N, a.pool_count);

    constexpr bool kStaged = EPT * kTopkThreads <= kRerankStaged;
    uint64_t keys[EPT];
    if constexpr (kStaged) {
        float sc[EPT];
        int tk[EPT], pr[EPT];
#pragma unroll
        for (int e = 0; e < EPT; ++e) {                      // all loads first: one round trip
            const int i = max(0, min(tid + e * kTopkThreads, a.pool_count - 1));
            sc[e] = a.pool_scores[i]; tk[e] = a.pool_tokens[i]; pr[e] = a.pool_parents[i];
        }
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            const int i = tid + e * kTopkThreads;
            keys[e] = (i < a.pool_count) ? make_key(sc[e], uint32_t(i)) : 0;
            s.sc[i] = sc[e]; s.tok[i] = tk[e]; s.par[i] = pr[e];
        }
    } else {
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            const int i = tid + e * kTopkThreads;
            const float sc = a.pool_scores[max(0, min(i, a.pool_count - 1))];
            keys[e] = (i < a.pool_count) ? make_key(sc, uint32_t(i)) : 0;
        }
    }
    for (int i = tid; i < a.pool_count; i += kTopkThreads) s.node_of[i] = -1;
    if (keep > 0) block_topk<EPT>(keys, keep, s.topk);
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
            tok = kStaged ? s.tok[my_pool] : a.pool_tokens[my_pool];
            sc = kStaged ? s.sc[my_pool] : a.pool_scores[my_pool];
            pidx = my_pool;
            const int pp = kStaged ? s.par[my_pool] : a.pool_parents[my_pool];
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

// ------------------------------------------------------------------ large batches: stream, then finish
// For many sequences per call the single launch above is bound by what every workgroup does around
// its share of the stream (one workgroup per CU, hand-over and ticket per chunk).  Two launches
// instead: a streaming kernel of small workgroups (several per CU, out of step with each other)
// without tickets or hand-over -- a wavefront owns 1024 consecutive logits, the four of a workgroup
// meet once to leave one top-k list, maximum and sum of exponentials per 4096 logits in the
// workspace -- then one workgroup per sequence that does what the last workgroup of the single
// launch does.
constexpr int kStreamThreads = 256;
constexpr int kStreamWaves = kStreamThreads / kWave;
constexpr int kStreamWaveLogits = 1024;
constexpr int kStreamChunk = kStreamWaves * kStreamWaveLogits;

// true: the sequence's cycle has stopped (or its state is out of range) and the call leaves it alone
__device__ __forceinline__ bool cycle_skips(const radar_cycle_state *st, int pool_count_max, int *pool_count) {
    if (st == nullptr || pool_count_max == 0) return false;        // no cycle, or its first call
    const int pc = st->pool_count;
    if (st->stopped != 0 || pc < 0 || pc > pool_count_max) return true;
    *pool_count = pc;
    return false;
}

template <bool VEC4>
__global__ __launch_bounds__(kStreamThreads) void expand_stream_kernel(ExpandArgs a) {
    __shared__ WaveTopkSmem wtk[kStreamWaves];
    __shared__ uint64_t wlists[kStreamWaves][kWaveListSlots];
    __shared__ float wave_m[kStreamWaves];
    __shared__ double wave_l[kStreamWaves];
    const int lane = lane_id(), w = wave_id();
    const int row = blockIdx.y;                                    // sequence * F + frontier row
    int unused;
    if (cycle_skips(a.cycle ? a.cycle + row / a.F : nullptr, a.pool_count, &unused)) return;   // the whole workgroup
    // which 1024 logits of the row; a wavefront past the end of the row sees -inf only and leaves an empty list
    const int base = blockIdx.x * kStreamChunk + w * kStreamWaveLogits;
    const float *rowp = a.logits + (size_t)row * a.V;
    const int K = a.k;
    // The prediction model's input-free part (w_hh h) of this row's sequence is shared out over the
    // sequence's workgroups, eight rows each, as the single launch does; the finish kernel reads it.
    if (a.has_policy && a.pol_has_state) {
        const int bz = row / a.F;
        float *gate = a.gate_pre + (size_t)bz * (4 * kPolH);
        policy_hidden_rows<4, kStreamThreads / 32>(a.pol, bz, (row - bz * a.F) * gridDim.x + blockIdx.x, a.F * gridDim.x,
                                                   [&](int r, float v) { gate[r] = v; });
    }

    float4 raw[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const int idx0 = base + g * (kWave * 4) + lane * 4;
        if (VEC4) {
            raw[g] = *reinterpret_cast<const float4 *>(rowp + (idx0 < a.V ? idx0 : 0));
        } else {
            raw[g].x = rowp[min(idx0 + 0, a.V - 1)];
            raw[g].y = rowp[min(idx0 + 1, a.V - 1)];
            raw[g].z = rowp[min(idx0 + 2, a.V - 1)];
            raw[g].w = rowp[min(idx0 + 3, a.V - 1)];
        }
    }
    float x[16];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        x[4 * g + 0] = raw[g].x; x[4 * g + 1] = raw[g].y; x[4 * g + 2] = raw[g].z; x[4 * g + 3] = raw[g].w;
    }
    if (base + kStreamWaveLogits > a.V) {                          // wave-uniform: the row's last wavefront(s) only
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int idx = base + (e >> 2) * (kWave * 4) + lane * 4 + (e & 3);
            x[e] = idx < a.V ? x[e] : -INFINITY;
        }
    }
    float tm = x[0];
#pragma unroll
    for (int e = 1; e < 16; ++e) tm = fmaxf(tm, x[e]);
    const float wm = wave_max_f32(tm);
    float tl = 0.f;
    if (wm > -INFINITY) {
#pragma unroll
        for (int e = 0; e < 16; ++e) tl += __builtin_amdgcn_exp2f((x[e] - wm) * kLog2eF);
    }
    const double wl = wave_sum_f64((double)tl);

    // the wavefront's candidates (unranked; ranked only where more than 32 of them pass the threshold)
    {
        uint64_t *list = &wlists[w][0];
        if (!wave_candidates_counted<16>(x, tm, uint32_t(base + lane * 4), uint32_t(kWave * 4), uint32_t(a.V), K, list)) {
            uint64_t k1[8], k2[9];
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int idx = base + (e >> 2) * (kWave * 4) + lane * 4 + (e & 3);
                const uint64_t key = idx < a.V ? make_key(x[e], uint32_t(idx)) : 0;
                if (e < 8) k1[e] = key; else k2[e - 8] = key;
            }
            k2[8] = wave_topk<8>(k1, K, wtk[w]);
            const uint64_t wt = wave_topk<9>(k2, K, wtk[w]);
            if (lane < kWaveListSlots) list[lane] = wt;            // lanes 16.. hold 0
        }
    }
    if (lane == 0) { wave_m[w] = wm; wave_l[w] = wl; }
    __syncthreads();
    const size_t slot = (size_t)row * a.nchunks + blockIdx.x;
    if (w == 0) {                                                              // the chunk's list: top-k of the four lists
        constexpr int NS = kStreamWaves * kWaveListSlots / kWave;
        uint64_t kk[NS];
#pragma unroll
        for (int e = 0; e < NS; ++e) kk[e] = (&wlists[0][0])[topk_slot_of(e)];   // rotated: the used slots lead each list
        const uint64_t ctop = wave_topk<NS>(kk, K, wtk[0]);
        if (lane < RADAR_K_MAX) a.part_keys[slot * RADAR_K_MAX + lane] = ctop;    // 0 beyond the k-th
    } else if (w == 1 && lane == 0) {                                          // fixed order of addition
        float m = wave_m[0];
#pragma unroll
        for (int i = 1; i < kStreamWaves; ++i) m = fmaxf(m, wave_m[i]);
        double l = 0.0;
#pragma unroll
        for (int i = 0; i < kStreamWaves; ++i)
            if (wave_m[i] > -INFINITY) l += wave_l[i] * (double)__builtin_amdgcn_exp2f((wave_m[i] - m) * kLog2eF);
        a.part_m[slot] = m;
        a.part_l[slot] = l;
    }
}

// one workgroup per sequence, after expand_stream_kernel
__global__ __launch_bounds__(kExpThreads, 1) void expand_finish_kernel(ExpandArgs a) {
    __shared__ ExpandSmem s;
    const int bz = blockIdx.x;
    if (bz != 0) sequence_view(a, bz);
    radar_cycle_state *const cycle = a.cycle;
    const bool cycle_first = cycle != nullptr && a.pool_count == 0;
    if (cycle_skips(cycle, a.pool_count, &a.pool_count)) return;
    // (the prediction model's input-free part was left in the workspace by the streaming kernel)
    expand_finish<true>(a, s, bz, cycle, cycle_first, [&](int row) { return a.gate_pre[row]; });
}

}  // namespace radar

using namespace radar;

// Logits per lane: the fewest (shortest critical path per workgroup) that keep the launch at one
// workgroup per CU; launches too large for that take the most, i.e. the fewest workgroups.
static int plan_expand_ept(int F, int V) {
    for (int ept = kExpMinEPT; ept <= 16; ept *= 2) {
        const int64_t chunk = (int64_t)kExpThreads * ept;
        if ((int64_t)F * (((int64_t)V + chunk - 1) / chunk) <= 256) return ept;
    }
    return 16;
}

// Workspace of a call over B sequences: [B] counter blocks, [B][F][chunks] chunk lists, sums and maxima
// (sized for the most chunks any plan uses), [B] w_hh h of the fused prediction model.
static size_t expand_gate_bytes(size_t B) { return (B * 4 * kPolH * sizeof(float) + 255) & ~size_t(255); }

static size_t expand_workspace_bytes(const radar_expand_desc *d, size_t B) {
    if (!d || d->F < 1 || d->V < 1 || B < 1) return 0;
    static_assert(kStreamChunk == kExpThreads * kExpMinEPT, "both paths' smallest chunk");
    const size_t per_chunk = (size_t)kExpThreads * kExpMinEPT;                // most chunks any plan uses
    const size_t nchunks = ((size_t)d->V + per_chunk - 1) / per_chunk;
    size_t bytes = B * kCounterBytes;
    bytes += B * d->F * nchunks * RADAR_K_MAX * sizeof(uint64_t);
    bytes += B * d->F * nchunks * (sizeof(double) + sizeof(float));
    return ((bytes + 255) & ~size_t(255)) + expand_gate_bytes(B);
}

extern "C" size_t radar_draft_expand_workspace_bytes(const radar_expand_desc *d) { return expand_workspace_bytes(d, 1); }

extern "C" size_t radar_draft_expand_batch_workspace_bytes(const radar_expand_desc *d, int32_t B) {
    return B < 1 ? 0 : expand_workspace_bytes(d, (size_t)B);
}

namespace radar { radar_status policy_args_from(const radar_policy_params *pp, PolicyArgs *out); }

static radar_status launch_expand(const float *logits, const float *parent_scores,
                                  const int32_t *parent_pool_idx, int32_t *cand_tokens, float *cand_scores,
                                  int32_t *frontier_pool_idx, int32_t *frontier_tokens,
                                  float *frontier_scores, float *frontier_conf, int32_t *pool_tokens,
                                  float *pool_scores, int32_t *pool_parents, const radar_expand_desc *d,
                                  const PolicyArgs *pol, radar_cycle_state *cycle, int B, void *workspace,
                                  size_t workspace_bytes, void *stream_, bool check_only = false) {
    if (!d || !logits || !parent_scores || !parent_pool_idx || !cand_tokens || !cand_scores || !frontier_pool_idx ||
        !frontier_tokens || !frontier_scores || !frontier_conf || !pool_tokens || !pool_scores || !pool_parents ||
        !workspace)
        return RADAR_INVALID_ARG;
    if (d->F < 1 || d->V < 1 || d->k < 1 || d->k > d->V || d->pool_count < 0 ||
        (int64_t)d->pool_count + (int64_t)d->F * d->k > (int64_t)d->pool_capacity)
        return RADAR_INVALID_ARG;
    if (B < 1) return RADAR_INVALID_ARG;
    if (B > 65535) return RADAR_UNSUPPORTED_SHAPE;
    // Batches large enough to fill the chip several times over take the two-launch streaming path.
    const bool stream = B > 1 && (int64_t)B * d->F <= 65535 &&
                        (int64_t)B * d->F * d->V >= kStreamMinLogits;
    const int ept = plan_expand_ept((int)std::min<int64_t>((int64_t)d->F * B, 1 << 20), d->V);
    const int64_t chunk = stream ? kStreamChunk : (int64_t)kExpThreads * ept;
    const int64_t nchunks = ((int64_t)d->V + chunk - 1) / chunk;
    if (d->F > RADAR_F_MAX || d->k > RADAR_K_MAX || nchunks > kExpMaxChunks) return RADAR_UNSUPPORTED_SHAPE;
    if (workspace_bytes < expand_workspace_bytes(d, (size_t)B)) return RADAR_WORKSPACE_TOO_SMALL;
    if (((uintptr_t)workspace & 255) != 0) return RADAR_INVALID_ARG;
    if (check_only) return RADAR_OK;                               // every argument is acceptable; nothing launched

    ExpandArgs a;
    a.logits = logits; a.parent_scores = parent_scores; a.parent_pool_idx = parent_pool_idx;
    a.cand_tokens = cand_tokens; a.cand_scores = cand_scores;
    a.frontier_pool_idx = frontier_pool_idx; a.frontier_tokens = frontier_tokens;
    a.frontier_scores = frontier_scores; a.frontier_conf = frontier_conf;
    a.pool_tokens = pool_tokens; a.pool_scores = pool_scores; a.pool_parents = pool_parents;
    a.F = d->F; a.V = d->V; a.k = d->k; a.nchunks = (int)nchunks; a.pool_count = d->pool_count;
    a.pool_capacity = d->pool_capacity;
    char *ws = static_cast<char *>(workspace);
    const size_t nb = (size_t)B, cbytes = nb * kCounterBytes;
    a.counters = reinterpret_cast<unsigned int *>(ws);
    a.part_keys = reinterpret_cast<uint64_t *>(ws + cbytes);
    const size_t nslots = nb * d->F * nchunks;
    a.part_l = reinterpret_cast<double *>(ws + cbytes + nslots * RADAR_K_MAX * sizeof(uint64_t));
    a.part_m = reinterpret_cast<float *>(ws + cbytes + nslots * (RADAR_K_MAX * sizeof(uint64_t) + sizeof(double)));
    a.gate_pre = reinterpret_cast<float *>(ws + expand_workspace_bytes(d, nb) - expand_gate_bytes(nb));
    a.cycle = cycle;
    a.pol = pol ? *pol : PolicyArgs{};
    a.has_policy = pol ? 1 : 0;
    a.pol_has_state = (pol && pol->h_in) ? 1 : 0;

    const dim3 grid((unsigned)nchunks, (unsigned)d->F, (unsigned)B), block(kExpThreads);
    const bool vec4 = (d->V % 4 == 0) && (((uintptr_t)logits & 15) == 0);
    hipStream_t st = static_cast<hipStream_t>(stream_);
    hipError_t e;
    if (stream) {
        const dim3 sgrid((unsigned)nchunks, (unsigned)(B * d->F));
        e = vec4 ? launch("expand_stream", expand_stream_kernel<true>, sgrid, dim3(kStreamThreads), 0, st, a)
                 : launch("expand_stream", expand_stream_kernel<false>, sgrid, dim3(kStreamThreads), 0, st, a);
        if (e != hipSuccess) return RADAR_HIP_ERROR;
        e = launch("expand_finish", expand_finish_kernel, dim3((unsigned)B), block, 0, st, a);
        return e == hipSuccess ? RADAR_OK : RADAR_HIP_ERROR;
    }
    const bool ext = pol != nullptr || cycle != nullptr || B > 1;
#define RADAR_EXPAND_LAUNCH(V4, E)                                                                   \
    (ext ? launch("expand", expand_kernel<V4, E, true>, grid, block, 0, st, a)                        \
         : launch("expand", expand_kernel<V4, E, false>, grid, block, 0, st, a))
    if (ept == 4)      e = vec4 ? RADAR_EXPAND_LAUNCH(true, 4) : RADAR_EXPAND_LAUNCH(false, 4);
    else if (ept == 8) e = vec4 ? RADAR_EXPAND_LAUNCH(true, 8) : RADAR_EXPAND_LAUNCH(false, 8);
    else               e = vec4 ? RADAR_EXPAND_LAUNCH(true, 16) : RADAR_EXPAND_LAUNCH(false, 16);
#undef RADAR_EXPAND_LAUNCH
    return e == hipSuccess ? RADAR_OK : RADAR_HIP_ERROR;
}

extern "C" radar_status radar_draft_expand(const float *logits, const float *parent_scores,
                                           const int32_t *parent_pool_idx, int32_t *cand_tokens, float *cand_scores,
                                           int32_t *frontier_pool_idx, int32_t *frontier_tokens,
                                           float *frontier_scores, float *frontier_conf, int32_t *pool_tokens,
                                           float *pool_scores, int32_t *pool_parents, const radar_expand_desc *d,
                                           void *workspace, size_t workspace_bytes, void *stream) {
    return launch_expand(logits, parent_scores, parent_pool_idx, cand_tokens, cand_scores, frontier_pool_idx,
                         frontier_tokens, frontier_scores, frontier_conf, pool_tokens, pool_scores, pool_parents, d,
                         nullptr, nullptr, 1, workspace, workspace_bytes, stream);
}

// ------------------------------------------------------------------ the entry point that allocates nothing
// For callers that cannot call hipMalloc (code under HIP graph capture, tight serving loops,
// harnesses that forbid it): radar_draft_expand with its workspace in a device array of this
// library instead of a caller-owned buffer.  The array lives in every GPU the library runs on
// until the process ends; its device address is looked up once per device.
static __device__ __align__(256) unsigned char scratch[RADAR_NOALLOC_SCRATCH_BYTES];

namespace {
constexpr int kScratchMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kScratchMaxDevices];      // device address of `scratch` on each device; null until looked up

__global__ void scratch_clear_kernel(uint4 *p, size_t n16) {
    const uint4 z = make_uint4(0u, 0u, 0u, 0u);
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x) p[i] = z;
}

// The current device's copy of `scratch` (in host code the array's name is only a handle for the
// lookup, never an address).  The first call on a device also clears the array on `stream`: the
// arrival counters at its head must start at zero, and every call leaves them at zero.
radar_status static_scratch(hipStream_t stream, void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return RADAR_HIP_ERROR;
    if (dev < 0 || dev >= kScratchMaxDevices) return RADAR_UNSUPPORTED_SHAPE;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return RADAR_HIP_ERROR;
        if (((uintptr_t)ptr & 255) != 0) return RADAR_HIP_ERROR;
        hipLaunchKernelGGL(scratch_clear_kernel, dim3(64), dim3(256), 0, stream, static_cast<uint4 *>(ptr),
                           (size_t)RADAR_NOALLOC_SCRATCH_BYTES / 16);
        if (hipGetLastError() != hipSuccess) return RADAR_HIP_ERROR;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return RADAR_OK;
}
}  // namespace

extern "C" radar_status radar_draft_expand_noalloc(const float *logits, const float *parent_scores,
                                                   const int32_t *parent_pool_idx, int32_t *cand_tokens,
                                                   float *cand_scores, int32_t *frontier_pool_idx,
                                                   int32_t *frontier_tokens, float *frontier_scores,
                                                   float *frontier_conf, int32_t *pool_tokens, float *pool_scores,
                                                   int32_t *pool_parents, const radar_expand_desc *d, void *stream) {
    if (!d || d->F < 1 || d->V < 1) return RADAR_INVALID_ARG;
    const size_t need = expand_workspace_bytes(d, 1);
    if (need == 0 || need > (size_t)RADAR_NOALLOC_SCRATCH_BYTES) return RADAR_UNSUPPORTED_SHAPE;   // F * V beyond the array
    // arguments first (against a stand-in for the array's address), so that an error launches nothing
    radar_status st = launch_expand(logits, parent_scores, parent_pool_idx, cand_tokens, cand_scores, frontier_pool_idx,
                                    frontier_tokens, frontier_scores, frontier_conf, pool_tokens, pool_scores,
                                    pool_parents, d, nullptr, nullptr, 1, reinterpret_cast<void *>(uintptr_t(256)),
                                    (size_t)RADAR_NOALLOC_SCRATCH_BYTES, stream, true);
    if (st != RADAR_OK) return st;
    void *ws = nullptr;
    st = static_scratch(static_cast<hipStream_t>(stream), &ws);
    if (st != RADAR_OK) return st;
    return launch_expand(logits, parent_scores, parent_pool_idx, cand_tokens, cand_scores, frontier_pool_idx,
                         frontier_tokens, frontier_scores, frontier_conf, pool_tokens, pool_scores, pool_parents, d,
                         nullptr, nullptr, 1, ws, (size_t)RADAR_NOALLOC_SCRATCH_BYTES, stream);
}

extern "C" radar_status radar_draft_expand_policy(const float *logits, const float *parent_scores,
                                                  const int32_t *parent_pool_idx, int32_t *cand_tokens,
                                                  float *cand_scores, int32_t *frontier_pool_idx,
                                                  int32_t *frontier_tokens, float *frontier_scores,
                                                  float *frontier_conf, int32_t *pool_tokens, float *pool_scores,
                                                  int32_t *pool_parents, const radar_expand_desc *d,
                                                  const radar_policy_params *params, const radar_policy_io *io,
                                                  void *workspace, size_t workspace_bytes, void *stream) {
    PolicyArgs pa;
    const radar_status st = policy_args_from(params, &pa);
    if (st != RADAR_OK) return st;
    if (!d || !io || !io->h_out || !io->c_out || !io->logits || !io->probs || !io->action) return RADAR_INVALID_ARG;
    if ((io->h_in == nullptr) != (io->c_in == nullptr) || ((uintptr_t)io->h_in & 15) != 0) return RADAR_INVALID_ARG;
    if (params->k != d->k) return RADAR_INVALID_ARG;               // the model reads exactly the k confidences
    pa.h_in = io->h_in; pa.c_in = io->c_in; pa.uniforms = io->uniform;
    pa.h_out = io->h_out; pa.c_out = io->c_out; pa.logits = io->logits; pa.probs = io->probs; pa.action = io->action;
    return launch_expand(logits, parent_scores, parent_pool_idx, cand_tokens, cand_scores, frontier_pool_idx,
                         frontier_tokens, frontier_scores, frontier_conf, pool_tokens, pool_scores, pool_parents, d,
                         &pa, nullptr, 1, workspace, workspace_bytes, stream);
}

// fill kernel for the cycle state (a graph may not hold a memset node)
__global__ void cycle_begin_kernel(radar_cycle_state *st) {
    if (threadIdx.x == 0) { st->stopped = 0; st->pool_count = 0; st->steps_done = 0; st->last_action = -1; }
}

extern "C" radar_status radar_cycle_begin(radar_cycle_state *state, void *stream) {
    if (!state) return RADAR_INVALID_ARG;
    const hipError_t e = launch("cycle_begin", cycle_begin_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream), state);
    return e == hipSuccess ? RADAR_OK : RADAR_HIP_ERROR;
}

extern "C" radar_status radar_draft_expand_cycle(const float *logits, const float *parent_scores,
                                                 const int32_t *parent_pool_idx, int32_t *cand_tokens,
                                                 float *cand_scores, int32_t *frontier_pool_idx,
                                                 int32_t *frontier_tokens, float *frontier_scores,
                                                 float *frontier_conf, int32_t *pool_tokens, float *pool_scores,
                                                 int32_t *pool_parents, const radar_expand_desc *d,
                                                 const radar_policy_params *params, const radar_policy_io *io,
                                                 radar_cycle_state *state, void *workspace, size_t workspace_bytes,
                                                 void *stream) {
    if (!state || !d) return RADAR_INVALID_ARG;
    if (!params) {
        if (io) return RADAR_INVALID_ARG;
        return launch_expand(logits, parent_scores, parent_pool_idx, cand_tokens, cand_scores, frontier_pool_idx,
                             frontier_tokens, frontier_scores, frontier_conf, pool_tokens, pool_scores, pool_parents, d,
                             nullptr, state, 1, workspace, workspace_bytes, stream);
    }
    PolicyArgs pa;
    const radar_status st = policy_args_from(params, &pa);
    if (st != RADAR_OK) return st;
    if (!io || !io->h_out || !io->c_out || !io->logits || !io->probs || !io->action) return RADAR_INVALID_ARG;
    if ((io->h_in == nullptr) != (io->c_in == nullptr) || ((uintptr_t)io->h_in & 15) != 0) return RADAR_INVALID_ARG;
    if (params->k != d->k) return RADAR_INVALID_ARG;
    pa.h_in = io->h_in; pa.c_in = io->c_in; pa.uniforms = io->uniform;
    pa.h_out = io->h_out; pa.c_out = io->c_out; pa.logits = io->logits; pa.probs = io->probs; pa.action = io->action;
    return launch_expand(logits, parent_scores, parent_pool_idx, cand_tokens, cand_scores, frontier_pool_idx,
                         frontier_tokens, frontier_scores, frontier_conf, pool_tokens, pool_scores, pool_parents, d,
                         &pa, state, 1, workspace, workspace_bytes, stream);
}

extern "C" radar_status radar_draft_expand_batch(const float *logits, const float *parent_scores,
                                                 const int32_t *parent_pool_idx, int32_t *cand_tokens,
                                                 float *cand_scores, int32_t *frontier_pool_idx,
                                                 int32_t *frontier_tokens, float *frontier_scores,
                                                 float *frontier_conf, int32_t *pool_tokens, float *pool_scores,
                                                 int32_t *pool_parents, const radar_expand_desc *d, int32_t B,
                                                 const radar_policy_params *params, const radar_policy_io *io,
                                                 radar_cycle_state *states, void *workspace, size_t workspace_bytes,
                                                 void *stream) {
    if (!d) return RADAR_INVALID_ARG;
    if (!params) {
        if (io) return RADAR_INVALID_ARG;
        return launch_expand(logits, parent_scores, parent_pool_idx, cand_tokens, cand_scores, frontier_pool_idx,
                             frontier_tokens, frontier_scores, frontier_conf, pool_tokens, pool_scores, pool_parents, d,
                             nullptr, states, B, workspace, workspace_bytes, stream);
    }
    PolicyArgs pa;
    const radar_status st = policy_args_from(params, &pa);
    if (st != RADAR_OK) return st;
    if (!io || !io->h_out || !io->c_out || !io->logits || !io->probs || !io->action) return RADAR_INVALID_ARG;
    if ((io->h_in == nullptr) != (io->c_in == nullptr) || ((uintptr_t)io->h_in & 15) != 0) return RADAR_INVALID_ARG;
    if (params->k != d->k) return RADAR_INVALID_ARG;
    pa.h_in = io->h_in; pa.c_in = io->c_in; pa.uniforms = io->uniform;
    pa.h_out = io->h_out; pa.c_out = io->c_out; pa.logits = io->logits; pa.probs = io->probs; pa.action = io->action;
    return launch_expand(logits, parent_scores, parent_pool_idx, cand_tokens, cand_scores, frontier_pool_idx,
                         frontier_tokens, frontier_scores, frontier_conf, pool_tokens, pool_scores, pool_parents, d,
                         &pa, states, B, workspace, workspace_bytes, stream);
}

extern "C" size_t radar_draft_rerank_workspace_bytes(int32_t pool_count, int32_t N) {
    (void)pool_count; (void)N;
    return 256;   // rerank keeps everything in LDS; a minimal workspace keeps the calling convention uniform
}

static radar_status launch_rerank(const int32_t *pool_tokens, const float *pool_scores, const int32_t *pool_parents,
                                  int32_t pool_count, const radar_cycle_state *cycle, int32_t N, int32_t root_token,
                                  int32_t *tree_tokens, int32_t *tree_parents, float *tree_scores,
                                  int32_t *tree_depth, int32_t *tree_pool_idx, int32_t *n_nodes_out, void *stream,
                                  int32_t B = 1, const int32_t *root_tokens = nullptr, int32_t pool_capacity = 0) {
    if (!pool_tokens || !pool_scores || !pool_parents || !tree_tokens || !tree_parents || !tree_scores ||
        !tree_depth || !tree_pool_idx || !n_nodes_out)
        return RADAR_INVALID_ARG;
    if (pool_count < 0 || N < 0) return RADAR_INVALID_ARG;
    if (pool_count > RADAR_POOL_MAX || N >= RADAR_T_MAX) return RADAR_UNSUPPORTED_SHAPE;
    if (B < 1 || (B > 1 && pool_capacity < pool_count)) return RADAR_INVALID_ARG;
    RerankArgs a;
    a.root_tokens = root_tokens; a.pool_capacity = pool_capacity;
    a.pool_tokens = pool_tokens; a.pool_scores = pool_scores; a.pool_parents = pool_parents;
    a.pool_count = pool_count; a.N = N; a.root_token = root_token; a.cycle = cycle;
    a.tree_tokens = tree_tokens; a.tree_parents = tree_parents; a.tree_scores = tree_scores;
    a.tree_depth = tree_depth; a.tree_pool_idx = tree_pool_idx; a.n_nodes_out = n_nodes_out;
    const hipError_t e = pool_count <= 4 * kTopkThreads
        ? launch("rerank", rerank_kernel<4>, dim3((unsigned)B), dim3(kTopkThreads), 0, static_cast<hipStream_t>(stream), a)
        : launch("rerank", rerank_kernel<16>, dim3((unsigned)B), dim3(kTopkThreads), 0, static_cast<hipStream_t>(stream), a);
    return e == hipSuccess ? RADAR_OK : RADAR_HIP_ERROR;
}

extern "C" radar_status radar_draft_rerank(const int32_t *pool_tokens, const float *pool_scores,
                                           const int32_t *pool_parents, int32_t pool_count, int32_t N,
                                           int32_t root_token, int32_t *tree_tokens, int32_t *tree_parents,
                                           float *tree_scores, int32_t *tree_depth, int32_t *tree_pool_idx,
                                           int32_t *n_nodes_out, void *workspace, size_t workspace_bytes,
                                           void *stream) {
    (void)workspace; (void)workspace_bytes;
    return launch_rerank(pool_tokens, pool_scores, pool_parents, pool_count, nullptr, N, root_token, tree_tokens,
                         tree_parents, tree_scores, tree_depth, tree_pool_idx, n_nodes_out, stream);
}

extern "C" radar_status radar_draft_rerank_cycle(const int32_t *pool_tokens, const float *pool_scores,
                                                 const int32_t *pool_parents, const radar_cycle_state *state,
                                                 int32_t pool_count_max, int32_t N, int32_t root_token,
                                                 int32_t *tree_tokens, int32_t *tree_parents, float *tree_scores,
                                                 int32_t *tree_depth, int32_t *tree_pool_idx, int32_t *n_nodes_out,
                                                 void *workspace, size_t workspace_bytes, void *stream) {
    (void)workspace; (void)workspace_bytes;
    if (!state) return RADAR_INVALID_ARG;
    return launch_rerank(pool_tokens, pool_scores, pool_parents, pool_count_max, state, N, root_token, tree_tokens,
                         tree_parents, tree_scores, tree_depth, tree_pool_idx, n_nodes_out, stream);
}

extern "C" radar_status radar_draft_rerank_batch(const int32_t *pool_tokens, const float *pool_scores,
                                                 const int32_t *pool_parents, const radar_cycle_state *states,
                                                 int32_t pool_count, int32_t pool_capacity, int32_t B, int32_t N,
                                                 const int32_t *root_tokens, int32_t *tree_tokens,
                                                 int32_t *tree_parents, float *tree_scores, int32_t *tree_depth,
                                                 int32_t *tree_pool_idx, int32_t *n_nodes_out, void *workspace,
                                                 size_t workspace_bytes, void *stream) {
    (void)workspace; (void)workspace_bytes;
    if (!root_tokens || B < 1 || pool_capacity < 0 || pool_count > pool_capacity) return RADAR_INVALID_ARG;
    if (B > 65535) return RADAR_UNSUPPORTED_SHAPE;
    return launch_rerank(pool_tokens, pool_scores, pool_parents, pool_count, states, N, 0, tree_tokens, tree_parents,
                         tree_scores, tree_depth, tree_pool_idx, n_nodes_out, stream, B, root_tokens, pool_capacity);
}
