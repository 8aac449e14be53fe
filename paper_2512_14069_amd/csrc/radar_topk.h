// Selection of the K largest 64-bit keys held in registers, by a workgroup (rerank) or by one
// wavefront (draft expansion).
//
// A key is (monotone image of an fp32 value) << 32 | ~index, so the larger key wins under
// "value descending, index ascending"; key 0 means "no element".
//
// Method: find a threshold tau that at least K elements reach, cheaply and without looking at
// every element pair; compact the elements >= tau into LDS (ballot + prefix count); rank those
// survivors exactly by counting larger keys with broadcast LDS reads.  Every step is exact; the
// threshold only limits how much is ranked.  Data with huge runs of equal values makes
// everything survive and is ranked by the same code in a slower loop.
#pragma once

#include "radar_device.h"

namespace radar {

constexpr int kTopkThreads = 256;
constexpr int kTopkWaves = kTopkThreads / kWave;
constexpr int kTopkMaxK = 64;
constexpr int kTopkMaxEPT = 16;

struct TopkSmem {
    uint64_t surv[kTopkThreads * kTopkMaxEPT + 8];    // compacted survivors (+8: grouped reads past the end)
    uint64_t top[kTopkMaxK];                          // result, best first; 0 where fewer than K exist
    uint32_t lmax[kTopkThreads];                      // largest value of each lane
    uint32_t tau;
    int count;                                        // number of survivors
};

// Workgroup version, 256 lanes, 1 <= K <= 64, EPT <= 16 keys per lane.  tau = the K-th largest
// of the 256 lane maxima (each lane ranks its maximum against all of them).  keys[e] == 0 marks
// an absent element.  All 256 threads must call this (it synchronises the workgroup).  On
// return s.top[0..K) is valid for every thread.
template <int EPT>
__device__ __forceinline__ void block_topk(const uint64_t (&keys)[EPT], int K, TopkSmem &s) {
    const int tid = threadIdx.x, lane = lane_id();

    uint32_t tmax = 0;
#pragma unroll
    for (int e = 0; e < EPT; ++e) tmax = max(tmax, uint32_t(keys[e] >> 32));
    s.lmax[tid] = tmax;
    if (tid == 0) { s.count = 0; s.tau = 0xffffffffu; }
    if (tid < kTopkMaxK) s.top[tid] = 0;
    __syncthreads();

    // ---- tau: smallest lane maximum that fewer than K lane maxima exceed
    {
        int larger = 0;
        for (int j = 0; j < kTopkThreads; j += 16) {              // broadcast reads, 16 values in flight
            uint32_t v[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) v[u] = s.lmax[j + u];
#pragma unroll
            for (int u = 0; u < 16; ++u) larger += (v[u] > tmax) ? 1 : 0;
        }
        uint32_t c = larger < K ? tmax : 0xffffffffu;
        c = min(c, dpp_u32<0xB1>(c));
        c = min(c, dpp_u32<0x4E>(c));
        c = min(c, dpp_u32<0x141>(c));
        c = min(c, dpp_u32<0x140>(c));
        const uint32_t wmin = min(min(readlane_u32(c, 0), readlane_u32(c, 16)), min(readlane_u32(c, 32), readlane_u32(c, 48)));
        if (lane == 0) atomicMin(&s.tau, wmin);
    }
    __syncthreads();
    const uint32_t tau = max(s.tau, 1u);                          // >= 1 so that absent keys (0) never pass

    // ---- compaction: count, reserve a range per wavefront, write
    int cnt = 0;
#pragma unroll
    for (int e = 0; e < EPT; ++e) cnt += __popcll(__ballot(uint32_t(keys[e] >> 32) >= tau));
    int base = 0;
    if (lane == 0 && cnt > 0) base = atomicAdd(&s.count, cnt);
    base = (int)readlane_u32((uint32_t)base, 0);
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        const bool keep = uint32_t(keys[e] >> 32) >= tau;
        const uint64_t m = __ballot(keep);
        if (m) {
            if (keep) s.surv[base + lanes_below(m)] = keys[e];
            base += __popcll(m);
        }
    }
    __syncthreads();
    const int n = s.count;
    if (tid < 8) s.surv[n + tid] = 0;                             // padding for the grouped reads
    __syncthreads();

    // ---- exact ranks among the n survivors; all lanes read the same LDS words (broadcast)
    for (int i = tid; i < n; i += kTopkThreads) {
        const uint64_t key = s.surv[i];
        int rank = 0;
        for (int j = 0; j < n; j += 8) {
            uint64_t kj[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) kj[u] = s.surv[j + u];
#pragma unroll
            for (int u = 0; u < 8; ++u) rank += (kj[u] > key) ? 1 : 0;
        }
        if (rank < K) s.top[rank] = key;
    }
    __syncthreads();
}

// ---------------------------------------------------------------------------------------------
// The same selection inside ONE wavefront, without workgroup barriers: K <= 16 largest of the
// 64 * EPL keys its lanes hold.  The 16 quads of the wavefront are the groups (tau = K-th
// largest quad maximum, so at least K keys pass; callers spread their keys over the quads, or
// few quads hold anything and tau filters little), survivors are compacted into the
// wavefront's private LDS scratch and ranked exactly.  Returns the r-th largest key in lane r
// (r < 16; 0 where fewer exist, and in lanes >= 16).  Callers on different wavefronts pass
// different scratch; all 64 lanes must call.
constexpr int kWaveTopkMaxEPL = 9;

// Threshold for a selection of the K <= 16 largest values held by the lanes of one wavefront
// (v = largest value of the lane, 0 if it holds none): the K-th largest of the 16 quad maxima.
// At least K values are >= the result (one per quad that reaches it), and unlike the smallest
// quad maximum it does not collapse when a few quads happen to hold only small values.
// Never 0, so that absent entries (0) fail the test "value >= threshold".
__device__ __forceinline__ uint32_t quad_threshold(uint32_t v, int K) {
    uint32_t g = v;
    g = max(g, dpp_u32<0xB1>(g));
    g = max(g, dpp_u32<0x4E>(g));                 // quad maximum in every lane of the quad
    int larger = 0;                               // quads whose maximum is strictly larger than this lane's
#pragma unroll
    for (int q = 0; q < 16; ++q) larger += (readlane_u32(g, 4 * q) > g) ? 1 : 0;
    uint32_t c = larger < K ? g : 0xffffffffu;    // the K largest quad maxima (and their ties) stay
    c = min(c, dpp_u32<0x141>(c));
    c = min(c, dpp_u32<0x140>(c));                // smallest of them within the 16-lane row
    const uint32_t t = min(min(readlane_u32(c, 0), readlane_u32(c, 16)), min(readlane_u32(c, 32), readlane_u32(c, 48)));
    return max(t, 1u);
}


struct WaveTopkSmem {
    uint64_t surv[kWave * kWaveTopkMaxEPL + 8];   // +8: the ranking reads keys eight at a time
    uint64_t top[16];
};

template <int EPL>
__device__ __forceinline__ uint64_t wave_topk(const uint64_t (&keys)[EPL], int K, WaveTopkSmem &s) {
    static_assert(EPL <= kWaveTopkMaxEPL, "scratch too small");
    const int lane = lane_id();
    uint32_t tmax = 0;
#pragma unroll
    for (int e = 0; e < EPL; ++e) tmax = max(tmax, uint32_t(keys[e] >> 32));
    const uint32_t tau = quad_threshold(tmax, K);

    int n = 0;                                    // survivors so far (wave-uniform)
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
        const bool keep = uint32_t(keys[e] >> 32) >= tau;
        const uint64_t m = __ballot(keep);
        if (keep) s.surv[n + lanes_below(m)] = keys[e];
        n += __popcll(m);
    }
    if (lane < 8) s.surv[n + lane] = 0;           // padding for the grouped reads
    if (lane < 16) s.top[lane] = 0;
    wave_lds_sync();
    for (int i0 = 0; i0 < n; i0 += kWave) {       // one pass unless nearly everything survived
        const int i = i0 + lane;
        const uint64_t key = s.surv[min(i, n - 1)];
        int rank = 0;
        for (int j = 0; j < n; j += 8) {          // broadcast reads (every lane reads the same keys),
            uint64_t kj[8];                       // eight in flight so that their latencies overlap
#pragma unroll
            for (int u = 0; u < 8; ++u) kj[u] = s.surv[j + u];
#pragma unroll
            for (int u = 0; u < 8; ++u) rank += (kj[u] > key) ? 1 : 0;
        }
        if (i < n && rank < K) s.top[rank] = key;
    }
    wave_lds_sync();
    const uint64_t r = s.top[lane & 15];
    wave_lds_sync();                              // scratch may be reused right after the return
    return lane < 16 ? r : 0;
}

// Candidates for a later selection, without ranking them: every element of the wavefront whose value
// reaches tau = the K-th largest quad maximum (so the wavefront's K largest are among them), as
// proper keys in list[0..32), 0 where there are fewer.  x[e] is element e of the lane (-inf where it
// lies past the row), its index is idx0 + (e / 4) * gstride + e % 4, indices of a lane ascend with
// e.  Keys are only built for the survivors (about K + 4 of them on random data).  Returns false,
// with list untouched, when more than 32 survive (long runs of equal values): the caller then
// ranks with wave_topk.  All 64 lanes must call; list is wavefront-private LDS.
constexpr int kWaveListSlots = 32;

template <int EPL>
__device__ __forceinline__ bool wave_candidates(const float (&x)[EPL], float lane_max, uint32_t idx0, uint32_t gstride,
                                                uint32_t V, int K, WaveTopkSmem &s, uint64_t *list) {
    static_assert(EPL <= kWaveTopkMaxEPL, "scratch too small");
    const int lane = lane_id();
    // a lane with no element inside the row counts as empty (0), not as a lane holding -inf
    const uint32_t tau = quad_threshold(idx0 < V ? ord_of(lane_max) : 0u, K);
    // as a float; thresholds at or below the image of -inf let every element of the row pass
    const float tau_f = tau < 0x00800000u ? -INFINITY : float_of_ord(tau);
    int n = 0;
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
        const uint32_t idx = idx0 + (uint32_t)(e >> 2) * gstride + (uint32_t)(e & 3);
        const bool keep = x[e] >= tau_f && idx < V;
        const uint64_t m = __ballot(keep);
        if (keep) s.surv[n + lanes_below(m)] = (uint64_t(__float_as_uint(x[e])) << 32) | idx;
        n += __popcll(m);
    }
    if (n > kWaveListSlots) return false;
    wave_lds_sync();
    if (lane < kWaveListSlots) {
        const uint64_t raw = s.surv[min(lane, max(n - 1, 0))];
        list[lane] = lane < n ? make_key(__uint_as_float(uint32_t(raw >> 32)), uint32_t(raw)) : 0;
    }
    wave_lds_sync();                              // scratch may be reused right after the return
    return true;
}

// The same for up to 16 elements per lane with the same small scratch: the survivors are counted
// first (comparison masks stay in scalar registers) and compacted only if they fit the list.
template <int EPL>
__device__ __forceinline__ bool wave_candidates_counted(const float (&x)[EPL], float lane_max, uint32_t idx0, uint32_t gstride,
                                                        uint32_t V, int K, uint64_t *list) {
    static_assert(EPL <= 16, "masks");
    const int lane = lane_id();
    const uint32_t tau = quad_threshold(idx0 < V ? ord_of(lane_max) : 0u, K);
    const float tau_f = tau < 0x00800000u ? -INFINITY : float_of_ord(tau);
    uint64_t m[EPL];
    int total = 0;
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
        const uint32_t idx = idx0 + (uint32_t)(e >> 2) * gstride + (uint32_t)(e & 3);
        m[e] = __ballot(x[e] >= tau_f && idx < V);
        total += __popcll(m[e]);
    }
    if (total > kWaveListSlots) return false;
    if (lane < kWaveListSlots) list[lane] = 0;
    wave_lds_sync();
    int n = 0;
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
        const uint32_t idx = idx0 + (uint32_t)(e >> 2) * gstride + (uint32_t)(e & 3);
        if ((m[e] >> lane) & 1) list[n + lanes_below(m[e])] = make_key(x[e], idx);
        n += __popcll(m[e]);
    }
    return true;
}

// Lists of 16 slots of which the first K are used (slot i: list i / 16, rank i % 16), taken 64
// slots per step: which slot a lane takes at step e.  Lanes rotate by 4 per step, so a lane
// meets slots of different ranks and every quad of lanes holds used slots.
__device__ __forceinline__ int topk_slot_of(int e) {
    return e * kWave + ((lane_id() + 4 * e) & (kWave - 1));
}

}  // namespace radar
