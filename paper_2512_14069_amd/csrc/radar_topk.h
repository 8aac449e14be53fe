// Workgroup-wide selection of the K largest 64-bit keys held in registers.
//
// Used by draft expansion (per-chunk top-k, per-row merge, frontier choice) and
// by rerank.  A key is (monotone image of an fp32 value) << 32 | ~index, so the
// larger key wins under "value descending, index ascending"; key 0 means
// "no element".  256 threads, four 64-wide wavefronts.
//
// Method.  Each wavefront first finds a threshold tau on the 32-bit value part:
// the K-th largest of its 64 per-lane maxima (at most K rounds of a DPP maximum
// with the winners struck out).  At least K of the wavefront's elements are
// >= tau, and on non-degenerate data few more, so only those "survivors" are
// compacted (ballot + prefix count) into LDS and ranked exactly by counting.
// The four wavefront lists (4*K <= 256 keys) are then ranked the same way.
// Every step is exact; thresholds only limit how much is ranked.
#pragma once

#include "radar_device.h"

namespace radar {

constexpr int kTopkThreads = 256;
constexpr int kTopkWaves = kTopkThreads / kWave;
constexpr int kTopkMaxK = 64;
constexpr int kTopkMaxEPT = 16;

struct TopkSmem {
    uint64_t surv[kTopkWaves][kTopkMaxEPT * kWave];   // survivors of each wavefront
    uint64_t wtop[kTopkWaves][kTopkMaxK];             // each wavefront's best K
    uint64_t top[kTopkMaxK];                          // result, best first; 0 where fewer than K exist
};

// keys[e] == 0 marks an absent element.  All 256 threads must call this
// (it synchronises the workgroup).  On return s.top[0..K) is valid for every
// thread.  1 <= K <= kTopkMaxK, EPT <= kTopkMaxEPT.
template <int EPT>
__device__ __forceinline__ void block_topk(const uint64_t (&keys)[EPT], int K, TopkSmem &s) {
    const int lane = lane_id(), w = wave_id();

    uint32_t tmax = 0;
#pragma unroll
    for (int e = 0; e < EPT; ++e) tmax = max(tmax, uint32_t(keys[e] >> 32));

    uint32_t cand = tmax, tau = 1;
    int remaining = K;
    for (int round = 0; round < kTopkMaxK; ++round) {       // wave-uniform loop, <= K rounds
        const uint32_t t = wave_max_u32(cand);
        if (t == 0) { tau = 1; break; }                     // fewer than K lanes hold anything
        tau = t;
        const uint64_t eq = __ballot(cand == t);
        remaining -= __popcll(eq);
        if (remaining <= 0) break;
        if (cand == t) cand = 0;
    }

    int n = 0;
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        const bool keep = uint32_t(keys[e] >> 32) >= tau;   // tau >= 1, so absent keys never pass
        const uint64_t m = __ballot(keep);
        if (m) {
            if (keep) s.surv[w][n + lanes_below(m)] = keys[e];
            n += __popcll(m);
        }
    }
    if (lane < kTopkMaxK) s.wtop[w][lane] = 0;
    if (threadIdx.x < kTopkMaxK) s.top[threadIdx.x] = 0;
    __syncthreads();

    for (int i = lane; i < n; i += kWave) {
        const uint64_t key = s.surv[w][i];
        int rank = 0;
        for (int j = 0; j < n; ++j) rank += (s.surv[w][j] > key) ? 1 : 0;
        if (rank < K) s.wtop[w][rank] = key;
    }
    __syncthreads();

    {
        const int ww = threadIdx.x >> 6, r = threadIdx.x & 63;
        const uint64_t key = (r < K) ? s.wtop[ww][r] : 0;
        if (key != 0) {
            int rank = 0;
            for (int w2 = 0; w2 < kTopkWaves; ++w2)
                for (int j = 0; j < K; ++j) rank += (s.wtop[w2][j] > key) ? 1 : 0;
            if (rank < K) s.top[rank] = key;
        }
    }
    __syncthreads();
}

}  // namespace radar
