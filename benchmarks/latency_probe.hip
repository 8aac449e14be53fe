// Latency probe for gfx950 (MI355X): what the building blocks of the single-launch kernels cost.
//
// The 8B-shaped calls of this library are chains of dependent steps (a cold load, a wavefront-wide
// selection, a hand-over between workgroups, ...), not streams, so their time is the sum of such
// latencies.  This program measures them: one workgroup of 1, 4 or 16 wavefronts repeats a pattern
// 2000 times between two reads of the core clock; it prints core cycles per repetition for the
// first wavefront and for the slowest one (how well several wavefronts per SIMD hide the latency).
//
//   hipcc --offload-arch=gfx950 -O3 -std=c++17 -Xclang -target-feature -Xclang -packed-fp32-ops \
//         benchmarks/latency_probe.hip -o benchmarks/latency_probe && ./benchmarks/latency_probe
//
// A summary of one run is in profiles/gfx950_latency_probe.txt.
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdint.h>
#include <vector>
#include <string>

#define CHECK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); return 1; } } while (0)

struct Res { unsigned long long cyc, wall; float sink; unsigned long long tend[16]; unsigned long long tbeg; };

template <int CTRL> __device__ __forceinline__ float dppf(float v) {
    return __uint_as_float((uint32_t)__builtin_amdgcn_update_dpp((int)__float_as_uint(v), (int)__float_as_uint(v), CTRL, 0xF, 0xF, false));
}

template <int PAT>
__global__ void k(Res *out, int N, float seed, unsigned int *gmem) {
    __shared__ float lds[4096];
    __shared__ unsigned int cnt;
    const int lane = threadIdx.x & 63;
    float a = seed + lane * 0.001f, b = seed * 0.5f, c = seed * 0.25f, d = seed * 0.125f;
    int acc = 0;
    lds[threadIdx.x] = a;
    if (threadIdx.x == 0) cnt = 0;
    __syncthreads();
    unsigned long long t0 = clock64(), w0 = wall_clock64();
    for (int i = 0; i < N; ++i) {
        if (PAT == 0) {            // dependent fp32 add chain, 16 per iteration
#pragma unroll
            for (int u = 0; u < 16; ++u) a = a + b;
        } else if (PAT == 1) {     // four independent chains
#pragma unroll
            for (int u = 0; u < 4; ++u) { a += seed; b += seed; c += seed; d += seed; }
        } else if (PAT == 2) {     // dependent exp2 chain
#pragma unroll
            for (int u = 0; u < 16; ++u) a = __builtin_amdgcn_exp2f(a) - 1.0f;
        } else if (PAT == 3) {     // independent exps (4 chains): (x - m) * c, exp2, add
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                a += __builtin_amdgcn_exp2f((b - seed) * 1.44f); b += 0.001f;
                c += __builtin_amdgcn_exp2f((d - seed) * 1.44f); d += 0.001f;
            }
        } else if (PAT == 4) {     // ballot + popcount accumulate, 16 per iteration
#pragma unroll
            for (int u = 0; u < 16; ++u) { acc += __popcll(__ballot(a >= b + u)); }
            a += 0.5f;
        } else if (PAT == 5) {     // readlane + compare + count, 16 per iteration
            const uint32_t ov = __float_as_uint(a);
            int larger = 0;
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                const uint32_t oj = (uint32_t)__builtin_amdgcn_readlane((int)ov, j);
                larger += (oj > ov || (oj == ov && j < (lane & 15))) ? 1 : 0;
            }
            acc += larger; a += 1.0f;
        } else if (PAT == 6) {     // DPP max reduction over a row (4 steps) x 4
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                a = fmaxf(a, dppf<0xB1>(a)); a = fmaxf(a, dppf<0x4E>(a)); a = fmaxf(a, dppf<0x141>(a)); a = fmaxf(a, dppf<0x140>(a));
                a += b;
            }
        } else if (PAT == 7) {     // LDS write -> wave sync -> read (dependent round trip)
            lds[(lane * 17 + i) & 1023] = a;
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront"); __builtin_amdgcn_wave_barrier(); __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            a += lds[(lane * 29 + i) & 1023];
        } else if (PAT == 8) {     // LDS atomic add with return by lane 0, broadcast
            int at = 0;
            if (lane == 0) at = (int)atomicAdd(&cnt, 1u);
            at = __builtin_amdgcn_readfirstlane(at);
            acc += at;
        } else if (PAT == 9) {     // workgroup barrier
            __syncthreads();
        } else if (PAT == 10) {    // global agent-scope fetch-add round trip by lane 0
            unsigned int v = 0;
            if (lane == 0) v = __hip_atomic_fetch_add(gmem + 64 * (threadIdx.x >> 6), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            acc += __builtin_amdgcn_readfirstlane((int)v);
        } else if (PAT == 11) {    // agent-scope store + wait for its acknowledgement
            __hip_atomic_store(gmem + 1024 + threadIdx.x, (unsigned int)i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        } else if (PAT == 12) {    // agent-scope load round trip (dependent address)
            unsigned int v = __hip_atomic_load(gmem + 4096 + ((threadIdx.x + acc) & 1023), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            acc += (int)v;
        } else if (PAT == 13) {    // plain load round trip (dependent address, L2 / L1 hit after the first)
            unsigned int v = gmem[4096 + ((threadIdx.x + acc) & 1023)];
            acc += (int)v;
        } else if (PAT == 14) {    // 64-bit compare + count from 8 LDS broadcast reads (the ranking loop)
            const uint64_t key = ((uint64_t)__float_as_uint(a) << 32) | lane;
            const uint64_t *p = reinterpret_cast<const uint64_t *>(lds);
            uint64_t kj[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) kj[u] = p[(i * 8 + u) & 511];
#pragma unroll
            for (int u = 0; u < 8; ++u) acc += (kj[u] > key) ? 1 : 0;
        } else if (PAT == 15) {    // fp64 add chain, 8 per iteration
            double x = a;
#pragma unroll
            for (int u = 0; u < 8; ++u) x = x + 1.25;
            a = (float)x;
        }
    }
    unsigned long long t1 = clock64(), w1 = wall_clock64();
    if (threadIdx.x == 0) { out->cyc = t1 - t0; out->wall = w1 - w0; out->tbeg = t0; }
    if (lane == 0) out->tend[threadIdx.x >> 6] = t1;
    if (a + b + c + d + acc == 12345.678f) out->sink = a;
}

typedef void (*Kern)(Res *, int, float, unsigned int *);

int main() {
    Res *d; unsigned int *g;
    CHECK(hipMalloc(&d, sizeof(Res))); CHECK(hipMalloc(&g, 1 << 20)); CHECK(hipMemset(g, 0, 1 << 20));
    const char *names[16] = {"dep fadd x16", "4 indep fadd chains x4 (16 ops)", "dep exp2+sub x16 (32 ops)", "8 exps in 4 chains (sub,mul,exp,add + inc)",
                             "ballot+popc+add x16", "readlane rank x16", "dpp row max x4 (16 dpp+max, 4 add)", "LDS write->sync->read", "LDS atomic ret + readfirstlane",
                             "__syncthreads", "global atomic add (agent) round trip", "agent store + vmcnt(0)", "agent load round trip", "plain load round trip (cached)",
                             "8 LDS bcast reads + 8 u64 cmp-count", "dep f64 add x8"};
    Kern ks[16] = {k<0>, k<1>, k<2>, k<3>, k<4>, k<5>, k<6>, k<7>, k<8>, k<9>, k<10>, k<11>, k<12>, k<13>, k<14>, k<15>};
    for (int waves : {1, 4, 16}) {
        printf("---- %d wavefront(s) in one workgroup\n", waves);
        for (int p = 0; p < 16; ++p) {
            const int N = 2000;
            Res r{};
            for (int rep = 0; rep < 3; ++rep) {
                hipLaunchKernelGGL(ks[p], dim3(1), dim3(64 * waves), 0, 0, d, N, 1.0f, g);
                CHECK(hipDeviceSynchronize());
                CHECK(hipMemcpy(&r, d, sizeof(r), hipMemcpyDeviceToHost));
            }
            unsigned long long last = 0; for (int w = 0; w < waves; ++w) last = r.tend[w] > last ? r.tend[w] : last;
            printf("%-48s wave0 %8.1f cyc/iter  all %8.1f cyc/iter\n", names[p], (double)r.cyc / N, (double)(last - r.tbeg) / N);
            fflush(stdout);
        }
    }
    return 0;
}
