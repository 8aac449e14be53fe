// Matrix-pipe probe for gfx950 (MI355X): how much vector-ALU work runs beside MFMAs, and at what clock.
//
// The long-range tree attention issues, per 64-row tile and wavefront, 32 v_mfma_f32_32x32x16_bf16
// (8 passes = 32 cycles each) and about as many cycles of softmax arithmetic; its time is close to
// the sum of the two.  This program measures the building blocks in isolation: workgroups of eight
// wavefronts (two per SIMD, as in that kernel) repeat a fixed instruction pattern between two reads
// of the core clock (s_memtime) and of the 100 MHz wall clock, on a quarter of the chip (64
// workgroups) and on all of it (256):
//   mfma        16 independent-by-four MFMAs per repetition, nothing else
//   valu        16 x 7 v_fma_f32 per repetition, nothing else
//   mfma+valu   each MFMA followed by 7 independent v_fma_f32 in the same wavefront
//   mfma+exp    each MFMA followed by 2 x (v_fma_f32, v_exp_f32, v_add_f32) and one more v_fma_f32
//   split       wavefronts 0-3 run `mfma`, wavefronts 4-7 (the other wavefront of each SIMD) run `valu`
//   mfma+ld/2   `mfma`, and every second repetition each wavefront loads 1 KB from global memory straight
//               into LDS (global_load_lds_dwordx4), streaming through a 512 MB buffer: ~2 TB/s on the whole chip
//   mfma+ld     the same with a load in every repetition: ~4 TB/s
//   exp+ld      `mfma+exp` with a load in every repetition
// Every pattern is one asm statement, so the order is the one written.  Output per pattern: core
// cycles per repetition (median wavefront), wall time per repetition, the clock they imply, and the
// MFMA rate of the whole launch in TFLOP/s.
//
//   hipcc --offload-arch=gfx950 -O3 -std=c++17 -Xclang -target-feature -Xclang -packed-fp32-ops \
//         benchmarks/mfma_probe.hip -o benchmarks/mfma_probe && ./benchmarks/mfma_probe
//
// A summary of one run is in profiles/gfx950_mfma_probe.txt.
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdint.h>
#include <algorithm>
#include <vector>

#define CHECK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); return 1; } } while (0)

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct Res { unsigned long long cyc, wall; float sink; int role; };

#define F1(x) "v_fma_f32 " x ", " x ", %[c], %[c]\n\t"
#define FMA7 F1("%[x0]") F1("%[x1]") F1("%[x2]") F1("%[x3]") F1("%[x4]") F1("%[x5]") F1("%[x6]")
#define E1(x, y, z) "v_fma_f32 " x ", " y ", %[c], %[c]\n\tv_exp_f32 " x ", " x "\n\tv_add_f32 " z ", " z ", " x "\n\t"
#define EXP7 E1("%[x0]", "%[x1]", "%[x2]") E1("%[x3]", "%[x4]", "%[x5]") F1("%[x6]")
#define MF(acc) "v_mfma_f32_32x32x16_bf16 " acc ", %[a], %[b], " acc "\n\t"

// PAT: 0 mfma, 1 valu, 2 mfma+valu, 3 mfma+exp, 4 split by wavefront; LD: a load every LD-th repetition (0: none)
template <int PAT, int LD>
__global__ __launch_bounds__(512) void probe(Res *out, int N, float seed, const unsigned char *stream, size_t stream_bytes) {
    __shared__ __attribute__((aligned(16))) unsigned char landing[8 * 4 * 1024];      // four 1 KB slots per wavefront
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    floatx16 acc0, acc1, acc2, acc3;
    for (int r = 0; r < 16; ++r) { acc0[r] = seed; acc1[r] = seed * 2; acc2[r] = seed * 3; acc3[r] = seed * 4; }
    bf16x8 a, b;
    for (int e = 0; e < 8; ++e) { a[e] = (__bf16)(seed * (lane + e) * 1e-3f); b[e] = (__bf16)(seed * (lane - e) * 1e-3f); }
    float x0 = seed, x1 = seed * 0.5f, x2 = 0.f, x3 = seed * 0.25f, x4 = seed * 0.125f, x5 = 0.f, x6 = seed * 0.3f;
    const float c = 0.999f;
    const int role = PAT == 4 ? (w < 4 ? 0 : 1) : PAT;
    // each wavefront streams through its own slice of the buffer and wraps around
    const size_t nwaves = (size_t)gridDim.x * 8, slice = (stream_bytes / nwaves) & ~size_t(1023);
    const unsigned char *mine = stream + ((size_t)blockIdx.x * 8 + w) * slice + lane * 16;
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) void *)landing + (uint32_t)w * 4096);
    size_t pos = 0;
    __syncthreads();
    const unsigned long long t0 = clock64(), w0 = wall_clock64();
    for (int i = 0; i < N; ++i) {
        if (LD > 0 && i % LD == 0) {
            const uint32_t dst = lds0 + ((uint32_t)(i / LD) & 3u) * 1024;
            asm volatile("s_waitcnt vmcnt(3)\n\ts_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(dst), "v"(mine + pos) : "memory", "m0");
            pos += 1024;
            if (pos >= slice) pos = 0;
        }
        if (role == 0) {
            asm volatile(MF("%[a0]") MF("%[a1]") MF("%[a2]") MF("%[a3]") MF("%[a0]") MF("%[a1]") MF("%[a2]") MF("%[a3]")
                         MF("%[a0]") MF("%[a1]") MF("%[a2]") MF("%[a3]") MF("%[a0]") MF("%[a1]") MF("%[a2]") MF("%[a3]")
                         : [a0] "+v"(acc0), [a1] "+v"(acc1), [a2] "+v"(acc2), [a3] "+v"(acc3) : [a] "v"(a), [b] "v"(b));
        } else if (role == 1) {
            asm volatile(FMA7 FMA7 FMA7 FMA7 FMA7 FMA7 FMA7 FMA7
                         FMA7 FMA7 FMA7 FMA7 FMA7 FMA7 FMA7 FMA7
                         : [x0] "+v"(x0), [x1] "+v"(x1), [x2] "+v"(x2), [x3] "+v"(x3), [x4] "+v"(x4), [x5] "+v"(x5), [x6] "+v"(x6)
                         : [c] "v"(c));
        } else if (role == 2) {
            asm volatile(MF("%[a0]") FMA7 MF("%[a1]") FMA7 MF("%[a2]") FMA7 MF("%[a3]") FMA7
                         MF("%[a0]") FMA7 MF("%[a1]") FMA7 MF("%[a2]") FMA7 MF("%[a3]") FMA7
                         MF("%[a0]") FMA7 MF("%[a1]") FMA7 MF("%[a2]") FMA7 MF("%[a3]") FMA7
                         MF("%[a0]") FMA7 MF("%[a1]") FMA7 MF("%[a2]") FMA7 MF("%[a3]") FMA7
                         : [a0] "+v"(acc0), [a1] "+v"(acc1), [a2] "+v"(acc2), [a3] "+v"(acc3),
                           [x0] "+v"(x0), [x1] "+v"(x1), [x2] "+v"(x2), [x3] "+v"(x3), [x4] "+v"(x4), [x5] "+v"(x5), [x6] "+v"(x6)
                         : [a] "v"(a), [b] "v"(b), [c] "v"(c));
        } else {
            asm volatile(MF("%[a0]") EXP7 MF("%[a1]") EXP7 MF("%[a2]") EXP7 MF("%[a3]") EXP7
                         MF("%[a0]") EXP7 MF("%[a1]") EXP7 MF("%[a2]") EXP7 MF("%[a3]") EXP7
                         MF("%[a0]") EXP7 MF("%[a1]") EXP7 MF("%[a2]") EXP7 MF("%[a3]") EXP7
                         MF("%[a0]") EXP7 MF("%[a1]") EXP7 MF("%[a2]") EXP7 MF("%[a3]") EXP7
                         : [a0] "+v"(acc0), [a1] "+v"(acc1), [a2] "+v"(acc2), [a3] "+v"(acc3),
                           [x0] "+v"(x0), [x1] "+v"(x1), [x2] "+v"(x2), [x3] "+v"(x3), [x4] "+v"(x4), [x5] "+v"(x5), [x6] "+v"(x6)
                         : [a] "v"(a), [b] "v"(b), [c] "v"(c));
        }
    }
    // the accumulators are read here: the last MFMAs have finished before the clock is
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    float sink = acc0[0] + acc1[1] + acc2[2] + acc3[3] + x0 + x1 + x2 + x3 + x4 + x5 + x6 + (float)landing[threadIdx.x];
    asm volatile("" : "+v"(sink));
    const unsigned long long t1 = clock64(), w1 = wall_clock64();
    if (lane == 0) {
        Res r; r.cyc = t1 - t0; r.wall = w1 - w0; r.sink = sink; r.role = role;
        out[blockIdx.x * 8 + w] = r;
    }
}

template <int PAT, int LD = 0>
static int run(const char *name, int nwg, Res *d, int N, const unsigned char *stream = nullptr, size_t stream_bytes = 0) {
    std::vector<Res> h(nwg * 8);
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
    probe<PAT, LD><<<nwg, 512>>>(d, N / 10, 1.0f, stream, stream_bytes);      // warm-up
    CHECK(hipDeviceSynchronize());
    CHECK(hipEventRecord(e0));
    probe<PAT, LD><<<nwg, 512>>>(d, N, 1.0f, stream, stream_bytes);
    CHECK(hipEventRecord(e1));
    CHECK(hipDeviceSynchronize());
    float ms = 0.f;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    CHECK(hipMemcpy(h.data(), d, sizeof(Res) * h.size(), hipMemcpyDeviceToHost));
    for (int role = 0; role < 4; ++role) {
        std::vector<double> cyc, wall;
        for (auto &r : h) if (r.role == role) { cyc.push_back((double)r.cyc / N); wall.push_back((double)r.wall / N * 10.0); }   // wall clock: 100 MHz -> ns
        if (cyc.empty()) continue;
        std::sort(cyc.begin(), cyc.end()); std::sort(wall.begin(), wall.end());
        const double c = cyc[cyc.size() / 2], wns = wall[wall.size() / 2];
        const bool has_mfma = role != 1;
        const int waves = (int)cyc.size();
        const double tflops = has_mfma ? (double)waves * N * 16 * 32768.0 / (ms * 1e-3) * 1e-12 : 0.0;
        const double tbs = LD > 0 ? (double)nwg * 8 * (N / LD) * 1024.0 / (ms * 1e-3) * 1e-12 : 0.0;
        printf("%-10s %3d WGs  role %d  %4d wavefronts  %7.1f cycles/rep  %7.1f ns/rep  clock %.2f GHz  kernel %.1f us  %s%.0f TFLOP/s  %.2f TB/s loaded\n",
               name, nwg, role, waves, c, wns, c / wns, ms * 1e3, has_mfma ? "" : "(no MFMA) ", tflops, tbs);
    }
    return 0;
}

int main() {
    Res *d;
    CHECK(hipMalloc(&d, sizeof(Res) * 256 * 8));
    const int N = 4000;                                           // 64000 MFMAs per wavefront: ~1 ms
    const size_t stream_bytes = size_t(512) << 20;
    unsigned char *stream;
    CHECK(hipMalloc(&stream, stream_bytes));
    CHECK(hipMemset(stream, 1, stream_bytes));
    for (int nwg : {64, 256}) {
        if (run<0>("mfma", nwg, d, N)) return 1;
        if (run<1>("valu", nwg, d, N)) return 1;
        if (run<2>("mfma+valu", nwg, d, N)) return 1;
        if (run<3>("mfma+exp", nwg, d, N)) return 1;
        if (run<4>("split", nwg, d, N)) return 1;
        if (run<0, 2>("mfma+ld/2", nwg, d, N, stream, stream_bytes)) return 1;
        if (run<0, 1>("mfma+ld", nwg, d, N, stream, stream_bytes)) return 1;
        if (run<3, 1>("exp+ld", nwg, d, N, stream, stream_bytes)) return 1;
    }
    CHECK(hipFree(stream));
    CHECK(hipFree(d));
    return 0;
}
