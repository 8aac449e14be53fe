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
//   mfma+lds    `mfma` with every MFMA's first operand read from LDS (ds_read_b128, 1 KB per MFMA and wavefront,
//               two reads in flight), as the attention kernels feed theirs
//   all         `mfma+exp` with the operand reads from LDS and a load from global memory in every repetition
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
// an MFMA whose first operand was read from LDS two steps ago; then the read for two steps ahead
#define ML(acc, use, next, off) "s_waitcnt lgkmcnt(1)\n\tv_mfma_f32_32x32x16_bf16 " acc ", " use ", %[b], " acc "\n\tds_read_b128 " next ", %[la] offset:" off "\n\t"

// PAT: 0 mfma, 1 valu, 2 mfma+valu, 3 mfma+exp, 4 split by wavefront; LD: a load every LD-th repetition (0: none)
template <int PAT, int LD, bool LDS = false>
__global__ __launch_bounds__(512) void probe(Res *out, int N, float seed, const unsigned char *stream, size_t stream_bytes) {
    __shared__ __attribute__((aligned(16))) unsigned char landing[8 * 4 * 1024];      // four 1 KB slots per wavefront
    __shared__ __attribute__((aligned(16))) unsigned char operands[17 * 1024];        // read as MFMA operands when LDS is set
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    floatx16 acc0, acc1, acc2, acc3;
    for (int r = 0; r < 16; ++r) { acc0[r] = seed; acc1[r] = seed * 2; acc2[r] = seed * 3; acc3[r] = seed * 4; }
    bf16x8 a, b;
    // operands with the statistics of real data (signs and mantissas that differ from element to element:
    // what the multipliers draw depends on how many bits toggle), magnitudes near one
    auto mix = [](uint32_t v) { v ^= v >> 16; v *= 0x7feb352du; v ^= v >> 15; v *= 0x846ca68bu; v ^= v >> 16; return v; };
    auto rnd_bf16 = [&](uint32_t v) { const uint32_t h = mix(v); return __builtin_bit_cast(__bf16, (uint16_t)((h & 0x807fu) | 0x3f00u | ((h >> 20) & 0x0080u))); };
    for (int e = 0; e < 8; ++e) { a[e] = rnd_bf16(threadIdx.x * 16 + e); b[e] = rnd_bf16(threadIdx.x * 16 + 8 + e + 7777u * (uint32_t)seed); }
    float x0 = seed, x1 = seed * 0.5f, x2 = 0.f, x3 = seed * 0.25f, x4 = seed * 0.125f, x5 = 0.f, x6 = seed * 0.3f;
    const float c = 0.999f;
    const int role = PAT == 4 ? (w < 4 ? 0 : 1) : PAT;
    // each wavefront streams through its own slice of the buffer and wraps around
    const size_t nwaves = (size_t)gridDim.x * 8, slice = (stream_bytes / nwaves) & ~size_t(1023);
    const unsigned char *mine = stream + ((size_t)blockIdx.x * 8 + w) * slice + lane * 16;
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(__attribute__((address_space(3))) void *)landing + (uint32_t)w * 4096);
    size_t pos = 0;
    for (int i = threadIdx.x; i < 17 * 1024 / 4; i += 512) {
        const uint32_t h = mix(i * 2654435761u + 12345u);
        reinterpret_cast<uint32_t *>(operands)[i] = (h & 0x807f807fu) | 0x3f003f00u | ((h >> 3) & 0x00800080u);
    }
    bf16x8 a0 = a, a1 = a, a2 = a, a3 = a;
    const uint32_t la = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void *)operands + lane * 16;
    __syncthreads();
    if (LDS) asm volatile("ds_read_b128 %0, %2\n\tds_read_b128 %1, %2 offset:1024" : "=v"(a0), "=v"(a1) : "v"(la) : "memory");
    const unsigned long long t0 = clock64(), w0 = wall_clock64();
    for (int i = 0; i < N; ++i) {
        if (LD > 0 && i % LD == 0) {
            const uint32_t dst = lds0 + ((uint32_t)(i / LD) & 3u) * 1024;
            asm volatile("s_waitcnt vmcnt(3)\n\ts_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(dst), "v"(mine + pos) : "memory", "m0");
            pos += 1024;
            if (pos >= slice) pos = 0;
        }
        if (LDS && role == 0) {
            asm volatile(ML("%[c0]", "%[r0]", "%[r2]", "2048") ML("%[c1]", "%[r1]", "%[r3]", "3072") ML("%[c2]", "%[r2]", "%[r0]", "4096") ML("%[c3]", "%[r3]", "%[r1]", "5120")
                         ML("%[c0]", "%[r0]", "%[r2]", "6144") ML("%[c1]", "%[r1]", "%[r3]", "7168") ML("%[c2]", "%[r2]", "%[r0]", "8192") ML("%[c3]", "%[r3]", "%[r1]", "9216")
                         ML("%[c0]", "%[r0]", "%[r2]", "10240") ML("%[c1]", "%[r1]", "%[r3]", "11264") ML("%[c2]", "%[r2]", "%[r0]", "12288") ML("%[c3]", "%[r3]", "%[r1]", "13312")
                         ML("%[c0]", "%[r0]", "%[r2]", "14336") ML("%[c1]", "%[r1]", "%[r3]", "15360") ML("%[c2]", "%[r2]", "%[r0]", "0") ML("%[c3]", "%[r3]", "%[r1]", "1024")
                         : [c0] "+v"(acc0), [c1] "+v"(acc1), [c2] "+v"(acc2), [c3] "+v"(acc3), [r0] "+v"(a0), [r1] "+v"(a1), [r2] "+v"(a2), [r3] "+v"(a3)
                         : [b] "v"(b), [la] "v"(la) : "memory");
        } else if (LDS) {
#define MLE(acc, use, next, off) ML(acc, use, next, off) EXP7
            asm volatile(MLE("%[c0]", "%[r0]", "%[r2]", "2048") MLE("%[c1]", "%[r1]", "%[r3]", "3072") MLE("%[c2]", "%[r2]", "%[r0]", "4096") MLE("%[c3]", "%[r3]", "%[r1]", "5120")
                         MLE("%[c0]", "%[r0]", "%[r2]", "6144") MLE("%[c1]", "%[r1]", "%[r3]", "7168") MLE("%[c2]", "%[r2]", "%[r0]", "8192") MLE("%[c3]", "%[r3]", "%[r1]", "9216")
                         MLE("%[c0]", "%[r0]", "%[r2]", "10240") MLE("%[c1]", "%[r1]", "%[r3]", "11264") MLE("%[c2]", "%[r2]", "%[r0]", "12288") MLE("%[c3]", "%[r3]", "%[r1]", "13312")
                         MLE("%[c0]", "%[r0]", "%[r2]", "14336") MLE("%[c1]", "%[r1]", "%[r3]", "15360") MLE("%[c2]", "%[r2]", "%[r0]", "0") MLE("%[c3]", "%[r3]", "%[r1]", "1024")
                         : [c0] "+v"(acc0), [c1] "+v"(acc1), [c2] "+v"(acc2), [c3] "+v"(acc3), [r0] "+v"(a0), [r1] "+v"(a1), [r2] "+v"(a2), [r3] "+v"(a3),
                           [x0] "+v"(x0), [x1] "+v"(x1), [x2] "+v"(x2), [x3] "+v"(x3), [x4] "+v"(x4), [x5] "+v"(x5), [x6] "+v"(x6)
                         : [b] "v"(b), [c] "v"(c), [la] "v"(la) : "memory");
        } else if (role == 0) {
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
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    float sink = (float)a0[0] + (float)a1[0] + (float)a2[0] + (float)a3[0] + acc0[0] + acc1[1] + acc2[2] + acc3[3] + x0 + x1 + x2 + x3 + x4 + x5 + x6 + (float)landing[threadIdx.x];
    asm volatile("" : "+v"(sink));
    const unsigned long long t1 = clock64(), w1 = wall_clock64();
    if (lane == 0) {
        Res r; r.cyc = t1 - t0; r.wall = w1 - w0; r.sink = sink; r.role = role;
        out[blockIdx.x * 8 + w] = r;
    }
}

template <int PAT, int LD = 0, bool LDS = false>
static int run(const char *name, int nwg, Res *d, int N, const unsigned char *stream = nullptr, size_t stream_bytes = 0) {
    std::vector<Res> h(nwg * 8);
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
    probe<PAT, LD, LDS><<<nwg, 512>>>(d, N / 10, 1.0f, stream, stream_bytes);      // warm-up
    CHECK(hipDeviceSynchronize());
    CHECK(hipEventRecord(e0));
    probe<PAT, LD, LDS><<<nwg, 512>>>(d, N, 1.0f, stream, stream_bytes);
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
        if (run<0, 0, true>("mfma+lds", nwg, d, N, stream, stream_bytes)) return 1;
        if (run<3, 1, true>("all", nwg, d, N, stream, stream_bytes)) return 1;
    }
    CHECK(hipFree(stream));
    CHECK(hipFree(d));
    return 0;
}
