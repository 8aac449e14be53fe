// Device-side helpers shared by the RADAR kernels (gfx950, 64-wide wavefronts).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/radar.h"

namespace radar {

constexpr int kWave = 64;

// ---------------------------------------------------------------- ordering
// Monotone map float -> uint32 (larger float <=> larger integer); -0.0 is folded
// onto +0.0 first so that it ties with it, as a float comparison would.
__device__ __forceinline__ uint32_t ord_of(float x) {
    x = x + 0.0f;
    uint32_t b = __float_as_uint(x);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float float_of_ord(uint32_t o) {
    uint32_t b = (o & 0x80000000u) ? (o & 0x7fffffffu) : ~o;
    return __uint_as_float(b);
}
// One 64-bit key per (value, index): comparing keys as unsigned integers gives
// "value descending, index ascending" when the larger key wins.
__device__ __forceinline__ uint64_t make_key(float x, uint32_t idx) {
    return (uint64_t(ord_of(x)) << 32) | uint64_t(~idx);
}
__device__ __forceinline__ uint32_t key_index(uint64_t key) { return ~uint32_t(key); }
__device__ __forceinline__ float key_value(uint64_t key) { return float_of_ord(uint32_t(key >> 32)); }

// ------------------------------------------------------------ DPP reductions
// dpp_ctrl: quad_perm [1,0,3,2] = 0xB1, [2,3,0,1] = 0x4E, row_half_mirror = 0x141,
// row_mirror = 0x140.  After the four steps every lane of a 16-lane row holds
// the row's reduction; the four rows are then combined through scalar reads.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, 0xF, 0xF, false);
}
template <int CTRL>
__device__ __forceinline__ uint64_t dpp_u64(uint64_t v) {
    uint32_t lo = dpp_u32<CTRL>(uint32_t(v));
    uint32_t hi = dpp_u32<CTRL>(uint32_t(v >> 32));
    return (uint64_t(hi) << 32) | lo;
}
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
    return __uint_as_float(dpp_u32<CTRL>(__float_as_uint(v)));
}

__device__ __forceinline__ uint32_t readlane_u32(uint32_t v, int lane) {
    return (uint32_t)__builtin_amdgcn_readlane((int)v, lane);
}
__device__ __forceinline__ uint64_t readlane_u64(uint64_t v, int lane) {
    return (uint64_t(readlane_u32(uint32_t(v >> 32), lane)) << 32) | readlane_u32(uint32_t(v), lane);
}
__device__ __forceinline__ float readlane_f32(float v, int lane) {
    return __uint_as_float(readlane_u32(__float_as_uint(v), lane));
}

__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
    v = max(v, dpp_u32<0xB1>(v));
    v = max(v, dpp_u32<0x4E>(v));
    v = max(v, dpp_u32<0x141>(v));
    v = max(v, dpp_u32<0x140>(v));
    uint32_t a = max(readlane_u32(v, 0), readlane_u32(v, 16));
    uint32_t b = max(readlane_u32(v, 32), readlane_u32(v, 48));
    return max(a, b);
}
__device__ __forceinline__ uint64_t max_u64(uint64_t a, uint64_t b) { return a > b ? a : b; }
__device__ __forceinline__ uint64_t wave_max_u64(uint64_t v) {
    v = max_u64(v, dpp_u64<0xB1>(v));
    v = max_u64(v, dpp_u64<0x4E>(v));
    v = max_u64(v, dpp_u64<0x141>(v));
    v = max_u64(v, dpp_u64<0x140>(v));
    uint64_t a = max_u64(readlane_u64(v, 0), readlane_u64(v, 16));
    uint64_t b = max_u64(readlane_u64(v, 32), readlane_u64(v, 48));
    return max_u64(a, b);
}
__device__ __forceinline__ float wave_max_f32(float v) {
    v = fmaxf(v, dpp_f32<0xB1>(v));
    v = fmaxf(v, dpp_f32<0x4E>(v));
    v = fmaxf(v, dpp_f32<0x141>(v));
    v = fmaxf(v, dpp_f32<0x140>(v));
    float a = fmaxf(readlane_f32(v, 0), readlane_f32(v, 16));
    float b = fmaxf(readlane_f32(v, 32), readlane_f32(v, 48));
    return fmaxf(a, b);
}
// Sum with a fixed association order (bit-reproducible from run to run).
__device__ __forceinline__ float wave_sum_f32(float v) {
    v = v + dpp_f32<0xB1>(v);
    v = v + dpp_f32<0x4E>(v);
    v = v + dpp_f32<0x141>(v);
    v = v + dpp_f32<0x140>(v);
    float a = readlane_f32(v, 0) + readlane_f32(v, 16);
    float b = readlane_f32(v, 32) + readlane_f32(v, 48);
    return a + b;
}

__device__ __forceinline__ double wave_sum_f64(double v) {
    auto step = [](double x, uint64_t moved) { return x + __longlong_as_double((long long)moved); };
    v = step(v, dpp_u64<0xB1>((uint64_t)__double_as_longlong(v)));
    v = step(v, dpp_u64<0x4E>((uint64_t)__double_as_longlong(v)));
    v = step(v, dpp_u64<0x141>((uint64_t)__double_as_longlong(v)));
    v = step(v, dpp_u64<0x140>((uint64_t)__double_as_longlong(v)));
    const uint64_t b = (uint64_t)__double_as_longlong(v);
    const double a0 = __longlong_as_double((long long)readlane_u64(b, 0));
    const double a1 = __longlong_as_double((long long)readlane_u64(b, 16));
    const double a2 = __longlong_as_double((long long)readlane_u64(b, 32));
    const double a3 = __longlong_as_double((long long)readlane_u64(b, 48));
    return (a0 + a1) + (a2 + a3);
}

__device__ __forceinline__ double readlane_f64(double v, int lane) {
    return __longlong_as_double((long long)readlane_u64((uint64_t)__double_as_longlong(v), lane));
}

// Inclusive prefix sum over the lanes of a wavefront by DPP moves (shift by 1, 2, 4, 8 inside each
// 16-lane row, then the row totals are carried into the following rows); fixed association order.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ double dpp_take_f64(double v) {
    const uint64_t b = (uint64_t)__double_as_longlong(v);
    // lanes without a source lane, and rows outside ROW_MASK, receive 0
    const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)b, CTRL, ROW_MASK, 0xF, true);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(b >> 32), CTRL, ROW_MASK, 0xF, true);
    return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
}
__device__ __forceinline__ double wave_scan_f64(double v) {
    v += dpp_take_f64<0x111, 0xF>(v);             // row_shr:1
    v += dpp_take_f64<0x112, 0xF>(v);             // row_shr:2
    v += dpp_take_f64<0x114, 0xF>(v);             // row_shr:4
    v += dpp_take_f64<0x118, 0xF>(v);             // row_shr:8
    v += dpp_take_f64<0x142, 0xA>(v);             // row_bcast:15 -> rows 1 and 3
    v += dpp_take_f64<0x143, 0xC>(v);             // row_bcast:31 -> rows 2 and 3
    return v;
}

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (kWave - 1)); }
__device__ __forceinline__ int wave_id() { return (int)(threadIdx.x >> 6); }

// Number of set bits of `mask` below this lane.
__device__ __forceinline__ int lanes_below(uint64_t mask) {
    return (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// Orders LDS traffic between the lanes of one wavefront (a lane reads what another
// lane of the same wavefront wrote earlier in program order).
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// ------------------------------------------------- cross-workgroup hand-over
// Results that one workgroup leaves for another workgroup of the SAME launch
// (partials merged by the last arriver) travel through device-scope accesses:
// every such store and load carries agent scope, so it is written through /
// fetched past the per-XCD L2 on its own.  This replaces agent-scope fences,
// which on this part write back and invalidate a whole L2 (measured: ~8 us per
// fence against ~0.1 us for the scoped accesses).  Protocol:
//   producer: store_shared_result(...) for everything it hands over;
//             publish_then_ticket() = wait until this lane's stores are
//             acknowledged (vmcnt 0), workgroup barrier, one relaxed device-
//             scope fetch-add by lane 0;
//   consumer (the workgroup whose ticket is the last): load_shared_result(...)
//             only -- it never reads handed-over data through a plain load.
template <typename T>
__device__ __forceinline__ T load_shared_result(const T *p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T>
__device__ __forceinline__ void store_shared_result(T *p, T v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Returns, to every lane of the workgroup, the value the counter had before this
// workgroup's arrival.  `flag` is one int of LDS.  All lanes must call it.
__device__ __forceinline__ unsigned int publish_then_ticket(unsigned int *counter, unsigned int *flag) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0)
        *flag = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    return *flag;
}

}  // namespace radar
