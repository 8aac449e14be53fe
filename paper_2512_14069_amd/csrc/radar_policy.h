// One call of RADAR's prediction model (Sec. 4.2; architecture per App. A.3) as a
// workgroup-wide device routine: LSTM cell over the k frontier confidences, the new
// hidden vector joined with those inputs, two-layer perceptron, softmax over
// {0 = stop, 1 = continue}.
//
// The routine is written for one workgroup of 1024 threads (16 wavefronts) per state and
// is used twice: by the stand-alone kernel behind radar_policy_step and as the tail of the
// expansion kernel's last workgroup, where the confidences are still in LDS.
//
// The work is 4H x (H + k) + M x (H + k) multiply-adds on fp32 weights that sit in L2
// between calls (about 350 KB at H = M = 128, k = 10): latency-bound, so the code issues
// every weight load of a phase before anything waits, keeps rows contiguous across lanes
// (a 128-float row of w_hh is 32 lanes x 16 bytes) and folds the per-row sums with a
// transposing butterfly (16 rows in 16 shuffles rather than 80).
#pragma once

#include "radar_device.h"

namespace radar {

constexpr int kPolThreads = 1024;
constexpr int kPolWaves = kPolThreads / kWave;       // 16
constexpr int kPolH = 128;                           // LSTM hidden size (App. A.3)
constexpr int kPolMMax = 128;                        // largest hidden size of the head
constexpr int kPolGateRows = 4 * kPolH / kPolWaves;  // 32 gate rows per wavefront
constexpr int kPolHeadRows = kPolMMax / kPolWaves;   // up to 8 head rows per wavefront

struct PolicyArgs {
    const float *w_ih, *w_hh, *b_ih, *b_hh, *w1, *b1, *w2, *b2;
    const float *h_in, *c_in;       // [B][H] or null = zero state
    const float *uniforms;          // [B] or null = argmax action
    float *h_out, *c_out;           // [B][H]
    float *logits, *probs;          // [B][2]
    int32_t *action;                // [B]
    int k, M;
};

struct alignas(16) PolicySmem {
    float x[RADAR_K_MAX];
    float h[kPolH];
    float gate[4 * kPolH];
    float hn[kPolH];
    float z[kPolMMax];
};

// Weights a lane holds between the issue of its loads and their use.
struct PolicyGateRegs {
    float4 whh[kPolGateRows / 2];   // row 32w + 2*it + (lane / 32), columns 4*(lane % 32) ..
    float wih[kPolGateRows / 4];    // column lane % 16 (< k) of pass it + 8 * ((lane / 16) % 2)
};
struct PolicyHeadRegs {
    float w[kPolHeadRows][3];       // row 8w + r (by M / 16 rows per wavefront), columns lane, lane + 64, lane + 128
};

// Issue the loads of this wavefront's 32 gate rows.  Needs nothing but the weights, so a
// caller may run it before the confidences exist.
__device__ __forceinline__ void policy_load_gate_rows(const PolicyArgs &p, bool has_state, PolicyGateRegs &g) {
    const int w = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int half = lane >> 5, j = lane & 31;
#pragma unroll
    for (int it = 0; it < kPolGateRows / 2; ++it) {
        const int row = kPolGateRows * w + 2 * it + half;
        g.whh[it] = has_state ? *reinterpret_cast<const float4 *>(p.w_hh + (size_t)row * kPolH + 4 * j)
                              : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    const int jj = j & 15, hi = j >> 4;
#pragma unroll
    for (int it = 0; it < kPolGateRows / 4; ++it) {
        const int row = kPolGateRows * w + 2 * (it + 8 * hi) + half;
        g.wih[it] = jj < p.k ? p.w_ih[(size_t)row * p.k + jj] : 0.f;
    }
}

__device__ __forceinline__ int policy_head_rows_per_wave(int M) { return (M + kPolWaves - 1) / kPolWaves; }

__device__ __forceinline__ void policy_load_head_rows(const PolicyArgs &p, PolicyHeadRegs &r) {
    const int w = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    const int rpw = policy_head_rows_per_wave(p.M), cols = kPolH + p.k;
#pragma unroll
    for (int i = 0; i < kPolHeadRows; ++i) {
        const int row = w * rpw + i;
        const bool live = i < rpw && row < p.M;
        const float *src = p.w1 + (size_t)(live ? row : 0) * cols;
        r.w[i][0] = live ? src[lane] : 0.f;
        r.w[i][1] = live ? src[lane + 64] : 0.f;
        r.w[i][2] = (live && lane + 128 < cols) ? src[lane + 128] : 0.f;
    }
}

// v[0..N) per lane -> sums over groups of lanes.  One step with lane distance OFF halves the
// number of values a lane carries: lanes whose bit OFF is set keep the upper half.
template <int N, int OFF>
__device__ __forceinline__ void fold_step(float *v, int lane) {
    const bool up = (lane & OFF) != 0;
#pragma unroll
    for (int i = 0; i < N / 2; ++i) {
        const float send = up ? v[i] : v[i + N / 2];
        const float keep = up ? v[i + N / 2] : v[i];
        v[i] = keep + __shfl_xor(send, OFF);
    }
}

// The whole step for state b.  `s.x[0..k)` must have been written by threads of this
// workgroup before they call (the routine's first barrier orders those writes before the
// reads).  `g` holds what policy_load_gate_rows returned.  Every thread of the workgroup must
// call it (it contains barriers).  h_out / c_out may be the arrays h_in / c_in.
__device__ __forceinline__ void policy_step_block(const PolicyArgs &p, int b, bool has_state, PolicyGateRegs &g,
                                                  PolicySmem &s) {
    const int tid = threadIdx.x, w = tid / kWave, lane = tid % kWave;
    const int half = lane >> 5, j = lane & 31;

    // state of unit u = tid (first two wavefronts)
    float c_prev = 0.f, bias[4] = {0.f, 0.f, 0.f, 0.f};
    if (tid < kPolH) {
        if (has_state) {
            s.h[tid] = p.h_in[(size_t)b * kPolH + tid];
            c_prev = p.c_in[(size_t)b * kPolH + tid];
        } else {
            s.h[tid] = 0.f;
        }
    }
    __syncthreads();

    // head operands this lane will need; loaded further down, used two barriers later
    PolicyHeadRegs hr;
    const int rpw = policy_head_rows_per_wave(p.M);
    const int head_i = ((lane >> 5) & 1) * 4 + ((lane >> 4) & 1) * 2 + ((lane >> 3) & 1);
    const int head_row = w * rpw + head_i;
    const bool head_live = head_i < rpw && head_row < p.M;
    float b1v = 0.f, w2v[2][2] = {{0.f, 0.f}, {0.f, 0.f}}, b2v[2] = {0.f, 0.f}, uni = 0.f;

    // ---- gate pre-activations: 32 rows per wavefront, two rows per pass over the lanes
    {
        const float4 h4 = *reinterpret_cast<const float4 *>(&s.h[4 * j]);
        const int jj = j & 15, hi = j >> 4;
        const float xj = jj < p.k ? s.x[jj] : 0.f;
        float v[kPolGateRows / 2];
#pragma unroll
        for (int it = 0; it < kPolGateRows / 2; ++it) {
            // input part: lanes 0..15 of a half carry passes 0..7, lanes 16..31 passes 8..15
            float a = ((it >> 3) == hi) ? g.wih[it & 7] * xj : 0.f;
            a = fmaf(g.whh[it].x, h4.x, a);
            a = fmaf(g.whh[it].y, h4.y, a);
            a = fmaf(g.whh[it].z, h4.z, a);
            a = fmaf(g.whh[it].w, h4.w, a);
            v[it] = a;
        }
        // the gate weights are consumed: fetch the head's while the sums are folded
        policy_load_head_rows(p, hr);
        if (tid < kPolH) {
#pragma unroll
            for (int q = 0; q < 4; ++q) bias[q] = p.b_ih[q * kPolH + tid] + p.b_hh[q * kPolH + tid];
        }
        if ((lane & 7) == 0 && head_live) b1v = p.b1[head_row];
        if (w == 0) {
            if (lane < p.M) { w2v[0][0] = p.w2[lane]; w2v[1][0] = p.w2[p.M + lane]; }
            if (lane + 64 < p.M) { w2v[0][1] = p.w2[lane + 64]; w2v[1][1] = p.w2[p.M + lane + 64]; }
            if (lane == 0) { b2v[0] = p.b2[0]; b2v[1] = p.b2[1]; uni = p.uniforms ? p.uniforms[b] : 0.f; }
        }
        fold_step<16, 16>(v, lane);
        fold_step<8, 8>(v, lane);
        fold_step<4, 4>(v, lane);
        fold_step<2, 2>(v, lane);
        const float sum = v[0] + __shfl_xor(v[0], 1);
        // the lane now holds pass it = 8*b4 + 4*b3 + 2*b2 + b1 of its half (b_n = bit n of the lane)
        const int it = ((lane >> 4) & 1) * 8 + ((lane >> 3) & 1) * 4 + ((lane >> 2) & 1) * 2 + ((lane >> 1) & 1);
        if ((lane & 1) == 0) s.gate[kPolGateRows * w + 2 * it + half] = sum;
    }
    __syncthreads();

    // ---- cell update, one unit per thread
    if (tid < kPolH) {
        const float ai = s.gate[tid] + bias[0];
        const float af = s.gate[kPolH + tid] + bias[1];
        const float ag = s.gate[2 * kPolH + tid] + bias[2];
        const float ao = s.gate[3 * kPolH + tid] + bias[3];
        const float ig = 1.f / (1.f + expf(-ai));
        const float fg = 1.f / (1.f + expf(-af));
        const float gg = tanhf(ag);
        const float og = 1.f / (1.f + expf(-ao));
        const float cn = fmaf(fg, c_prev, ig * gg);
        const float hn = og * tanhf(cn);
        s.hn[tid] = hn;
        p.c_out[(size_t)b * kPolH + tid] = cn;
        p.h_out[(size_t)b * kPolH + tid] = hn;
    }
    __syncthreads();

    // ---- first layer of the head on [h'; x], ReLU
    {
        const float in0 = s.hn[lane], in1 = s.hn[lane + 64];
        const float in2 = lane < p.k ? s.x[lane] : 0.f;
        float v[kPolHeadRows];
#pragma unroll
        for (int i = 0; i < kPolHeadRows; ++i) v[i] = fmaf(hr.w[i][0], in0, fmaf(hr.w[i][1], in1, hr.w[i][2] * in2));
        fold_step<8, 32>(v, lane);
        fold_step<4, 16>(v, lane);
        fold_step<2, 8>(v, lane);
        float sum = v[0];
        sum += __shfl_xor(sum, 4);
        sum += __shfl_xor(sum, 2);
        sum += __shfl_xor(sum, 1);
        // the lane now holds row head_i = 4*b5 + 2*b4 + b3 of its wavefront
        if ((lane & 7) == 0 && head_live) s.z[head_row] = fmaxf(sum + b1v, 0.f);
    }
    __syncthreads();

    // ---- two logits, softmax, action
    if (w == 0) {
        const float z0 = lane < p.M ? s.z[lane] : 0.f;
        const float z1 = lane + 64 < p.M ? s.z[lane + 64] : 0.f;
        float l0 = fmaf(w2v[0][0], z0, w2v[0][1] * z1);
        float l1 = fmaf(w2v[1][0], z0, w2v[1][1] * z1);
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            l0 += __shfl_xor(l0, off);
            l1 += __shfl_xor(l1, off);
        }
        if (lane == 0) {
            l0 += b2v[0];
            l1 += b2v[1];
            const float p1 = 1.f / (1.f + expf(l0 - l1));
            const float p0 = 1.f / (1.f + expf(l1 - l0));
            p.logits[2 * b] = l0;
            p.logits[2 * b + 1] = l1;
            p.probs[2 * b] = p0;
            p.probs[2 * b + 1] = p1;
            p.action[b] = p.uniforms ? (uni < p1 ? 1 : 0) : (l1 > l0 ? 1 : 0);
        }
    }
}

}  // namespace radar
