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
// every load before anything waits, keeps rows contiguous across lanes (a 128-float row of
// w_hh is 32 lanes x 16 bytes), folds the per-row sums with a transposing butterfly (16 rows
// in 16 shuffles rather than 80), and orders the work so that nothing but arithmetic is left
// once the confidences exist.
#pragma once

#include "radar_device.h"

namespace radar {

constexpr int kPolThreads = 1024;
constexpr int kPolWaves = kPolThreads / kWave;       // 16
constexpr int kPolWorkers = kPolWaves - 1;           // wavefront 0 supplies the inputs, the others compute
constexpr int kPolH = 128;                           // LSTM hidden size (App. A.3)
constexpr int kPolMMax = 128;                        // largest hidden size of the head
constexpr int kPolHeadRows = (kPolMMax + kPolWorkers - 1) / kPolWorkers;   // up to 9 head rows per worker
static_assert(kPolHeadRows == 9, "the head fold below is written for 8 + 1 rows");

struct PolicyArgs {
    const float *w_ih, *w_hh, *b_ih, *b_hh, *w1, *b1, *w2, *b2;
    const float *h_in, *c_in;       // [B][H] or null = zero state
    const float *uniforms;          // [B] or null = argmax action
    float *h_out, *c_out;           // [B][H]
    float *logits, *probs;          // [B][2]
    int32_t *action;                // [B]
    int k, M;
};

// Row r of w_ih sits at wih[r * k + r / kPolH]: the one-word shift per gate block spreads the
// four gates of a unit over different LDS banks when 64 lanes read "their" row.
struct alignas(16) PolicySmem {
    float x[RADAR_K_MAX];
    float gate[4 * kPolH];          // w_hh h (stand-alone kernel; the fused path keeps it in global memory)
    float hn[kPolH];
    float z[kPolMMax];
    float wih[4 * kPolH * RADAR_K_MAX + 4];
};

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

// Logistic function and tanh from the hardware exponential and reciprocal (a few 1e-7 of
// absolute error; both saturate cleanly for large arguments of either sign).
__device__ __forceinline__ float fast_sigmoid(float a) { return __frcp_rn(1.f + __expf(-a)); }
__device__ __forceinline__ float fast_tanh(float a) { return 1.f - 2.f * __frcp_rn(1.f + __expf(2.f * a)); }

// The part of the gate pre-activations that needs no input: rows of w_hh times h_in.  A row is
// 128 floats = one 32-lane half-wavefront x 16 bytes.  The calling workgroup is part `part` of
// `parts` that share the 4H rows; its HW half-wavefronts (32 in a workgroup of 1024 lanes) take rows
// (part + parts * i) * HW + half-wavefront for i = 0, 1, ... in batches of NR (4 or 16) rows per lane,
// all loads of a batch issued before its sums are folded.  store(row, value) is called by one lane per row.
template <int NR, int HW = 32, typename Store>
__device__ __forceinline__ void policy_hidden_rows(const PolicyArgs &p, int b, int part, int parts, Store &&store) {
    static_assert(NR == 4 || NR == 16, "NR");
    const int lane = threadIdx.x % kWave, j = lane & 31, hwave = threadIdx.x >> 5;
    const int rows = 4 * kPolH;
    if (part * HW >= rows) return;
    const float4 h4 = *reinterpret_cast<const float4 *>(p.h_in + (size_t)b * kPolH + 4 * j);
    for (int i0 = 0; (part + parts * i0) * HW < rows; i0 += NR) {
        float v[NR];
#pragma unroll
        for (int i = 0; i < NR; ++i) {
            const int row = min((part + parts * (i0 + i)) * HW + hwave, rows - 1);      // clamped: stays a legal read
            const float4 wv = *reinterpret_cast<const float4 *>(p.w_hh + (size_t)row * kPolH + 4 * j);
            v[i] = fmaf(wv.x, h4.x, fmaf(wv.y, h4.y, fmaf(wv.z, h4.z, wv.w * h4.w)));
        }
        int mine;                                                    // which of the NR rows this lane ends up with
        if (NR == 16) {
            fold_step<16, 16>(v, lane);
            fold_step<8, 8>(v, lane);
            fold_step<4, 4>(v, lane);
            fold_step<2, 2>(v, lane);
            v[0] += __shfl_xor(v[0], 1);
            mine = ((lane >> 4) & 1) * 8 + ((lane >> 3) & 1) * 4 + ((lane >> 2) & 1) * 2 + ((lane >> 1) & 1);
        } else {
            fold_step<4, 16>(v, lane);
            fold_step<2, 8>(v, lane);
            v[0] += __shfl_xor(v[0], 4);
            v[0] += __shfl_xor(v[0], 2);
            v[0] += __shfl_xor(v[0], 1);
            mine = ((lane >> 4) & 1) * 2 + ((lane >> 3) & 1);
        }
        const int blk = part + parts * (i0 + mine);
        const bool writer = NR == 16 ? (lane & 1) == 0 : (lane & 7) == 0;
        if (writer && blk * HW < rows) store(blk * HW + hwave, v[0]);
    }
}

// The step for state b once the input-free part exists, by one workgroup of kPolThreads threads;
// every thread must call it (it contains barriers).  Wavefront 0 only runs `wave0_inputs()`,
// which must leave the k confidences in s.x; meanwhile the other wavefronts fetch what the
// later phases need (w_ih into LDS, the head's rows into registers), so that once the inputs
// exist only arithmetic is left: cell update (wavefronts 8-15), head layer (1-15), logits (1).
// hidden(row) returns (w_hh h)[row] and is called only if has_state: with EARLY among the first
// loads (a value in global memory, complete before the call), otherwise after the first barrier
// (a value this workgroup wrote to LDS just before the call).
// h_out / c_out may be the arrays h_in / c_in.
// decided(action) is called by the one lane that has just written the outputs.
template <bool EARLY, typename Hidden, typename Inputs, typename Decided>
__device__ __forceinline__ void policy_step_block(const PolicyArgs &p, int b, bool has_state, PolicySmem &s,
                                                  Hidden &&hidden, Inputs &&wave0_inputs, Decided &&decided) {
    const int tid = threadIdx.x, w = tid / kWave, lane = tid % kWave;
    const int wk = w - 1;                                            // worker index, -1 for wavefront 0
    // cell update: wavefronts 8..15, 16 units each; lane = 16 * gate + unit within the wavefront
    const bool cell_thread = w >= kPolWaves / 2;
    const int gate_q = lane >> 4;
    const int u = (w - kPolWaves / 2) * 16 + (lane & 15);
    const int gate_row = gate_q * kPolH + u;

    float c_prev = 0.f, bias = 0.f, hid = 0.f;
    float hw[kPolHeadRows][3], b1v;                                  // head rows: columns lane, lane+64, lane+128
    float w2v[2][2], b2v[2], uni;
    const int rpw = (p.M + kPolWorkers - 1) / kPolWorkers, cols = kPolH + p.k;
    // after the head's fold a lane holds row 4*b5 + 2*b4 + b3 of its worker (b_n = bit n of the lane)
    const int head_i = ((lane >> 5) & 1) * 4 + ((lane >> 4) & 1) * 2 + ((lane >> 3) & 1);
    const int head_row = wk * rpw + head_i, last_row = wk * rpw + 8;
    const bool head_live = wk >= 0 && head_i < rpw && head_row < p.M;
    const bool last_live = wk >= 0 && 8 < rpw && last_row < p.M;

    if (w == 0) {
        wave0_inputs();
    } else {
        // Every lane loads from a clamped, valid address (a load under a lane mask makes the
        // compiler wait for it before the next one); rows and columns that do not exist are
        // discarded where the values are used.
        // ---- operands of the cell update (few, needed first)
        float b_a = 0.f, b_b = 0.f;
        if (cell_thread) {
            b_a = p.b_ih[gate_row];
            b_b = p.b_hh[gate_row];
            if (has_state) c_prev = p.c_in[(size_t)b * kPolH + u];
            if (EARLY && has_state) hid = hidden(gate_row);
        }
        // ---- w_ih: 4H * k floats, copied to LDS with coalesced loads (up to 9 per lane)
        constexpr int kCopies = (4 * kPolH * RADAR_K_MAX + kPolWorkers * kWave - 1) / (kPolWorkers * kWave);
        const int n_ih = 4 * kPolH * p.k, t = tid - kWave;
        float cp[kCopies];
#pragma unroll
        for (int i = 0; i < kCopies; ++i)
            if (i * kPolWorkers * kWave < n_ih) cp[i] = p.w_ih[min(t + i * kPolWorkers * kWave, n_ih - 1)];
        // ---- operands of the head
#pragma unroll
        for (int i = 0; i < kPolHeadRows; ++i) {
            const float *src = p.w1 + (size_t)min(wk * rpw + i, p.M - 1) * cols;
            hw[i][0] = src[lane];
            hw[i][1] = src[lane + 64];
            hw[i][2] = src[lane < p.k ? lane + 128 : 0];
        }
        b1v = p.b1[min(lane == 1 ? last_row : head_row, p.M - 1)];
        // (all workers fetch the last layer's few operands; only wavefront 1 uses them)
        w2v[0][0] = p.w2[min(lane, p.M - 1)];
        w2v[1][0] = p.w2[p.M + min(lane, p.M - 1)];
        w2v[0][1] = p.w2[min(lane + 64, p.M - 1)];
        w2v[1][1] = p.w2[p.M + min(lane + 64, p.M - 1)];
        b2v[0] = p.b2[0];
        b2v[1] = p.b2[1];
        uni = *(p.uniforms ? p.uniforms + b : p.b2);
#pragma unroll
        for (int i = 0; i < kCopies; ++i) {
            const int e = t + i * kPolWorkers * kWave;
            if (e < n_ih) s.wih[e + e / (kPolH * p.k)] = cp[i];
        }
        bias = b_a + b_b;
    }
    __syncthreads();

    // ---- cell update: every lane finishes one gate (input part, biases, activation; tanh of the
    // candidate gate as 2 sigm(2a) - 1 so that all lanes run the same code), then the four gates of
    // a unit meet in the lane of its input gate
    if (cell_thread) {
        if (!EARLY && has_state) hid = hidden(gate_row);
        float pre = bias + hid;
        const float *wrow = &s.wih[gate_row * p.k + gate_q];
        for (int i = 0; i < p.k; ++i) pre = fmaf(wrow[i], s.x[i], pre);
        const bool cand = gate_q == 2;
        const float sg = fast_sigmoid(cand ? 2.f * pre : pre);
        const float act = cand ? 2.f * sg - 1.f : sg;
        const float fg = __shfl(act, (lane & 15) + 16), gg = __shfl(act, (lane & 15) + 32), og = __shfl(act, (lane & 15) + 48);
        if (gate_q == 0) {
            const float cn = fmaf(fg, c_prev, act * gg);
            const float hn = og * fast_tanh(cn);
            s.hn[u] = hn;
            p.c_out[(size_t)b * kPolH + u] = cn;
            p.h_out[(size_t)b * kPolH + u] = hn;
        }
    }
    __syncthreads();

    // ---- first layer of the head on [h'; x], ReLU: up to 9 rows per worker
    if (w != 0) {
        const float in0 = s.hn[lane], in1 = s.hn[lane + 64];
        const float in2 = lane < p.k ? s.x[lane] : 0.f;
        float v[kPolHeadRows];
#pragma unroll
        for (int i = 0; i < kPolHeadRows; ++i) v[i] = fmaf(hw[i][0], in0, fmaf(hw[i][1], in1, hw[i][2] * in2));
        float last = v[8];
        fold_step<8, 32>(v, lane);
        fold_step<4, 16>(v, lane);
        fold_step<2, 8>(v, lane);
        float sum = v[0];
#pragma unroll
        for (int off = 4; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) last += __shfl_xor(last, off);
        if ((lane & 7) == 0 && head_live) s.z[head_row] = fmaxf(sum + b1v, 0.f);
        if (lane == 1 && last_live) s.z[last_row] = fmaxf(last + b1v, 0.f);
    }
    __syncthreads();

    // ---- two logits, softmax, action
    if (w == 1) {
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
            const float p1 = __frcp_rn(1.f + __expf(l0 - l1));
            const float p0 = __frcp_rn(1.f + __expf(l1 - l0));
            p.logits[2 * b] = l0;
            p.logits[2 * b + 1] = l1;
            p.probs[2 * b] = p0;
            p.probs[2 * b + 1] = p1;
            const int act = p.uniforms ? (uni < p1 ? 1 : 0) : (l1 > l0 ? 1 : 0);
            p.action[b] = act;
            decided(act);
        }
    }
}

}  // namespace radar
