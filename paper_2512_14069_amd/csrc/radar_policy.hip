// radar_policy_step: one call of the prediction model per state, one workgroup each
// (Sec. 4.2; App. A.3).  The arithmetic lives in radar_policy.h, shared with the fused tail
// of the expansion kernel.
#include "radar_host.h"
#include "radar_policy.h"

namespace radar {

__global__ __launch_bounds__(kPolThreads) void policy_kernel(PolicyArgs p, const float *conf, int has_state) {
    __shared__ PolicySmem s;
    const int b = blockIdx.x;
    if (has_state)
        policy_hidden_rows<16>(p, b, 0, 1, [&](int row, float v) { s.gate[row] = v; });
    policy_step_block<false>(
        p, b, has_state != 0, s, [&](int row) { return s.gate[row]; },
        [&] {
            if ((int)threadIdx.x < p.k) s.x[threadIdx.x] = conf[(size_t)b * p.k + threadIdx.x];
        },
        [](int) {});
}

// Host-side check of a parameter block; fills the kernel's argument struct.
radar_status policy_args_from(const radar_policy_params *pp, PolicyArgs *out) {
    if (!pp || !pp->w_ih || !pp->w_hh || !pp->b_ih || !pp->b_hh || !pp->w1 || !pp->b1 || !pp->w2 || !pp->b2)
        return RADAR_INVALID_ARG;
    if (pp->k < 1 || pp->M < 1 || pp->H < 1) return RADAR_INVALID_ARG;
    if (pp->H != kPolH || pp->k > RADAR_K_MAX || pp->M > kPolMMax) return RADAR_UNSUPPORTED_SHAPE;
    if (((uintptr_t)pp->w_hh & 15) != 0) return RADAR_INVALID_ARG;              // rows are read 16 bytes per lane
    PolicyArgs a{};
    a.w_ih = pp->w_ih; a.w_hh = pp->w_hh; a.b_ih = pp->b_ih; a.b_hh = pp->b_hh;
    a.w1 = pp->w1; a.b1 = pp->b1; a.w2 = pp->w2; a.b2 = pp->b2;
    a.k = pp->k; a.M = pp->M;
    *out = a;
    return RADAR_OK;
}

}  // namespace radar

using namespace radar;

extern "C" radar_status radar_policy_step(const float *conf, const float *h_in, const float *c_in,
                                          const radar_policy_params *params, const float *uniforms,
                                          float *h_out, float *c_out, float *logits, float *probs,
                                          int32_t *action, int32_t B, void *stream) {
    PolicyArgs a;
    const radar_status st = policy_args_from(params, &a);
    if (st != RADAR_OK) return st;
    if (!conf || !h_out || !c_out || !logits || !probs || !action || B < 0) return RADAR_INVALID_ARG;
    if ((h_in == nullptr) != (c_in == nullptr) || ((uintptr_t)h_in & 15) != 0) return RADAR_INVALID_ARG;
    if (B == 0) return RADAR_OK;
    a.h_in = h_in; a.c_in = c_in; a.uniforms = uniforms;
    a.h_out = h_out; a.c_out = c_out; a.logits = logits; a.probs = probs; a.action = action;
    const hipError_t e = launch("policy_step", policy_kernel, dim3(B), dim3(kPolThreads), 0,
                                static_cast<hipStream_t>(stream), a, conf, h_in ? 1 : 0);
    return e == hipSuccess ? RADAR_OK : RADAR_HIP_ERROR;
}
