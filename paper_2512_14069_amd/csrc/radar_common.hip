// Entry points that belong to no single step: status text, version, workspace clearing and the
// per-kernel timing table used for measurement.
#include <atomic>
#include <mutex>
#include <string.h>
#include <vector>

#include "radar_device.h"
#include "radar_host.h"

namespace radar {

__global__ void zero_fill_kernel(uint4 *p, size_t n16) {
    const uint4 z = make_uint4(0u, 0u, 0u, 0u);
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x) p[i] = z;
}

// Reads n16 x 16 bytes once, four independent loads per lane in flight, and keeps nothing: what a
// pure streaming read costs on this chip, the floor every streaming kernel here is compared with.
__global__ __launch_bounds__(256) void hbm_read_probe_kernel(const uint4 *p, size_t n16, uint32_t *sink) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    uint32_t acc = 0;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const uint4 a = p[i], b = p[i + stride], c = p[i + 2 * stride], d = p[i + 3 * stride];
        acc ^= (a.x ^ a.y ^ a.z ^ a.w) ^ (b.x ^ b.y ^ b.z ^ b.w) ^ (c.x ^ c.y ^ c.z ^ c.w) ^ (d.x ^ d.y ^ d.z ^ d.w);
    }
    for (; i < n16; i += stride) {
        const uint4 a = p[i];
        acc ^= a.x ^ a.y ^ a.z ^ a.w;
    }
    if (acc == 0x9e3779b9u && sink) *sink = acc;          // keeps the loads alive; practically never taken
}

namespace {
struct ProfRecord { const char *name; hipEvent_t start, stop; };
std::mutex g_prof_mutex;
std::vector<ProfRecord> g_prof;          // event pairs created by radar_profile_begin
size_t g_prof_used = 0;
std::atomic<bool> g_prof_on{false};
}  // namespace

bool profile_slot(const char *name, hipEvent_t *start, hipEvent_t *stop) {
    if (!g_prof_on) return false;        // unlocked fast path: the flag only changes in begin/end
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    if (!g_prof_on || g_prof_used >= g_prof.size()) return false;
    ProfRecord &r = g_prof[g_prof_used++];
    r.name = name;
    *start = r.start;
    *stop = r.stop;
    return true;
}

static void profile_release() {
    for (ProfRecord &r : g_prof) {
        if (r.start) (void)hipEventDestroy(r.start);
        if (r.stop) (void)hipEventDestroy(r.stop);
    }
    g_prof.clear();
    g_prof_used = 0;
    g_prof_on = false;
}

}  // namespace radar

using namespace radar;

extern "C" radar_status radar_workspace_init(void *workspace, size_t bytes, void *stream) {
    if (!workspace || bytes < 4096 || ((uintptr_t)workspace & 255) != 0) return RADAR_INVALID_ARG;
    const size_t n16 = bytes / 16;
    const unsigned blocks = (unsigned)((n16 + 255) / 256 > 1024 ? 1024 : (n16 + 255) / 256);
    const hipError_t e = launch("zero_fill", zero_fill_kernel, dim3(blocks), dim3(256), 0,
                                static_cast<hipStream_t>(stream), static_cast<uint4 *>(workspace), n16);
    return e == hipSuccess ? RADAR_OK : RADAR_HIP_ERROR;
}

extern "C" radar_status radar_probe_hbm_read(const void *src, size_t bytes, uint32_t *sink, void *stream) {
    if (!src || bytes < 16 || ((uintptr_t)src & 15) != 0) return RADAR_INVALID_ARG;
    const size_t n16 = bytes / 16;
    // one 16-byte load per lane and pass; at most eight workgroups of 256 lanes per CU's worth of grid
    const size_t want = (n16 + 4 * 256 - 1) / (4 * 256);
    const unsigned blocks = (unsigned)(want < 1 ? 1 : (want > 2048 ? 2048 : want));
    const hipError_t e = launch("hbm_read_probe", hbm_read_probe_kernel, dim3(blocks), dim3(256), 0,
                                static_cast<hipStream_t>(stream), static_cast<const uint4 *>(src), n16, sink);
    return e == hipSuccess ? RADAR_OK : RADAR_HIP_ERROR;
}

extern "C" const char *radar_status_string(radar_status status) {
    switch (status) {
        case RADAR_OK: return "ok";
        case RADAR_INVALID_ARG: return "invalid argument";
        case RADAR_UNSUPPORTED_SHAPE: return "shape outside the compiled limits";
        case RADAR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case RADAR_HIP_ERROR: return "HIP runtime error";
        default: return "unknown status";
    }
}

extern "C" int radar_version(void) { return 300; }   // 0.3.0: draft calls for a batch of sequences; 0.2.0: prediction model, cycle state, draft-distribution verification

extern "C" radar_status radar_profile_begin(int32_t max_launches) {
    if (max_launches < 1 || max_launches > (1 << 20)) return RADAR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    profile_release();
    g_prof.resize((size_t)max_launches, ProfRecord{nullptr, nullptr, nullptr});
    for (ProfRecord &r : g_prof) {
        if (hipEventCreate(&r.start) != hipSuccess || hipEventCreate(&r.stop) != hipSuccess) {
            profile_release();
            return RADAR_HIP_ERROR;
        }
    }
    g_prof_on = true;
    return RADAR_OK;
}

extern "C" radar_status radar_profile_end(radar_kernel_time *out, int32_t capacity, int32_t *n_out) {
    if (!n_out || capacity < 0 || (capacity > 0 && !out)) return RADAR_INVALID_ARG;
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    g_prof_on = false;
    int n = 0;
    radar_status st = RADAR_OK;
    for (size_t i = 0; i < g_prof_used; ++i) {
        const ProfRecord &r = g_prof[i];
        if (hipEventSynchronize(r.stop) != hipSuccess) { st = RADAR_HIP_ERROR; break; }
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess) { st = RADAR_HIP_ERROR; break; }
        const double us = (double)ms * 1e3;
        int j = 0;
        while (j < n && strncmp(out[j].name, r.name, sizeof(out[j].name) - 1) != 0) ++j;
        if (j == n) {
            if (n == capacity) continue;                 // table full: further names are dropped
            memset(&out[n], 0, sizeof(out[n]));
            strncpy(out[n].name, r.name, sizeof(out[n].name) - 1);
            out[n].min_us = us;
            out[n].max_us = us;
            ++n;
        }
        out[j].calls += 1;
        out[j].total_us += us;
        if (us < out[j].min_us) out[j].min_us = us;
        if (us > out[j].max_us) out[j].max_us = us;
    }
    profile_release();
    *n_out = n;
    return st;
}
