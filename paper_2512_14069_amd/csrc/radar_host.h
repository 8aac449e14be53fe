// Host-side launch helper shared by the entry points.
//
// Every kernel of the library is launched through radar::launch().  Normally that is a plain
// launch.  Between radar_profile_begin and radar_profile_end each launch carries a pair of
// events that the runtime stamps with the dispatch's own begin and end times on the device
// (the same time stamps a kernel trace shows), so a caller can read per-kernel durations
// without a profiler attached.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

namespace radar {

// Next free (start, stop) pair for a launch named `name` (static string), or false when
// profiling is off or the table is full.
bool profile_slot(const char *name, hipEvent_t *start, hipEvent_t *stop);

template <typename... Params, typename... Args>
inline hipError_t launch(const char *name, void (*kernel)(Params...), dim3 grid, dim3 block, unsigned smem,
                         hipStream_t stream, Args... args) {
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (profile_slot(name, &e0, &e1))
        hipExtLaunchKernelGGL(kernel, grid, block, smem, stream, e0, e1, 0u, static_cast<Params>(args)...);
    else
        hipLaunchKernelGGL(kernel, grid, block, smem, stream, static_cast<Params>(args)...);   // the form a stream capture records
    return hipGetLastError();
}

}  // namespace radar
