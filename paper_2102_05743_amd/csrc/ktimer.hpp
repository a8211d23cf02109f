// Kernel launch helper with optional per-kernel timing.  When timing is switched on, a launch
// goes through hipExtLaunchKernelGGL with a start and a stop event attached to the kernel's own
// dispatch, so the elapsed time between them is the kernel's execution time (what a profiler's
// kernel trace reports), not the time between two separately enqueued event markers.
// Off by default; not thread-safe; meant for single-threaded measurement.
#pragma once
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>

namespace hmm {

bool ktimer_enabled();
// Appends a record for one launch and hands out its two events (nullptr if none could be made).
void ktimer_new_record(const char* name, hipEvent_t* start, hipEvent_t* stop);

template <class... KArgs, class... Args>
inline void launch(const char* name, void (*kernel)(KArgs...), dim3 grid, dim3 block, hipStream_t stream,
                   Args&&... args) {
    if (ktimer_enabled()) {
        hipEvent_t e0 = nullptr, e1 = nullptr;
        ktimer_new_record(name, &e0, &e1);
        hipExtLaunchKernelGGL(kernel, grid, block, 0, stream, e0, e1, 0, static_cast<KArgs>(args)...);
    } else {
        hipLaunchKernelGGL(kernel, grid, block, 0, stream, static_cast<KArgs>(args)...);
    }
}

// Same with dynamic LDS.
template <class... KArgs, class... Args>
inline void launch_dyn(const char* name, void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds_bytes,
                       hipStream_t stream, Args&&... args) {
    if (ktimer_enabled()) {
        hipEvent_t e0 = nullptr, e1 = nullptr;
        ktimer_new_record(name, &e0, &e1);
        hipExtLaunchKernelGGL(kernel, grid, block, (uint32_t)lds_bytes, stream, e0, e1, 0, static_cast<KArgs>(args)...);
    } else {
        hipLaunchKernelGGL(kernel, grid, block, (uint32_t)lds_bytes, stream, static_cast<KArgs>(args)...);
    }
}

}  // namespace hmm
