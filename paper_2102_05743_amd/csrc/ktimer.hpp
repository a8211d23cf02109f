// Optional per-kernel timing: when switched on, every kernel launch of the library is bracketed by
// HIP events recorded on the caller's stream, so a benchmark can attribute time to kernels without
// an external profiler.  Off by default; not thread-safe; meant for single-threaded measurement.
#pragma once
#include <hip/hip_runtime.h>

namespace hmm {

bool ktimer_enabled();
void ktimer_begin(const char* name, hipStream_t stream);
void ktimer_end(hipStream_t stream);

struct KernelScope {
    hipStream_t s;
    bool on;
    KernelScope(const char* name, hipStream_t stream) : s(stream), on(ktimer_enabled()) {
        if (on) ktimer_begin(name, s);
    }
    ~KernelScope() {
        if (on) ktimer_end(s);
    }
};

}  // namespace hmm
