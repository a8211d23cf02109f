// hmm_smooth_static: hmm_smooth for callers that cannot allocate device memory (code under HIP
// graph capture, serving loops, harnesses that forbid hipMalloc).  The scratch memory that
// hmm_smooth takes as its workspace argument is a file-scope device array of this library instead;
// every kernel is the one hmm_smooth launches and receives the array's device address as its
// workspace pointer.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "../../include/hmmscan.h"

namespace {

// One copy per GPU that loads the library, held until the process ends.
static __device__ __align__(256) unsigned char scratch[HMM_STATIC_SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex g_lock;
void* g_scratch_ptr[MAX_DEVICES];   // device address of `scratch` on each device, looked up once per device

// Device address of the current device's copy of `scratch` (in host code the array's name is only a
// handle for this lookup, never a device address).
hmm_status scratch_address(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return HMM_ERR_DEVICE;
    std::lock_guard<std::mutex> guard(g_lock);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return HMM_ERR_DEVICE;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return HMM_OK;
}

}  // namespace

extern "C" hmm_status hmm_smooth_static(const float* prior, const float* A, const float* loglik, int64_t T, int32_t D,
                                        int32_t batch, int32_t shared_model, float* marginals, float* filtered,
                                        double* loglik_out, void* hip_stream) {
    // argument errors first, exactly as hmm_smooth reports them: with no workspace a call with valid arguments
    // can only end in HMM_ERR_WORKSPACE, anything else is the verdict on the arguments
    const hmm_status args = hmm_smooth(prior, A, loglik, T, D, batch, shared_model, marginals, filtered, loglik_out,
                                       nullptr, 0, hip_stream);
    if (args != HMM_ERR_WORKSPACE) return args;
    // the shape's scratch need is known on the host: too large a shape is refused before any device call
    size_t need = 0;
    const hmm_status st = hmm_workspace_bytes(T, D, batch, &need, nullptr);
    if (st != HMM_OK) return st;
    if (need > (size_t)HMM_STATIC_SCRATCH_BYTES) return HMM_ERR_WORKSPACE;
    void* ws = nullptr;
    const hmm_status sa = scratch_address(&ws);
    if (sa != HMM_OK) return sa;
    return hmm_smooth(prior, A, loglik, T, D, batch, shared_model, marginals, filtered, loglik_out, ws,
                      (size_t)HMM_STATIC_SCRATCH_BYTES, hip_stream);
}
