// Host-side entry points of the large-state-space path (9 <= D <= 128).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace hmm {

struct LargeArgs {
    const float* prior;
    const float* A;
    const float* ll;
    long long T;
    int D;            // number of states as given by the caller (kernels pad it internally)
    int batch;
    int shared_model;
    void* ws;
    size_t ws_bytes;
    hipStream_t stream;
};

struct LargePlan {
    int DP;             // padded state count: 16, 32, 64 or 128
    int Lc;             // time steps per chunk (multiple of 16)
    int cps;            // chunks per sequence
    long long nchunks;  // cps * batch
};

LargePlan large_plan(int D, long long T, int batch);

// Return codes follow hmm_status (0 ok, 2 unsupported, 3 workspace, 4 device).
size_t large_d_smooth_ws_bytes(int D, long long T, int batch);
int large_d_smooth(const LargeArgs& a, float* marg, float* filt, double* loglik_out);
size_t large_d_viterbi_ws_bytes(int D, long long T, int batch);
int large_d_viterbi(const LargeArgs& a, int32_t* path, double* logprob_out);
size_t large_d_max_product_ws_bytes(int D, long long T, int batch);   // never more than the smoother's
int large_d_max_product(const LargeArgs& a, float* maxmarg, int32_t* path, double* logprob_out);

// Block-wise elements (a.prior unused).
LargePlan element_plan(int D, long long T, int batch);
size_t large_d_element_sp_ws_bytes(int D, long long T, int batch);
int large_d_element_sp(const LargeArgs& a, float* element, double* log_scale);
size_t large_d_element_mp_ws_bytes(int D, long long T, int batch);
int large_d_element_mp(const LargeArgs& a, float* element, double* log_scale);

}  // namespace hmm
