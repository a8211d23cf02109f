// Host-side entry points of the expectation-step statistics.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace hmm {

struct EstepArgs {
    const float* A;
    const float* filtered;
    const float* marginals;
    long long T;
    int D;
    int batch;
    int shared_model;
    void* ws;
    size_t ws_bytes;
    hipStream_t stream;
};

// Return codes follow hmm_status (0 ok, 2 unsupported, 3 workspace, 4 device).
size_t transition_counts_ws_bytes(int D, long long T, int batch);
int transition_counts(const EstepArgs& a, double* counts);
// counts[seq] = sum over the sequence's G partial sums (partial[seq][G][D*D] floats, D <= 8), in fp64
int reduce_pair_partials(const float* partial, int G, int D, int batch, double* counts, hipStream_t stream);

}  // namespace hmm
