// Host-side entry point of the carries between the blocks of a sequence.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace hmm {

struct BlockCarryArgs {
    const float* prior;
    const float* A;
    const float* elements;      // [S][batch][D][D]
    const double* log_scales;   // [S][batch]
    int S;
    int D;
    int batch;
    int shared_model;
    int max_product;
    hipStream_t stream;
};

// Return codes follow hmm_status (0 ok, 4 device).
int block_carries(const BlockCarryArgs& a, float* carry_rows, float* lookahead_rows, double* total);

}  // namespace hmm
