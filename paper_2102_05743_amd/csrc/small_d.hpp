// Host-side entry points of the register-resident (D <= 8) path.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace hmm {

struct SmallArgs {
    const float* prior;
    const float* A;
    const float* ll;
    long long T;
    int batch;
    int shared_model;
    void* ws;
    size_t ws_bytes;
    hipStream_t stream;
};

constexpr int SMALL_D_MAX = 8;

// Every workspace of the library begins with the exchange region of the single-launch plan (header and
// tagged slots for up to XCH_MAX_TILES co-resident tiles of up to SMALL_D_MAX states); see
// small_d_device.hpp.  It must be zero before a workspace's first use.
constexpr int XCH_MAX_TILES = 512;
constexpr size_t XCH_REGION_BYTES = 384 * 1024;

// One explicit instantiation per D, each in its own translation unit (small_d_kernels.hip
// compiled with -DHMM_SMALL_D=<D>).  Return codes follow hmm_status.
template <int D>
struct SmallD {
    static size_t smooth_ws_bytes(long long T, int batch);
    static long long tiles(long long T);   // tiles per sequence
    static size_t viterbi_ws_bytes(long long T, int batch);
    static int smooth(const SmallArgs& a, float* marg, float* filt, double* loglik_out);
    // the smoother that also leaves per-tile sums of pairwise posteriors (pair_partial[batch * tiles][D*D], tiles =
    // tiles per sequence, reported)
    static int smooth_pairs(const SmallArgs& a, float* marg, double* loglik_out, float* pair_partial, long long* tiles);
    static int viterbi(const SmallArgs& a, int32_t* path, double* logprob_out);
    static int max_product(const SmallArgs& a, float* maxmarg, int32_t* path, double* logprob_out);
    static size_t element_ws_bytes(long long T, int batch);
    static int block_element(const SmallArgs& a, int max_product, float* element, double* log_scale);   // a.prior unused
};

size_t small_d_smooth_ws_bytes(int D, long long T, int batch);
size_t small_d_viterbi_ws_bytes(int D, long long T, int batch);
int small_d_smooth(int D, const SmallArgs& a, float* marg, float* filt, double* loglik_out);
int small_d_smooth_pairs(int D, const SmallArgs& a, float* marg, double* loglik_out, float* pair_partial, long long* tiles);
long long small_d_tiles(int D, long long T);   // tiles per sequence (0 for sizes this path does not take)
int small_d_viterbi(int D, const SmallArgs& a, int32_t* path, double* logprob_out);
int small_d_max_product(int D, const SmallArgs& a, float* maxmarg, int32_t* path, double* logprob_out);
size_t small_d_element_ws_bytes(int D, long long T, int batch);
int small_d_block_element(int D, const SmallArgs& a, int max_product, float* element, double* log_scale);
int small_d_zero_region(void* ws, size_t bytes, hipStream_t stream);   // zero fill enqueued on the stream

}  // namespace hmm
