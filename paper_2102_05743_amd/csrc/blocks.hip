// Carries between the blocks of a sequence from the blocks' elements (Sec. V-B: a block of
// consecutive steps is one element of the scan; Theorems 1-2 and the lemma of Sec. IV-C applied at
// block granularity).
//
// With W_s the element of block s (joint weight of the block's observations and its last state given
// its first state, no transition into the first step) and p_0 = prior:
//     c_s = p_s (x) W_s        forward potential at the last step of block s (scaled: sum one / max zero)
//     p_{s+1} = c_s (x) A      its prediction for the first step of the next block
// and with r_{S-1} = neutral:
//     u_s = W_s (x) r_s        backward potential at the first step of block s, that step's emission
//                              factor included (scaled: max one / zero)
//     r_{s-1} = A (x) u_s      backward potential at the last step of block s-1.
// log c_{s-1} and log u_{s+1} are what block s needs from the rest of the sequence: as one more
// log-likelihood row in front of and behind its own rows they make a stand-alone call on the block
// reproduce the whole sequence's results on its steps.
//
// The number of blocks is small and every hop is a D x D matrix-vector product: one workgroup per
// sequence walks the blocks in order, lane j owning component j.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "blocks.hpp"
#include "ktimer.hpp"

namespace hmm {

#define HMM_DEV __device__ __forceinline__

namespace {

constexpr int BC_THREADS = 128;

template <bool MP>
HMM_DEV float bc_zero() { return MP ? -INFINITY : 0.0f; }

template <bool MP>
HMM_DEV float bc_acc(float acc, float a, float b) { return MP ? fmaxf(acc, a + b) : fmaf(a, b, acc); }

HMM_DEV float bc_log(float p) { return p > 0.0f ? logf(p) : -INFINITY; }

// Sum or maximum over the workgroup's lanes, delivered to every lane.
template <bool MAX>
HMM_DEV float bc_reduce(float v, float* red) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        const float o = __shfl_xor(v, d, 64);
        v = MAX ? fmaxf(v, o) : v + o;
    }
    __syncthreads();   // earlier readers of red are done
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return MAX ? fmaxf(red[0], red[1]) : red[0] + red[1];
}

template <bool MP>
__global__ __launch_bounds__(BC_THREADS) void block_carries_kernel(const float* __restrict__ prior, const float* __restrict__ A,
                                                                   const float* __restrict__ elements,
                                                                   const double* __restrict__ log_scales, int S, int D,
                                                                   int batch, int shared_model,
                                                                   float* __restrict__ carry_rows,
                                                                   float* __restrict__ lookahead_rows,
                                                                   double* __restrict__ total) {
    __shared__ float vec[BC_THREADS];
    __shared__ float red[2];
    const int b = blockIdx.x, j = threadIdx.x;
    const bool live = j < D;
    const float* Am = A + (shared_model ? 0 : (size_t)b * D * D);
    const float* pr = prior + (shared_model ? 0 : (size_t)b * D);
    auto W = [&](int s) { return elements + ((size_t)s * batch + b) * D * D; };
    auto row = [&](float* rows, int s) { return rows + ((size_t)s * batch + b) * D; };
    auto a_dom = [&](int i, int k) { const float a = Am[(size_t)i * D + k]; return MP ? bc_log(a) : a; };

    // forward
    float p = live ? pr[j] : 0.0f;
    {
        const float pm = bc_reduce<true>(live ? p : 0.0f, red);
        if (live) row(carry_rows, 0)[j] = bc_log(p / pm);
    }
    if (MP) p = live ? bc_log(p) : -INFINITY;
    double tot = 0.0;
    for (int s = 0; s < S; ++s) {
        __syncthreads();
        vec[j] = live ? p : bc_zero<MP>();
        __syncthreads();
        float c = bc_zero<MP>();
        if (live) {
            const float* Ws = W(s);
            for (int i = 0; i < D; ++i) c = bc_acc<MP>(c, vec[i], Ws[(size_t)i * D + j]);
        }
        const float nrm = bc_reduce<MP>(c, red);
        tot += (MP ? (double)nrm : log((double)nrm)) + log_scales[(size_t)s * batch + b];
        c = MP ? c - nrm : c / nrm;
        if (live && s + 1 < S) row(carry_rows, s + 1)[j] = MP ? c : bc_log(c);
        __syncthreads();
        vec[j] = live ? c : bc_zero<MP>();
        __syncthreads();
        p = bc_zero<MP>();
        if (live)
            for (int i = 0; i < D; ++i) p = bc_acc<MP>(p, vec[i], a_dom(i, j));
    }
    if (j == 0) total[b] = tot;

    // backward
    float r = MP ? 0.0f : 1.0f;
    if (live) row(lookahead_rows, S - 1)[j] = 0.0f;
    for (int s = S - 1; s >= 1; --s) {
        __syncthreads();
        vec[j] = live ? r : bc_zero<MP>();
        __syncthreads();
        float u = bc_zero<MP>();
        if (live) {
            const float* Ws = W(s) + (size_t)j * D;
            for (int k = 0; k < D; ++k) u = bc_acc<MP>(u, Ws[k], vec[k]);
        }
        const float m = bc_reduce<true>(live ? u : bc_zero<MP>(), red);
        u = MP ? u - m : u / m;
        if (live) row(lookahead_rows, s - 1)[j] = MP ? u : bc_log(u);
        __syncthreads();
        vec[j] = live ? u : bc_zero<MP>();
        __syncthreads();
        r = bc_zero<MP>();
        if (live)
            for (int k = 0; k < D; ++k) r = bc_acc<MP>(r, a_dom(j, k), vec[k]);
    }
}

}  // namespace

int block_carries(const BlockCarryArgs& a, float* carry_rows, float* lookahead_rows, double* total) {
    const dim3 grid((unsigned)a.batch), block(BC_THREADS);
    if (a.max_product)
        launch("block_carries_mp", block_carries_kernel<true>, grid, block, a.stream, a.prior, a.A, a.elements, a.log_scales,
               a.S, a.D, a.batch, a.shared_model, carry_rows, lookahead_rows, total);
    else
        launch("block_carries_sp", block_carries_kernel<false>, grid, block, a.stream, a.prior, a.A, a.elements, a.log_scales,
               a.S, a.D, a.batch, a.shared_model, carry_rows, lookahead_rows, total);
    return hipGetLastError() == hipSuccess ? 0 : 4;
}

}  // namespace hmm
