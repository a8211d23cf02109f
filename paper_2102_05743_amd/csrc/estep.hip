// Expected transition counts of the Baum-Welch expectation step (Sec. V-C: its core is the
// forward-backward recursion, i.e. hmm_smooth), computed from the smoother's own outputs.
//
// The pairwise posterior of the chain, p(x_{k-1}=i, x_k=j | y_{1:T}) = psi^f_{k-1}(i) psi_k(i,j) psi^b_k(j) / Z,
// summed over j gives the marginal of step k-1 and summed over i the marginal gamma_k(j) of step k.
// With the filtering distribution fh_{k-1}(i) = p(x_{k-1}=i | y_{1:k-1}) and its one-step prediction
// pred_k(j) = sum_i fh_{k-1}(i) A(i,j), every factor that depends on j alone collects into
// gamma_k(j) / pred_k(j), so
//     counts(i,j) = A(i,j) * sum_{k=2..T} fh_{k-1}(i) * gamma_k(j) / pred_k(j)            (0 where pred_k(j) = 0):
// a pass over the filtered and smoothed arrays with 2 D^2 multiply-adds per step.  Steps are split
// over workgroups, each leaves a partial D x D sum in the workspace, a last kernel adds them in fp64.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "estep.hpp"
#include "ktimer.hpp"
#include "large_d_device.hpp"

namespace hmm {

// transitions k = 1..T-1 (0-based step index of the later state) of one sequence, split over G workgroups
// A predicted probability pred_k(j) below the smallest normal number counts as zero: the pairwise posteriors it
// scales sum to gamma_k(j) <= pred_k(j) e_k(j) b_k(j) / Z_k, i.e. nothing at this precision, while the fast
// reciprocal of a subnormal is infinite and would turn a marginal that has itself underflowed to zero into NaN.
constexpr float PRED_MIN = 1.17549435e-38f;

struct StepRange { long long k0, k1; };
HMM_DEV StepRange step_range(long long T, int G, int g) {
    const long long n = T - 1;
    const long long per = (n + G - 1) / G;
    StepRange r;
    r.k0 = 1 + (long long)g * per;
    r.k1 = r.k0 + per;
    if (r.k1 > T) r.k1 = T;
    if (r.k0 > T) r.k0 = T;
    return r;
}

// ---------------------------------------------------------------------------------------------
// D <= 8: one lane per step, the D x D accumulator in registers.
template <int D>
__global__ __launch_bounds__(256) void tc_small_kernel(const float* __restrict__ A, const float* __restrict__ filt,
                                                       const float* __restrict__ marg, long long T, int G,
                                                       int shared_model, float* __restrict__ partial,
                                                       double* __restrict__ direct) {
    __shared__ float red[4 * D * D];
    const int seq = blockIdx.x / G, g = blockIdx.x % G;
    const StepRange sr = step_range(T, G, g);
    const float* Am = A + (shared_model ? 0 : (size_t)seq * D * D);
    float a[D * D], acc[D * D];
#pragma unroll
    for (int e = 0; e < D * D; ++e) { a[e] = Am[e]; acc[e] = 0.0f; }
    const float* fs = filt + (size_t)seq * T * D;
    const float* ms = marg + (size_t)seq * T * D;
    for (long long k = sr.k0 + threadIdx.x; k < sr.k1; k += 256) {
        float f[D], gm[D];
#pragma unroll
        for (int j = 0; j < D; ++j) { f[j] = fs[(size_t)(k - 1) * D + j]; gm[j] = ms[(size_t)k * D + j]; }
        float w[D];
#pragma unroll
        for (int j = 0; j < D; ++j) {
            float pred = 0.0f;
#pragma unroll
            for (int i = 0; i < D; ++i) pred = fmaf(f[i], a[i * D + j], pred);
            w[j] = pred >= PRED_MIN ? gm[j] / pred : 0.0f;
        }
#pragma unroll
        for (int i = 0; i < D; ++i)
#pragma unroll
            for (int j = 0; j < D; ++j) acc[i * D + j] = fmaf(f[i], w[j], acc[i * D + j]);
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int e = 0; e < D * D; ++e) {
        float v = acc[e] * a[e];
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) v += __shfl_down(v, d, 64);
        if (lane == 0) red[wave * D * D + e] = v;
    }
    __syncthreads();
    if (threadIdx.x < D * D) {
        const float v =
            (red[threadIdx.x] + red[D * D + threadIdx.x]) + (red[2 * D * D + threadIdx.x] + red[3 * D * D + threadIdx.x]);
        // one workgroup per sequence (G == 1): the sum is the sequence's count, written without a second pass
        if (direct != nullptr) direct[(size_t)blockIdx.x * D * D + threadIdx.x] = (double)v;
        else partial[(size_t)blockIdx.x * D * D + threadIdx.x] = v;
    }
}

// The same for short sequences (at most 1025 steps): a sequence takes an aligned group of 2^lg lanes of a
// wave (at most 16 steps per lane), several sequences share a workgroup, the group's lanes are summed by
// shuffles and its first lane writes the sequence's counts directly: one launch, no partial sums.
template <int D>
__global__ __launch_bounds__(256) void tc_small_packed_kernel(const float* __restrict__ A, const float* __restrict__ filt,
                                                              const float* __restrict__ marg, long long T, int batch,
                                                              int lg, int shared_model, double* __restrict__ counts) {
    const int gsz = 1 << lg;
    const int spw = 256 >> lg;
    const int q = (int)threadIdx.x >> lg, c = (int)threadIdx.x & (gsz - 1);
    const long long seq_raw = (long long)blockIdx.x * spw + q;
    const bool live = seq_raw < batch;
    const size_t seq = live ? (size_t)seq_raw : 0;
    const float* Am = A + (shared_model ? 0 : seq * D * D);
    float a[D * D], acc[D * D];
#pragma unroll
    for (int e = 0; e < D * D; ++e) { a[e] = Am[e]; acc[e] = 0.0f; }
    const float* fs = filt + seq * T * D;
    const float* ms = marg + seq * T * D;
    if (live) {
        for (long long k = 1 + c; k < T; k += gsz) {
            float f[D], gm[D];
#pragma unroll
            for (int j = 0; j < D; ++j) { f[j] = fs[(size_t)(k - 1) * D + j]; gm[j] = ms[(size_t)k * D + j]; }
            float w[D];
#pragma unroll
            for (int j = 0; j < D; ++j) {
                float pred = 0.0f;
#pragma unroll
                for (int i = 0; i < D; ++i) pred = fmaf(f[i], a[i * D + j], pred);
                w[j] = pred >= PRED_MIN ? gm[j] / pred : 0.0f;
            }
#pragma unroll
            for (int i = 0; i < D; ++i)
#pragma unroll
                for (int j = 0; j < D; ++j) acc[i * D + j] = fmaf(f[i], w[j], acc[i * D + j]);
        }
    }
#pragma unroll
    for (int e = 0; e < D * D; ++e) {
        float v = acc[e] * a[e];
        for (int d = gsz >> 1; d >= 1; d >>= 1) v += __shfl_down(v, d, 64);
        if (live && c == 0) counts[seq * D * D + e] = (double)v;
    }
}

// ---------------------------------------------------------------------------------------------
// 9 <= D <= 32 (padded to DP = 16 or 32): one time step per DPP row of 16 lanes, sixteen steps per
// workgroup round, no LDS in the loop.  Lane l holds components 16 q + l of fh_{k-1} and gamma_k.  Both the
// prediction pred_k(j) = sum_i fh_{k-1}(i) A(i,j) and the outer product fh_{k-1}(i) w_k(j) pair component
// (l - r) mod 16 of one vector with component l of another: the first operand of a multiply-add read
// through a rotation of the row by r lanes.  The lane accumulates entry (16 qs + (l - r) mod 16, 16 qd + l)
// in acc[(qs, qd)][r].  Steps are independent, so four of a row's steps have their loads in flight at once.
template <int DP>
__global__ __launch_bounds__(256) void tc_row_kernel(const float* __restrict__ A, const float* __restrict__ filt,
                                                     const float* __restrict__ marg, long long T, int Dr, int G,
                                                     int shared_model, float* __restrict__ partial,
                                                     double* __restrict__ direct) {
    static_assert(DP == 16 || DP == 32, "one DPP row per step");
    constexpr int NQ = DP / 16;
    constexpr int UNR = 4;
    __shared__ float red[4 * DP * DP];
    const int seq = blockIdx.x / G, g = blockIdx.x % G;
    const StepRange sr = step_range(T, G, g);
    const int l = threadIdx.x & 15, row = threadIdx.x >> 4;
    const float* Am = A + (shared_model ? 0 : (size_t)seq * Dr * Dr);
    float a[NQ * NQ * 16];
#pragma unroll
    for (int qs = 0; qs < NQ; ++qs)
#pragma unroll
        for (int qd = 0; qd < NQ; ++qd)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int i = 16 * qs + ((l - r) & 15), j = 16 * qd + l;
                a[(qs * NQ + qd) * 16 + r] = (i < Dr && j < Dr) ? Am[(size_t)i * Dr + j] : 0.0f;
            }
    float acc[NQ * NQ][16];
#pragma unroll
    for (int b = 0; b < NQ * NQ; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[b][r] = 0.0f;
    const float* fs = filt + (size_t)seq * T * Dr;
    const float* ms = marg + (size_t)seq * T * Dr;
    int col[NQ];
    bool have[NQ];
#pragma unroll
    for (int q = 0; q < NQ; ++q) { have[q] = 16 * q + l < Dr; col[q] = have[q] ? 16 * q + l : 0; }
    for (long long kb = sr.k0 + row; kb < sr.k1; kb += 16 * UNR) {
        float f[UNR][NQ], gm[UNR][NQ];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const long long k = kb + 16 * u;
            const long long kc = k < sr.k1 ? k : sr.k1 - 1;   // past the range: a valid step, contribution masked below
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                f[u][q] = fs[(size_t)(kc - 1) * Dr + col[q]];
                gm[u][q] = ms[(size_t)kc * Dr + col[q]];
            }
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const bool valid = kb + 16 * u < sr.k1;
            float fv[NQ];
#pragma unroll
            for (int q = 0; q < NQ; ++q) fv[q] = (valid && have[q]) ? f[u][q] : 0.0f;
            float pp[NQ][4];
            row_matvec_terms<NQ>(fv, a, pp);
#pragma unroll
            for (int qd = 0; qd < NQ; ++qd) {
                const float pred = (pp[qd][0] + pp[qd][1]) + (pp[qd][2] + pp[qd][3]);
                const float w = (pred >= PRED_MIN && have[qd]) ? gm[u][qd] * __builtin_amdgcn_rcpf(pred) : 0.0f;
#pragma unroll
                for (int qs = 0; qs < NQ; ++qs) row_outer16(fv[qs], w, acc[qs * NQ + qd]);
            }
        }
    }
    // entries times A(i, j), summed over the wave's four rows, then over the four waves through LDS
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int qs = 0; qs < NQ; ++qs)
#pragma unroll
        for (int qd = 0; qd < NQ; ++qd)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float v = acc[qs * NQ + qd][r] * a[(qs * NQ + qd) * 16 + r];
                v += __shfl_xor(v, 16, 64);
                v += __shfl_xor(v, 32, 64);
                if (lane < 16) {
                    const int i = 16 * qs + ((l - r) & 15), j = 16 * qd + l;
                    red[wave * DP * DP + i * DP + j] = v;
                }
            }
    __syncthreads();
    for (int e = threadIdx.x; e < DP * DP; e += 256) {
        const float v = (red[e] + red[DP * DP + e]) + (red[2 * DP * DP + e] + red[3 * DP * DP + e]);
        if (direct != nullptr) {   // G == 1: the sequence's count itself
            const int i = e / DP, j = e % DP;
            if (i < Dr && j < Dr) direct[((size_t)blockIdx.x * Dr + i) * Dr + j] = (double)v;
        } else {
            partial[(size_t)blockIdx.x * DP * DP + e] = v;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// D > 32 (padded to DP = 64 or 128): both sums are dense contractions over a slab of 32 time steps and
// run on the FP32 matrix cores (v_mfma_f32_32x32x2_f32):
//     pred  (32 x DP)  = F_slab (32 x DP) * A (DP x DP)           first operand from LDS, second (A) in registers
//     W     (32 x DP)  = Gamma_slab / pred                        element-wise on the result registers
//     C     (DP x DP) += F_slab^T (DP x 32) * W (32 x DP)         first operand from LDS, second = the W registers
// A wave owns a block of 32 columns j.  A result register r of lane group g = lane / 32 holds row
// 8 (r / 4) + 4 g + r % 4 of its tile, and the second operand of the next product wants one row of W per
// lane group: enumerating the time steps of the slab in exactly that order (first operand read from LDS
// accordingly) lets the W registers be fed back as they are.  With DP = 64 there are two column blocks;
// the other two waves take every second slab and the two partial results are added at the end.
template <int DP>
__global__ __launch_bounds__(256) void tc_mfma_kernel(const float* __restrict__ A, const float* __restrict__ filt,
                                                      const float* __restrict__ marg, long long T, int Dr, int G,
                                                      int shared_model, float* __restrict__ partial,
                                                      double* __restrict__ direct) {
    static_assert(DP == 64 || DP == 128, "column blocks of 32");
    constexpr int NB = DP / 32;          // column blocks = row blocks
    constexpr int SPW = 4 / NB;          // waves sharing a column block, each on its own slabs
    constexpr int SLAB = 32;
    constexpr int STR = DP + 1;          // LDS row stride (floats): conflict-free for both access patterns
    constexpr int PER = SPW * SLAB * DP / 256;   // staged values per thread and array
    typedef float v16 __attribute__((ext_vector_type(16)));
    __shared__ float fs[SPW * SLAB * STR];
    __shared__ float gs[SPW * SLAB * STR];
    const int seq = blockIdx.x / G, g = blockIdx.x % G;
    const StepRange sr = step_range(T, G, g);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int cb = wave % NB, sp = wave / NB;
    const int lg = lane >> 5, ln = lane & 31;
    const float* Am = A + (shared_model ? 0 : (size_t)seq * Dr * Dr);
    const float* fsq = filt + (size_t)seq * T * Dr;
    const float* msq = marg + (size_t)seq * T * Dr;
    // second operand of the first product: breg[kk] = A(2 kk + lg, 32 cb + ln)
    float breg[DP / 2];
#pragma unroll
    for (int kk = 0; kk < DP / 2; ++kk) {
        const int i = 2 * kk + lg, j = 32 * cb + ln;
        breg[kk] = (i < Dr && j < Dr) ? Am[(size_t)i * Dr + j] : 0.0f;
    }
    v16 acc[NB];
#pragma unroll
    for (int rb = 0; rb < NB; ++rb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[rb][r] = 0.0f;
    auto tile_row = [&](int r) { return 8 * (r / 4) + 4 * lg + (r % 4); };
    float pf[PER], pg[PER];
    auto load_round = [&](long long kb) {   // the SPW slabs starting at step kb, SLAB steps each
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            const int idx = q * 256 + tid;
            const int s = idx / DP, i = idx % DP;        // s over SPW * SLAB steps
            const long long k = kb + s;
            const bool valid = k < sr.k1 && i < Dr;
            pf[q] = valid ? fsq[(size_t)(k - 1) * Dr + i] : 0.0f;
            pg[q] = valid ? msq[(size_t)k * Dr + i] : 0.0f;
        }
    };
    auto store_round = [&]() {
#pragma unroll
        for (int q = 0; q < PER; ++q) {
            const int idx = q * 256 + tid;
            const int s = idx / DP, i = idx % DP;
            fs[s * STR + i] = pf[q];
            gs[s * STR + i] = pg[q];
        }
    };
    const long long round_steps = (long long)SPW * SLAB;
    if (sr.k0 < sr.k1) load_round(sr.k0);
    for (long long kb = sr.k0; kb < sr.k1; kb += round_steps) {
        __syncthreads();                 // the previous round's reads of the staging buffers are done
        store_round();
        __syncthreads();
        if (kb + round_steps < sr.k1) load_round(kb + round_steps);   // in flight during the products
        const float* fw = fs + sp * SLAB * STR;     // this wave's slab
        const float* gw = gs + sp * SLAB * STR;
        // pred = F_slab * A: rows = steps (ln), reduction over states i = 2 kk + lg
        v16 pred;
#pragma unroll
        for (int r = 0; r < 16; ++r) pred[r] = 0.0f;
#pragma unroll
        for (int kk = 0; kk < DP / 2; ++kk)
            pred = __builtin_amdgcn_mfma_f32_32x32x2f32(fw[ln * STR + 2 * kk + lg], breg[kk], pred, 0, 0, 0);
        // W = Gamma / pred in place (row tile_row(r), column 32 cb + ln)
        v16 w;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const float gm = gw[tile_row(r) * STR + 32 * cb + ln];
            w[r] = pred[r] >= PRED_MIN ? gm * __builtin_amdgcn_rcpf(pred[r]) : 0.0f;
        }
        // C(row block rb) += F_slab^T * W: reduction over the slab's steps in the order of the result rows
#pragma unroll
        for (int rb = 0; rb < NB; ++rb)
#pragma unroll
            for (int pr = 0; pr < 16; ++pr)
                acc[rb] = __builtin_amdgcn_mfma_f32_32x32x2f32(fw[tile_row(pr) * STR + 32 * rb + ln], w[pr], acc[rb], 0, 0, 0);
    }
    // entries times A(i, j); with two waves per column block their results are added through LDS first
    __syncthreads();
    if constexpr (SPW == 2) {
        // waves with sp = 1 deposit into the (now free) staging buffers, waves with sp = 0 add
        static_assert(SPW * SLAB * STR >= NB * 16 * 64, "room for a wave's partial results");
        float* buf = (cb == 0) ? fs : gs;
        if (sp == 1) {
#pragma unroll
            for (int rb = 0; rb < NB; ++rb)
#pragma unroll
                for (int r = 0; r < 16; ++r) buf[(rb * 16 + r) * 64 + lane] = acc[rb][r];
        }
        __syncthreads();
        if (sp == 0) {
#pragma unroll
            for (int rb = 0; rb < NB; ++rb)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[rb][r] += buf[(rb * 16 + r) * 64 + lane];
        }
    }
    if (sp == 0) {
#pragma unroll
        for (int rb = 0; rb < NB; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int i = 32 * rb + tile_row(r), j = 32 * cb + ln;
                const float a = (i < Dr && j < Dr) ? Am[(size_t)i * Dr + j] : 0.0f;
                if (direct != nullptr) {   // G == 1: the sequence's count itself
                    if (i < Dr && j < Dr) direct[((size_t)blockIdx.x * Dr + i) * Dr + j] = (double)(acc[rb][r] * a);
                } else {
                    partial[(size_t)blockIdx.x * DP * DP + (size_t)i * DP + j] = acc[rb][r] * a;
                }
            }
    }
}

// ---------------------------------------------------------------------------------------------
// 9 <= D <= 32 for large batches of short sequences: a DPP row of 16 lanes takes one whole sequence, step
// after step (four steps' loads in flight), sixteen sequences per workgroup; nothing is summed across rows,
// and every lane writes the entries it accumulated directly.
template <int DP>
__global__ __launch_bounds__(256) void tc_row_packed_kernel(const float* __restrict__ A, const float* __restrict__ filt,
                                                            const float* __restrict__ marg, long long T, int Dr,
                                                            int batch, int shared_model, double* __restrict__ counts) {
    static_assert(DP == 16 || DP == 32, "one DPP row per sequence");
    constexpr int NQ = DP / 16;
    constexpr int UNR = 4;
    const int l = threadIdx.x & 15, row = threadIdx.x >> 4;
    const long long seq_raw = (long long)blockIdx.x * 16 + row;
    const bool live = seq_raw < batch;
    const size_t seq = live ? (size_t)seq_raw : 0;
    const float* Am = A + (shared_model ? 0 : seq * Dr * Dr);
    float a[NQ * NQ * 16];
#pragma unroll
    for (int qs = 0; qs < NQ; ++qs)
#pragma unroll
        for (int qd = 0; qd < NQ; ++qd)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int i = 16 * qs + ((l - r) & 15), j = 16 * qd + l;
                a[(qs * NQ + qd) * 16 + r] = (i < Dr && j < Dr) ? Am[(size_t)i * Dr + j] : 0.0f;
            }
    float acc[NQ * NQ][16];
#pragma unroll
    for (int b = 0; b < NQ * NQ; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[b][r] = 0.0f;
    const float* fs = filt + seq * T * Dr;
    const float* ms = marg + seq * T * Dr;
    int col[NQ];
    bool have[NQ];
#pragma unroll
    for (int q = 0; q < NQ; ++q) { have[q] = 16 * q + l < Dr; col[q] = have[q] ? 16 * q + l : 0; }
    const long long kend = live ? T : 1;     // rows past the batch take no steps (all rows run the same instructions)
    for (long long kb = 1; kb < T; kb += UNR) {
        float f[UNR][NQ], gm[UNR][NQ];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const long long k = kb + u;
            const long long kc = k < T ? k : T - 1;   // past the end: a valid step, contribution masked below
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                f[u][q] = fs[(size_t)(kc - 1) * Dr + col[q]];
                gm[u][q] = ms[(size_t)kc * Dr + col[q]];
            }
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const bool valid = kb + u < kend;
            float fv[NQ];
#pragma unroll
            for (int q = 0; q < NQ; ++q) fv[q] = (valid && have[q]) ? f[u][q] : 0.0f;
            float pp[NQ][4];
            row_matvec_terms<NQ>(fv, a, pp);
#pragma unroll
            for (int qd = 0; qd < NQ; ++qd) {
                const float pred = (pp[qd][0] + pp[qd][1]) + (pp[qd][2] + pp[qd][3]);
                const float w = (pred >= PRED_MIN && have[qd]) ? gm[u][qd] * __builtin_amdgcn_rcpf(pred) : 0.0f;
#pragma unroll
                for (int qs = 0; qs < NQ; ++qs) row_outer16(fv[qs], w, acc[qs * NQ + qd]);
            }
        }
    }
    if (live) {
#pragma unroll
        for (int qs = 0; qs < NQ; ++qs)
#pragma unroll
            for (int qd = 0; qd < NQ; ++qd)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int i = 16 * qs + ((l - r) & 15), j = 16 * qd + l;
                    if (i < Dr && j < Dr)
                        counts[(seq * Dr + i) * Dr + j] = (double)(acc[qs * NQ + qd][r] * a[(qs * NQ + qd) * 16 + r]);
                }
    }
}

// counts[seq][i][j] = sum over the sequence's G partial sums, in fp64.  blockIdx.x = sequence,
// blockIdx.y = group of EPB entries; the 256 threads are (entry, slice of the partial sums), slices
// added in a fixed order.
__global__ __launch_bounds__(256) void tc_reduce_kernel(const float* __restrict__ partial, int G, int PS, int Dr,
                                                        int EPB, double* __restrict__ counts) {
    __shared__ double red[256];
    const int seq = blockIdx.x;
    const int SL = 256 / EPB;
    const int el = threadIdx.x % EPB, slice = threadIdx.x / EPB;
    const int e = blockIdx.y * EPB + el;
    double acc = 0.0;
    if (e < Dr * Dr) {
        const int i = e / Dr, j = e % Dr;
        const float* src = partial + (size_t)seq * G * PS * PS + (size_t)i * PS + j;
#pragma unroll 4
        for (int g = slice; g < G; g += SL) acc += (double)src[(size_t)g * PS * PS];
    }
    red[threadIdx.x] = acc;
    __syncthreads();
    if (slice == 0 && e < Dr * Dr) {
        double tot = 0.0;
        for (int sl = 0; sl < SL; ++sl) tot += red[sl * EPB + el];
        counts[(size_t)seq * Dr * Dr + e] = tot;
    }
}

// =============================================================================================
static int padded(int D) { return D <= 8 ? D : D <= 16 ? 16 : D <= 32 ? 32 : D <= 64 ? 64 : 128; }

static int groups_per_sequence(int D, long long T, int batch) {
    // about four workgroups per compute unit in total; one per unit where a partial sum is large (64 KiB at D > 64)
    const int total = D > 64 ? 256 : D > 16 ? 512 : 1024;
    long long G = (total + batch - 1) / batch;
    const long long most = (T - 1 + 255) / 256;               // at least 256 steps each
    if (G > most) G = most;
    if (G < 1) G = 1;
    return (int)G;
}

size_t transition_counts_ws_bytes(int D, long long T, int batch) {
    const size_t PS = (size_t)padded(D);
    return ((size_t)batch * groups_per_sequence(D, T, batch) * PS * PS * sizeof(float) + 255) / 256 * 256;
}

template <int D>
static void launch_small(const EstepArgs& a, int G, float* partial, double* direct) {
    launch("tc_accumulate", tc_small_kernel<D>, dim3((unsigned)(a.batch * G)), dim3(256), a.stream, a.A, a.filtered,
           a.marginals, a.T, G, a.shared_model, partial, direct);
}

// D <= 8, at most 1025 steps: lanes per sequence (log2) of the packed form
static int packed_group_log2(long long T) {
    const long long n = T - 1;                  // transitions
    int lg = 0;
    while ((1LL << lg) < n && lg < 6) ++lg;
    return lg;
}

template <int D>
static void launch_small_packed(const EstepArgs& a, double* counts) {
    const int lg = packed_group_log2(a.T);
    const int spw = 256 >> lg;
    launch("tc_accumulate", tc_small_packed_kernel<D>, dim3((unsigned)((a.batch + spw - 1) / spw)), dim3(256), a.stream,
           a.A, a.filtered, a.marginals, a.T, a.batch, lg, a.shared_model, counts);
}

template <int DP>
static void launch_row(const EstepArgs& a, int G, float* partial, double* direct) {
    launch("tc_accumulate", tc_row_kernel<DP>, dim3((unsigned)(a.batch * G)), dim3(256), a.stream, a.A, a.filtered,
           a.marginals, a.T, a.D, G, a.shared_model, partial, direct);
}

template <int DP>
static void launch_row_packed(const EstepArgs& a, double* counts) {
    launch("tc_accumulate", tc_row_packed_kernel<DP>, dim3((unsigned)((a.batch + 15) / 16)), dim3(256), a.stream, a.A,
           a.filtered, a.marginals, a.T, a.D, a.batch, a.shared_model, counts);
}

template <int DP>
static void launch_mfma(const EstepArgs& a, int G, float* partial, double* direct) {
    launch("tc_accumulate", tc_mfma_kernel<DP>, dim3((unsigned)(a.batch * G)), dim3(256), a.stream, a.A, a.filtered,
           a.marginals, a.T, a.D, G, a.shared_model, partial, direct);
}

int transition_counts(const EstepArgs& a, double* counts) {
    const int G = groups_per_sequence(a.D, a.T, a.batch);
    if ((long long)a.batch * G > 0x7fffffffLL) return 2;
    if (a.ws_bytes < transition_counts_ws_bytes(a.D, a.T, a.batch)) return 3;
    float* partial = static_cast<float*>(a.ws);
    const int PS = padded(a.D);
    if (PS <= 8 && a.T <= 1025) {
        switch (PS) {
            case 1: launch_small_packed<1>(a, counts); break;
            case 2: launch_small_packed<2>(a, counts); break;
            case 3: launch_small_packed<3>(a, counts); break;
            case 4: launch_small_packed<4>(a, counts); break;
            case 5: launch_small_packed<5>(a, counts); break;
            case 6: launch_small_packed<6>(a, counts); break;
            case 7: launch_small_packed<7>(a, counts); break;
            default: launch_small_packed<8>(a, counts); break;
        }
        return hipGetLastError() == hipSuccess ? 0 : 4;
    }
    if ((PS == 16 || PS == 32) && a.T <= 257 && a.batch >= 1024) {
        // large batches of short sequences: a row of lanes per sequence, counts written directly
        if (PS == 16) launch_row_packed<16>(a, counts);
        else launch_row_packed<32>(a, counts);
        return hipGetLastError() == hipSuccess ? 0 : 4;
    }
    double* direct = (G == 1) ? counts : nullptr;   // one workgroup per sequence writes the counts itself
    switch (PS) {
        case 1: launch_small<1>(a, G, partial, direct); break;
        case 2: launch_small<2>(a, G, partial, direct); break;
        case 3: launch_small<3>(a, G, partial, direct); break;
        case 4: launch_small<4>(a, G, partial, direct); break;
        case 5: launch_small<5>(a, G, partial, direct); break;
        case 6: launch_small<6>(a, G, partial, direct); break;
        case 7: launch_small<7>(a, G, partial, direct); break;
        case 8: launch_small<8>(a, G, partial, direct); break;
        case 16: launch_row<16>(a, G, partial, direct); break;
        case 32: launch_row<32>(a, G, partial, direct); break;
        case 64: launch_mfma<64>(a, G, partial, direct); break;
        case 128: launch_mfma<128>(a, G, partial, direct); break;
        default: return 2;
    }
    if (direct != nullptr) return hipGetLastError() == hipSuccess ? 0 : 4;
    const int E = a.D * a.D;
    int EPB = 1;                       // entries per workgroup: few, so that many workgroups share the partial sums
    while (EPB < E && EPB < 32) EPB <<= 1;
    launch("tc_reduce", tc_reduce_kernel, dim3((unsigned)a.batch, (unsigned)((E + EPB - 1) / EPB)), dim3(256), a.stream,
           (const float*)partial, G, PS, a.D, EPB, counts);
    return hipGetLastError() == hipSuccess ? 0 : 4;
}

int reduce_pair_partials(const float* partial, int G, int D, int batch, double* counts, hipStream_t stream) {
    const int E = D * D;
    int EPB = 1;
    while (EPB < E && EPB < 32) EPB <<= 1;
    launch("tc_reduce", tc_reduce_kernel, dim3((unsigned)batch, (unsigned)((E + EPB - 1) / EPB)), dim3(256), stream, partial,
           G, D, D, EPB, counts);
    return hipGetLastError() == hipSuccess ? 0 : 4;
}

}  // namespace hmm
