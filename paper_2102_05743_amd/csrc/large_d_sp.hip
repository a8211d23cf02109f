// Sum-product smoother for large state spaces (9 <= D <= 128, padded to 16 / 32 / 64 / 128).
//
// Chunked all-prefix-sums ("block-wise elements", Sec. V-B): time is cut into chunks of Lc steps.
//   rowmax     m_t = max_j ll_t(j)                                   (one pass over the input)
//   aggregate  chunk aggregates a_{k0-1:k0} (x) ... (x) a_{k1-2:k1-1} on the FP32 matrix cores
//   product    aggregates of groups of consecutive chunks (second scan level of long sequences; applied
//              repeatedly it also reduces a block to its single element, Sec. V-B)
//   carry      forward / backward potentials at chunk boundaries (vector x aggregate along the groups,
//              then inside all groups at once; both directions concurrently)
//   forward    a_{0:k} inside each chunk (Theorem 1), written normalised = filtering distribution
//   backward   a_{k:T+1} inside each chunk (Theorem 2)
//   combine    p(x_k) = a_{0:k} a_{k:T+1} / Z_k, and log Z from the chunk-local evidences
// Elements are never stored: each step's psi_k = A diag(e_k) is rebuilt from A and ll_k.
// States D..DP-1 of the padded model are unreachable (prior 0, self-loop only, e = 0).
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include <type_traits>

#include "ktimer.hpp"
#include "large_d.hpp"
#include "large_d_device.hpp"

namespace hmm {

constexpr float LOG2E = 1.4426950408889634f;
constexpr int ZERO_STRIP_EXP = -(1 << 28);   // power-of-two scale recorded for an all-zero strip of an aggregate
// Rows of an aggregate share a scale per strip, and strips are reconciled to the largest scale where they meet
// a carry.  That is harmless while the carry puts weight on the rows that set those scales, which it does when
// the evidence of the chunk agrees with where the chain was: the product carry x aggregate then comes out near
// the size of its factors (both are kept at a largest entry in [1/2, 1)).  A product that comes out smaller
// than this limit means that the carry sat on rows far below the scale -- rows that may have lost entries to
// it -- and the sequence is marked for ld_repair.
constexpr float HOP_LOSS_LIMIT = 0x1p-32f;

// ---------------------------------------------------------------------------------------------
// m_t = max_j ll_t(j).  A power-of-two group of lanes per row, four consecutive values per lane, so
// that a wave reads whole consecutive rows (coalesced for every D); 16-byte loads when rows are
// 16-byte aligned (D a multiple of four).  A wave takes STREAM_UNROLL such groups of rows, all loads
// issued before the first is used: a streaming pass needs that many bytes in flight per lane.
constexpr int STREAM_UNROLL = 4;

__global__ __launch_bounds__(256) void ld_rowmax_kernel(const float* __restrict__ ll, long long rows, int Dr,
                                                        float* __restrict__ rowmax, int* __restrict__ suspect,
                                                        int batch) {
    // (first kernel of a call: it also clears the per-sequence flags that the aggregate kernels may raise)
    if (suspect != nullptr && blockIdx.x == 0)
        for (int i = threadIdx.x; i < batch; i += 256) suspect[i] = 0;
    const int lpr = (Dr + 3) / 4;                  // lanes per row
    int width = 1;
    while (width < lpr) width <<= 1;               // power of two <= 32 for Dr <= 128
    const int rows_per_wave = 64 / width;
    const int lane = threadIdx.x & 63;
    const long long wave = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int sub = lane % width;
    const long long row0 = wave * (STREAM_UNROLL * rows_per_wave) + lane / width;
    float m[STREAM_UNROLL];
    if ((Dr & 3) == 0) {
        float4 x[STREAM_UNROLL];
#pragma unroll
        for (int u = 0; u < STREAM_UNROLL; ++u) {
            const long long row = row0 + u * rows_per_wave;
            x[u] = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
            if (row < rows && sub < lpr)
                x[u] = *reinterpret_cast<const float4*>(ll + row * Dr + 4 * sub);   // read again soon: keep it cached
        }
#pragma unroll
        for (int u = 0; u < STREAM_UNROLL; ++u) m[u] = fmaxf(fmaxf(x[u].x, x[u].y), fmaxf(x[u].z, x[u].w));
    } else {
#pragma unroll
        for (int u = 0; u < STREAM_UNROLL; ++u) {
            const long long row = row0 + u * rows_per_wave;
            m[u] = -INFINITY;
            if (row < rows && sub < lpr) {
                const float* p = ll + row * Dr + 4 * sub;
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (4 * sub + q < Dr) m[u] = fmaxf(m[u], p[q]);
            }
        }
    }
#pragma unroll
    for (int u = 0; u < STREAM_UNROLL; ++u) {
        for (int d = 1; d < width; d <<= 1) m[u] = fmaxf(m[u], __shfl_xor(m[u], d, 64));
        const long long row = row0 + u * rows_per_wave;
        if (row < rows && sub == 0) rowmax[row] = m[u];
    }
}

// ---------------------------------------------------------------------------------------------
// Chunk aggregates on the matrix cores.  One wave owns a TS-column strip of P^T (= TS rows of P,
// which evolve independently); WPC waves make a chunk, CPW chunks share a workgroup.
template <int D>
__global__ __launch_bounds__(256, (D <= 32) ? 2 : 1) void ld_aggregate_kernel(const float* __restrict__ A, const float* __restrict__ ll,
                                                           float* __restrict__ rowmax, int own_rowmax, long long T, int Dr,
                                                           int Lc, int cps, long long nchunks, int shared_model,
                                                           float* __restrict__ agg, float* __restrict__ aggT,
                                                           int* __restrict__ exps, int* __restrict__ suspect, int batch) {
    // own_rowmax (D <= 32 only): this is the first kernel of the call -- it forms the row maxima itself and
    // clears the per-sequence flags that the carries may raise
    if (suspect != nullptr && blockIdx.x == 0)
        for (int i = threadIdx.x; i < batch; i += 256) suspect[i] = 0;
    using C = LargeCfg<D>;
    using Acc = typename AccT<C::TS>::type;
    constexpr int EPT = C::EB * D / (C::WPC * 64);   // emission values per lane per batch
    __shared__ __align__(16) float at_all[C::CPW * C::AT_FLOATS];
    __shared__ __align__(16) float e_all[2 * C::CPW * C::EB * D];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int cl = wave / C::WPC, strip = wave % C::WPC;
    const int tic = threadIdx.x - cl * C::WPC * 64;   // lane index inside the chunk's group of waves
    const int g = lane / C::TS;
    const long long chunk = (long long)blockIdx.x * C::CPW + cl;
    const ChunkCoord cc = chunk_coord(chunk, nchunks, cps, T, Lc);
    float* at = at_all + cl * C::AT_FLOATS;

    // A^T in first-operand order: at[(mo*64 + l)*ASTR + s] = A[mfma_row(s)][TS*mo + l % TS]
    {
        const float* Am = A + (shared_model ? 0 : (size_t)cc.seq * Dr * Dr);
        for (int idx = tic; idx < C::MT * 64 * C::NS; idx += C::WPC * 64) {
            const int s = idx % C::NS, l = (idx / C::NS) % 64, mo = idx / (C::NS * 64);
            const int k = mfma_row<D>(s / C::NACC, s % C::NACC, l / C::TS);
            const int m = C::TS * mo + l % C::TS;
            float a = (k == m) ? 1.0f : 0.0f;
            if (k < Dr && m < Dr) a = Am[(size_t)k * Dr + m];
            at[(mo * 64 + l) * C::ASTR + s] = a;
        }
    }
    const float* lseq = ll + (size_t)cc.seq * T * Dr;
    float* mseq = rowmax + (size_t)cc.seq * T;
    // Whole batches of an unpadded model whose rows are 16-byte aligned: a batch is EB * D consecutive floats, four
    // per lane in one 16-byte load (EPT = 4), a step's D values in D / 4 neighbouring lanes.  Everything in this
    // kernel that is not a matrix instruction takes issue cycles from the matrix pipe of its SIMD, and forming the
    // emission factors is most of it; this path needs about a fifth of the instructions of the general one below.
    const bool vec_rows = D <= 32 && own_rowmax && Dr == D && (reinterpret_cast<uintptr_t>(ll) & 15) == 0;
    bool vec_batch = false;   // layout of the batch held in er: four consecutive values per lane, or strided
    auto load_batch = [&](int b, float (&er)[EPT]) {
        if constexpr (D <= 32) {
            static_assert(EPT == 4, "one 16-byte load per lane and batch");
            vec_batch = vec_rows && (b + 1) * C::EB <= cc.nsteps;
            if (vec_batch) {
                const int sb = (4 * tic) / D, j0 = (4 * tic) % D;
                const long long t = cc.t0 + b * C::EB + sb;
                const float4 x = *reinterpret_cast<const float4*>(lseq + (size_t)t * D + j0);
                float m = fmaxf(fmaxf(x.x, x.y), fmaxf(x.z, x.w));
#pragma unroll
                for (int d = 1; d < D / 4; d <<= 1) m = fmaxf(m, __shfl_xor(m, d, 64));
                if (j0 == 0) mseq[t] = m;
                m = (m == -INFINITY) ? 0.0f : m;
                const float off = -LOG2E * m;
                er[0] = __builtin_amdgcn_exp2f(fmaf(x.x, LOG2E, off));
                er[1] = __builtin_amdgcn_exp2f(fmaf(x.y, LOG2E, off));
                er[2] = __builtin_amdgcn_exp2f(fmaf(x.z, LOG2E, off));
                er[3] = __builtin_amdgcn_exp2f(fmaf(x.w, LOG2E, off));
                return;
            }
            if (own_rowmax) {
                // m_t = max_j ll_t(j) formed here: the D values of a step sit in D consecutive lanes of one wave
                // (aligned), so the maximum is a few cross-lane steps, and the separate pass over the
                // log-likelihoods is not needed; m_t is stored for the kernels that follow
                float x[EPT];
#pragma unroll
                for (int q = 0; q < EPT; ++q) {
                    const int idx = q * (C::WPC * 64) + tic;
                    const int sb = idx / D, j = idx - sb * D;
                    const int step = b * C::EB + sb;
                    x[q] = -INFINITY;
                    if (step < cc.nsteps && j < Dr) x[q] = lseq[(size_t)(cc.t0 + step) * Dr + j];
                }
#pragma unroll
                for (int q = 0; q < EPT; ++q) {
                    const int idx = q * (C::WPC * 64) + tic;
                    const int sb = idx / D, j = idx - sb * D;
                    const int step = b * C::EB + sb;
                    float m = x[q];
#pragma unroll
                    for (int d = 1; d < D; d <<= 1) m = fmaxf(m, __shfl_xor(m, d, 64));
                    if (j == 0 && step < cc.nsteps) mseq[cc.t0 + step] = m;
                    m = (m == -INFINITY) ? 0.0f : m;
                    er[q] = __builtin_amdgcn_exp2f(fmaf(x[q], LOG2E, -LOG2E * m));
                }
                return;
            }
        }
#pragma unroll
        for (int q = 0; q < EPT; ++q) {
            const int idx = q * (C::WPC * 64) + tic;
            const int sb = idx / D, j = idx - sb * D;
            const int step = b * C::EB + sb;
            float x = -INFINITY, m = 0.0f;
            if (step < cc.nsteps) {
                m = mseq[cc.t0 + step];
                if (j < Dr) x = lseq[(size_t)(cc.t0 + step) * Dr + j];
            }
            m = (m == -INFINITY) ? 0.0f : m;
            er[q] = __builtin_amdgcn_exp2f(fmaf(x, LOG2E, -LOG2E * m));
        }
    };
    auto store_batch = [&](int b, const float (&er)[EPT]) {
        float* eb = e_all + ((b & 1) * C::CPW + cl) * C::EB * D;
        if constexpr (D <= 32) {
            if (vec_batch) {
                *reinterpret_cast<float4*>(eb + 4 * tic) = make_float4(er[0], er[1], er[2], er[3]);
                return;
            }
        }
#pragma unroll
        for (int q = 0; q < EPT; ++q) eb[q * (C::WPC * 64) + tic] = er[q];
    };

    Acc acc[C::MT];
    const int ncol = C::TS * strip + lane % C::TS;
#pragma unroll
    for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
        for (int r = 0; r < C::NACC; ++r) acc[mt][r] = (mfma_row<D>(mt, r, g) == ncol) ? 1.0f : 0.0f;
    int exsum = 0;
    auto rescale = [&]() -> float {
        float m = 0.0f;
#pragma unroll
        for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
            for (int r = 0; r < C::NACC; ++r) m = fmaxf(m, acc[mt][r]);
        m = wave_max_nonneg(m);   // products of non-negative factors
        // the exponent goes into every entry directly: as a factor, 2^-ex overflows to infinity for a strip
        // whose largest entry has become subnormal (ex < -127), and the strip would turn into infinities and NaNs
        const int ex = __builtin_amdgcn_frexp_expf(m);
#pragma unroll
        for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
            for (int r = 0; r < C::NACC; ++r) acc[mt][r] = ldexpf(acc[mt][r], -ex);
        exsum += ex;
        return m;
    };

    const int nb = (Lc + C::EB - 1) / C::EB;
    float er[EPT];
    load_batch(0, er);
    store_batch(0, er);
    __syncthreads();
    const float* arow = at + lane * C::ASTR;
    if constexpr (D <= 32) {
        // Small tiles: the first operands of a wave fit in registers (MT * NS values).  With one result tile
        // (D = 16) the emission factor of result row m multiplies the first operand's row m instead of the
        // result, so a step is MFMAs fed by the previous step's results and nothing else touches the
        // accumulators; with two (D = 32) the results are scaled, which takes half as many multiplications.
        // The sequence's first element (no transition part) uses the identity in place of A^T.
        const int nsteps = __builtin_amdgcn_readfirstlane(cc.nsteps);   // uniform over the wave: scalar loop bounds
        const bool seq_start = __builtin_amdgcn_readfirstlane(cc.t0 == 0 ? 1 : 0) != 0;
        float areg[C::MT][C::NS];
#pragma unroll
        for (int mo = 0; mo < C::MT; ++mo)
#pragma unroll
            for (int s4 = 0; s4 < C::NS; s4 += 4) {
                const float4 a4 = *reinterpret_cast<const float4*>(arow + mo * 64 * C::ASTR + s4);
                areg[mo][s4] = a4.x; areg[mo][s4 + 1] = a4.y; areg[mo][s4 + 2] = a4.z; areg[mo][s4 + 3] = a4.w;
            }
        auto advance = [&](const float (&a)[C::MT][C::NS], const float* erow) {
            Acc nw[C::MT];
#pragma unroll
            for (int mo = 0; mo < C::MT; ++mo)
#pragma unroll
                for (int r = 0; r < C::NACC; ++r) nw[mo][r] = 0.0f;
            if constexpr (C::MT == 1) {
                // All first operands, scaled by the emission factor of their row, before the first matrix instruction:
                // formed one by one between them, each would be followed by the wait states a matrix instruction needs
                // after a write of its operand.
                float ae[C::NS];
                const float em = erow[lane % C::TS];
#pragma unroll
                for (int s = 0; s < C::NS; ++s) ae[s] = a[0][s] * em;
                __builtin_amdgcn_sched_barrier(0);   // (the scheduler would interleave them again)
#pragma unroll
                for (int s = 0; s < C::NS; ++s) nw[0] = mfma_step<C::TS>(ae[s], acc[0][s], nw[0]);
                acc[0] = nw[0];
            } else {
                // Two result tiles: scaling the results (NACC registers per tile) takes half the multiplications that
                // scaling the first operands would (NS per tile).  The tiles' instructions alternate, so that none
                // follows the one whose result it adds to.
#pragma unroll
                for (int s = 0; s < C::NS; ++s)
#pragma unroll
                    for (int mo = 0; mo < C::MT; ++mo)
                        nw[mo] = mfma_step<C::TS>(a[mo][s], acc[s / C::NACC][s % C::NACC], nw[mo]);
#pragma unroll
                for (int mo = 0; mo < C::MT; ++mo) {
                    const float4 e4 = *reinterpret_cast<const float4*>(erow + mfma_row<D>(mo, 0, g));
                    acc[mo][0] = nw[mo][0] * e4.x;
                    acc[mo][1] = nw[mo][1] * e4.y;
                    acc[mo][2] = nw[mo][2] * e4.z;
                    acc[mo][3] = nw[mo][3] * e4.w;
                }
            }
        };
        for (int b = 0; b < nb; ++b) {
            if (b + 1 < nb) load_batch(b + 1, er);
            const float* eb = e_all + ((b & 1) * C::CPW + cl) * C::EB * D;
            const int s_end = min(C::EB, nsteps - b * C::EB);
            int sb = 0;
            if (b == 0 && seq_start && s_end > 0) {
                float aid[C::MT][C::NS];
#pragma unroll
                for (int mo = 0; mo < C::MT; ++mo)
#pragma unroll
                    for (int s = 0; s < C::NS; ++s)
                        aid[mo][s] = (mfma_row<D>(s / C::NACC, s % C::NACC, g) == C::TS * mo + lane % C::TS) ? 1.0f : 0.0f;
                advance(aid, eb);
                sb = 1;
            }
#pragma unroll 1
            for (; sb < s_end; ++sb) {
                advance(areg, eb + sb * D);
                if (((b * C::EB + sb) % C::NORM_EVERY) == C::NORM_EVERY - 1) rescale();
            }
            if (b + 1 < nb) store_batch(b + 1, er);
            __syncthreads();
        }
    } else {
        // Loop bounds are scalars and the sequence's first element (no transition part: the strip is only scaled) is
        // taken out of the loop, so that the loop body has no branch around the matrix instructions -- the compiler
        // keeps their results in accumulation registers, and at a join with the path that skips them it copied the
        // whole strip into those registers and back, every step.
        const int nsteps = __builtin_amdgcn_readfirstlane(cc.nsteps);
        const bool seq_start = __builtin_amdgcn_readfirstlane(cc.t0 == 0 ? 1 : 0) != 0;
        auto scale_rows = [&](const float* erow) {   // rows of P^T scaled by a step's emission factors
#pragma unroll
            for (int mo = 0; mo < C::MT; ++mo)
#pragma unroll
                for (int q = 0; q < C::NACC / 4; ++q) {
                    const float4 e4 = *reinterpret_cast<const float4*>(erow + mfma_row<D>(mo, 4 * q, g));
                    acc[mo][4 * q + 0] *= e4.x;
                    acc[mo][4 * q + 1] *= e4.y;
                    acc[mo][4 * q + 2] *= e4.z;
                    acc[mo][4 * q + 3] *= e4.w;
                }
        };
        for (int b = 0; b < nb; ++b) {
            if (b + 1 < nb) load_batch(b + 1, er);
            const float* eb = e_all + ((b & 1) * C::CPW + cl) * C::EB * D;
            const int s_end = min(C::EB, nsteps - b * C::EB);
            int sb = 0;
            if (b == 0 && seq_start && s_end > 0) {
                scale_rows(eb);
                sb = 1;
            }
#pragma unroll 1
            for (; sb < s_end; ++sb) {
                // (the first operands are read from LDS again in every step: kept in registers across steps they would
                // not fit beside the two strips)
                asm volatile("" ::: "memory");
                Acc nw[C::MT];
#pragma unroll
                for (int mo = 0; mo < C::MT; ++mo) {
#pragma unroll
                    for (int r = 0; r < C::NACC; ++r) nw[mo][r] = 0.0f;
#pragma unroll
                    for (int s4 = 0; s4 < C::NS; s4 += 4) {
                        const float4 a4 = *reinterpret_cast<const float4*>(arow + mo * 64 * C::ASTR + s4);
                        nw[mo] = mfma_step<C::TS>(a4.x, acc[(s4 + 0) / C::NACC][(s4 + 0) % C::NACC], nw[mo]);
                        nw[mo] = mfma_step<C::TS>(a4.y, acc[(s4 + 1) / C::NACC][(s4 + 1) % C::NACC], nw[mo]);
                        nw[mo] = mfma_step<C::TS>(a4.z, acc[(s4 + 2) / C::NACC][(s4 + 2) % C::NACC], nw[mo]);
                        nw[mo] = mfma_step<C::TS>(a4.w, acc[(s4 + 3) / C::NACC][(s4 + 3) % C::NACC], nw[mo]);
                    }
                }
#pragma unroll
                for (int mo = 0; mo < C::MT; ++mo) acc[mo] = nw[mo];
                scale_rows(eb + sb * D);
                if (((b * C::EB + sb) % C::NORM_EVERY) == C::NORM_EVERY - 1) rescale();
            }
            if (b + 1 < nb) store_batch(b + 1, er);
            __syncthreads();
        }
    }
    if (cc.nsteps > 0) {
        // a strip of zeros (start states the first observation excludes) has no scale of its own: give
        // it the lowest one, so that it cannot set the common scale when strips are reconciled
        if (rescale() == 0.0f) exsum = ZERO_STRIP_EXP;
        float* dst = agg + (size_t)chunk * D * D;     // P[n][k]
        float* dstT = aggT + (size_t)chunk * D * D;   // P^T[k][n]
#pragma unroll
        for (int mt = 0; mt < C::MT; ++mt) {
#pragma unroll
            for (int q = 0; q < C::NACC / 4; ++q)
                *reinterpret_cast<float4*>(dst + (size_t)ncol * D + mfma_row<D>(mt, 4 * q, g)) =
                    make_float4(acc[mt][4 * q], acc[mt][4 * q + 1], acc[mt][4 * q + 2], acc[mt][4 * q + 3]);
#pragma unroll
            for (int r = 0; r < C::NACC; ++r) dstT[(size_t)mfma_row<D>(mt, r, g) * D + ncol] = acc[mt][r];
        }
        if (lane == 0) exps[chunk * C::WPC + strip] = exsum;
    }
}

// ---------------------------------------------------------------------------------------------
// Second level of the scan: the aggregate of a group of consecutive chunks, X = P_c0 P_c0+1 ... ,
// so that the carries of a long sequence need about 2 sqrt(chunks) sequential hops instead of one
// per chunk.  Same scheme as the chunk aggregates, X^T <- P_c^T X^T with X^T fed back from the
// accumulators, except that the first operand changes with every hop: P_c is brought into LDS in
// first-operand order (from its transposed copy, whose rows hold the reduction index contiguously),
// its strips reconciled to one scale on the way.  Output in the same format as the chunk aggregates.
template <int D>
__global__ __launch_bounds__(256) void ld_product_kernel(const float* __restrict__ aggT, const int* __restrict__ exps,
                                                         int cps, int g, int G, long long ngroups,
                                                         float* __restrict__ gagg, float* __restrict__ gaggT,
                                                         int* __restrict__ gexps) {
    using C = LargeCfg<D>;
    using Acc = typename AccT<C::TS>::type;
    __shared__ __align__(16) float at_all[C::CPW * C::AT_FLOATS];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int cl = wave / C::WPC, strip = wave % C::WPC;
    const int tic = threadIdx.x - cl * C::WPC * 64;   // lane index inside the group's waves
    const int gl = lane / C::TS;
    const long long gidx = (long long)blockIdx.x * C::CPW + cl;
    const bool live = gidx < ngroups;
    const int seq = live ? (int)(gidx / G) : 0, grp = live ? (int)(gidx % G) : 0;
    const int c0 = grp * g;
    const int nh = live ? min(cps, c0 + g) - c0 : 0;
    float* at = at_all + cl * C::AT_FLOATS;
    Acc acc[C::MT];
    const int ncol = C::TS * strip + lane % C::TS;
#pragma unroll
    for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
        for (int r = 0; r < C::NACC; ++r) acc[mt][r] = (mfma_row<D>(mt, r, gl) == ncol) ? 1.0f : 0.0f;
    int exsum = 0;
    auto rescale = [&]() -> float {
        float m = 0.0f;
#pragma unroll
        for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
            for (int r = 0; r < C::NACC; ++r) m = fmaxf(m, acc[mt][r]);
        m = wave_max_nonneg(m);   // products of non-negative factors
        // the exponent goes into every entry directly: as a factor, 2^-ex overflows to infinity for a strip
        // whose largest entry has become subnormal (ex < -127), and the strip would turn into infinities and NaNs
        const int ex = __builtin_amdgcn_frexp_expf(m);
#pragma unroll
        for (int mt = 0; mt < C::MT; ++mt)
#pragma unroll
            for (int r = 0; r < C::NACC; ++r) acc[mt][r] = ldexpf(acc[mt][r], -ex);
        exsum += ex;
        return m;
    };
    const float* arow = at + lane * C::ASTR;
    for (int hop = 0; hop < g; ++hop) {     // every wave runs g hops (barriers inside); idle hops do nothing else
        const bool active = hop < nh;
        __syncthreads();                    // the previous hop's reads of the operand are done
        if (active) {
            const float* MT_ = aggT + ((size_t)seq * cps + c0 + hop) * D * D;   // P^T[m][k]
            const int* ex = exps + ((size_t)seq * cps + c0 + hop) * C::WPC;
            int exv[C::WPC];
            int exmax = ex[0];
#pragma unroll
            for (int w = 0; w < C::WPC; ++w) { exv[w] = ex[w]; exmax = max(exmax, exv[w]); }
            if (exmax != ZERO_STRIP_EXP) exsum += exmax;   // common to all strips: keeps the product's absolute scale
            // at[(mo*64 + l)*ASTR + s] = P(k, m) 2^(ex[strip of k] - exmax), k = mfma_row(s), m = TS*mo + l % TS,
            // four consecutive s (= four consecutive k) per access
            for (int idx = tic; idx < C::MT * 64 * (C::NS / 4); idx += C::WPC * 64) {
                const int s4 = idx % (C::NS / 4), l = (idx / (C::NS / 4)) % 64, mo = idx / ((C::NS / 4) * 64);
                const int s = 4 * s4;
                const int k = mfma_row<D>(s / C::NACC, s % C::NACC, l / C::TS);
                const int m = C::TS * mo + l % C::TS;
                float4 x = *reinterpret_cast<const float4*>(MT_ + (size_t)m * D + k);
                int ek = exv[0];
#pragma unroll
                for (int w = 1; w < C::WPC; ++w) ek = (k / C::TS == w) ? exv[w] : ek;
                const float sc = ldexpf(1.0f, max(ek - exmax, -126));
                x.x *= sc; x.y *= sc; x.z *= sc; x.w *= sc;
                *reinterpret_cast<float4*>(at + (mo * 64 + l) * C::ASTR + s) = x;
            }
        }
        __syncthreads();
        if (active) {
            Acc nw[C::MT];
#pragma unroll
            for (int mo = 0; mo < C::MT; ++mo) {
#pragma unroll
                for (int r = 0; r < C::NACC; ++r) nw[mo][r] = 0.0f;
#pragma unroll
                for (int s4 = 0; s4 < C::NS; s4 += 4) {
                    const float4 a4 = *reinterpret_cast<const float4*>(arow + mo * 64 * C::ASTR + s4);
                    nw[mo] = mfma_step<C::TS>(a4.x, acc[(s4 + 0) / C::NACC][(s4 + 0) % C::NACC], nw[mo]);
                    nw[mo] = mfma_step<C::TS>(a4.y, acc[(s4 + 1) / C::NACC][(s4 + 1) % C::NACC], nw[mo]);
                    nw[mo] = mfma_step<C::TS>(a4.z, acc[(s4 + 2) / C::NACC][(s4 + 2) % C::NACC], nw[mo]);
                    nw[mo] = mfma_step<C::TS>(a4.w, acc[(s4 + 3) / C::NACC][(s4 + 3) % C::NACC], nw[mo]);
                }
            }
#pragma unroll
            for (int mo = 0; mo < C::MT; ++mo) acc[mo] = nw[mo];
            rescale();
        }
    }
    if (nh > 0) {
        if (rescale() == 0.0f) exsum = ZERO_STRIP_EXP;
        float* dst = gagg + (size_t)gidx * D * D;     // X[n][k]
        float* dstT = gaggT + (size_t)gidx * D * D;   // X^T[k][n]
#pragma unroll
        for (int mt = 0; mt < C::MT; ++mt) {
#pragma unroll
            for (int q = 0; q < C::NACC / 4; ++q)
                *reinterpret_cast<float4*>(dst + (size_t)ncol * D + mfma_row<D>(mt, 4 * q, gl)) =
                    make_float4(acc[mt][4 * q], acc[mt][4 * q + 1], acc[mt][4 * q + 2], acc[mt][4 * q + 3]);
#pragma unroll
            for (int r = 0; r < C::NACC; ++r) dstT[(size_t)mfma_row<D>(mt, r, gl) * D + ncol] = acc[mt][r];
        }
        if (lane == 0) gexps[gidx * C::WPC + strip] = exsum;
    }
}

// ---------------------------------------------------------------------------------------------
// Carries between the chunks of a sequence.  blockIdx = 2*seq + dir; dir 0 walks the chunks left
// to right with v <- v P_c (matrix = agg), dir 1 right to left with v <- P_c v (matrix = aggT,
// read row by row so that both directions stream memory the same way).  Strips of an aggregate
// carry their own power-of-two scale, reconciled here.
template <int D>
__global__ __launch_bounds__(256) void ld_carry_kernel(const float* __restrict__ prior, int Dr, int cps,
                                                       int shared_model, const float* __restrict__ agg,
                                                       const float* __restrict__ aggT, const int* __restrict__ exps,
                                                       float* __restrict__ fin, float* __restrict__ bout,
                                                       int seglen, int nseg, const float* __restrict__ start_f,
                                                       const float* __restrict__ start_b, int* __restrict__ suspect) {
    // The chunks of a sequence may be cut into nseg segments of seglen chunks that are walked
    // independently (blockIdx = 2*(seq*nseg + seg) + dir), each from its own start vector: the
    // forward potential before the segment (start_f) or the backward potential at its last step
    // (start_b).  Without start vectors (nseg = 1) the walk starts from the prior / the ones vector.
    using C = LargeCfg<D>;
    constexpr int CG = D / 4;                                   // groups of four columns
    constexpr int RP = (256 / CG < D) ? 256 / CG : D;           // lane groups splitting the summation
    constexpr int RPT = D / RP;                                 // summation terms per lane
    __shared__ __align__(16) float vec[D];                      // current vector (pre-scaled for dir 0)
    __shared__ __align__(16) float partial[RP * D];
    __shared__ float wmx[4];
    const int unit = blockIdx.x >> 1, dir = blockIdx.x & 1;
    const int seq = unit / nseg, seg = unit % nseg;
    const int c_begin = seg * seglen, c_end = min(cps, c_begin + seglen);
    const int nhops = c_end - c_begin;
    const int tid = threadIdx.x;
    const bool worker = tid < CG * RP;
    const int cg = tid % CG, rp = tid / CG;
    const int j = tid;                                          // component owned by lanes tid < D
    const float* mats = (dir == 0 ? agg : aggT) + (size_t)seq * cps * D * D;
    const int* ex = exps + (size_t)seq * cps * C::WPC;
    float* out = (dir == 0 ? fin : bout) + (size_t)seq * cps * D;
    float v = 0.0f;
    if (j < D) {
        if (dir == 0) {
            if (start_f != nullptr) v = start_f[(size_t)unit * D + j];
            else v = (j < Dr) ? prior[(shared_model ? 0 : (size_t)seq * Dr) + j] : 0.0f;
        } else {
            if (start_b != nullptr) v = start_b[(size_t)unit * D + j];
            else v = (j < Dr) ? 1.0f : 0.0f;
        }
    }
    float4 pm[RPT];
    int exn[C::WPC];
    auto load_mat = [&](int c) {   // aggregate c and its strip exponents, prefetched one hop ahead
        const float* M = mats + (size_t)c * D * D;
        if (worker) {
#pragma unroll
            for (int r = 0; r < RPT; ++r) pm[r] = *reinterpret_cast<const float4*>(M + (size_t)(rp * RPT + r) * D + 4 * cg);
        }
#pragma unroll
        for (int s = 0; s < C::WPC; ++s) exn[s] = ex[c * C::WPC + s];
    };
    auto strip_exp = [&](const int (&e)[C::WPC], int col) {
        const int st = col / C::TS;
        int r = e[0];
#pragma unroll
        for (int s = 1; s < C::WPC; ++s) r = (st == s) ? e[s] : r;
        return r;
    };
    int c = dir == 0 ? c_begin : c_end - 1;
    load_mat(c);
    for (int it = 0; it < nhops; ++it) {
        int exc[C::WPC];
        int exmax = exn[0];
#pragma unroll
        for (int s = 0; s < C::WPC; ++s) { exc[s] = exn[s]; exmax = max(exmax, exn[s]); }
        if (j < D) {
            out[(size_t)c * D + j] = v;
            // dir 0 sums over rows of P, whose scale depends on the row's strip: fold it into the vector
            vec[j] = (dir == 0) ? ldexpf(v, strip_exp(exc, j) - exmax) : v;
        }
        lds_barrier();
        float4 acc = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        if (worker) {
#pragma unroll
            for (int r = 0; r < RPT; ++r) {
                const float x = vec[rp * RPT + r];
                acc.x = fmaf(x, pm[r].x, acc.x);
                acc.y = fmaf(x, pm[r].y, acc.y);
                acc.z = fmaf(x, pm[r].z, acc.z);
                acc.w = fmaf(x, pm[r].w, acc.w);
            }
        }
        const int cn = dir == 0 ? c + 1 : c - 1;
        if (it + 1 < nhops) load_mat(cn);   // the next aggregate streams in while this one is reduced
        if (worker) *reinterpret_cast<float4*>(partial + rp * D + 4 * cg) = acc;
        lds_barrier();
        float g = 0.0f;
        if (j < D) {
#pragma unroll 8
            for (int p = 0; p < RP; ++p) g += partial[p * D + j];
            // dir 1 produces rows of P: scale by the row's strip
            if (dir == 1) g = ldexpf(g, strip_exp(exc, j) - exmax);
        }
        // keep the vector in range with an exact power of two (its scale is irrelevant downstream)
        float m = wave_max(j < D ? g : 0.0f);
        if constexpr (D > 64) {
            if ((tid & 63) == 0) wmx[tid >> 6] = m;
            lds_barrier();
            m = fmaxf(wmx[0], wmx[1]);
        }
        if (m < HOP_LOSS_LIMIT && tid == 0) suspect[seq] = 1;   // (see HOP_LOSS_LIMIT)
        v = ldexpf(g, -__builtin_amdgcn_frexp_expf(m));
        c = cn;
    }
}

// The same carries for D <= 32 by a single wave per (sequence, direction): lane = (column j, part h
// of the summation range), parts combined with quad permutes, the vector passed through LDS with
// wave-level ordering only.  A hop costs a few hundred cycles instead of three workgroup barriers,
// which is what bounds a long sequence (its chunks are visited one after the other); aggregates are
// prefetched PF hops ahead because a hop is much shorter than a memory round trip.
template <int D>
__global__ __launch_bounds__(64) void ld_carry_wave_kernel(const float* __restrict__ prior, int Dr, int cps,
                                                           int shared_model, const float* __restrict__ agg,
                                                           const float* __restrict__ aggT,
                                                           const int* __restrict__ exps, float* __restrict__ fin,
                                                           float* __restrict__ bout, int seglen, int nseg,
                                                           const float* __restrict__ start_f,
                                                           const float* __restrict__ start_b, int* __restrict__ suspect) {
    using C = LargeCfg<D>;
    static_assert(D <= 32, "one wave covers the columns");
    constexpr int PARTS = 64 / D;       // 2 or 4 lanes per column
    constexpr int RPT = D / PARTS;      // summation terms per lane
    constexpr int PF = 8;               // prefetch distance in hops
    __shared__ __align__(16) float vec[D];
    const int unit = blockIdx.x >> 1, dir = blockIdx.x & 1;   // segments as in ld_carry_kernel
    const int seq = unit / nseg, seg = unit % nseg;
    const int c_begin = seg * seglen, c_end = min(cps, c_begin + seglen);
    const int nhops = c_end - c_begin;
    const int lane = threadIdx.x;
    const int h = lane % PARTS, j = lane / PARTS;
    // the lane's terms M(h*RPT + r, j) are contiguous in the transposed copy: 16-byte loads
    const float* mats = (dir == 0 ? aggT : agg) + (size_t)seq * cps * D * D;
    const int* ex = exps + (size_t)seq * cps * C::WPC;
    float* out = (dir == 0 ? fin : bout) + (size_t)seq * cps * D;
    float v;
    if (dir == 0) {
        if (start_f != nullptr) v = start_f[(size_t)unit * D + j];
        else v = (j < Dr) ? prior[(shared_model ? 0 : (size_t)seq * Dr) + j] : 0.0f;
    } else {
        if (start_b != nullptr) v = start_b[(size_t)unit * D + j];
        else v = (j < Dr) ? 1.0f : 0.0f;
    }
    settle_loaded(v);
    float pm[PF][RPT];
    int exn[PF][C::WPC];
    bool lost = false;
    auto chunk_of = [&](int it) { return dir == 0 ? c_begin + it : c_end - 1 - it; };
    // Loads are unconditional (the hop index is clamped) and the exponents come through vector loads:
    // the compiler can then count outstanding loads exactly and wait only for the slot it needs,
    // where a conditional or scalar load would make every hop wait for the newest prefetch.
    const int lane_zero = __builtin_amdgcn_mbcnt_lo(0u, 0u);   // 0, but not known to be uniform
    auto load_mat = [&](int it, float (&m)[RPT], int (&e)[C::WPC]) {
        const int c = chunk_of(it < nhops ? it : nhops - 1);
        const float* M = mats + (size_t)c * D * D + (size_t)j * D + h * RPT;
#pragma unroll
        for (int r4 = 0; r4 < RPT; r4 += 4) {
            const float4 x = *reinterpret_cast<const float4*>(M + r4);
            m[r4] = x.x; m[r4 + 1] = x.y; m[r4 + 2] = x.z; m[r4 + 3] = x.w;
        }
#pragma unroll
        for (int s = 0; s < C::WPC; ++s) e[s] = ex[c * C::WPC + s + lane_zero];
    };
    auto hop = [&](int it, const float (&m)[RPT], const int (&e)[C::WPC]) {
        const int c = chunk_of(it);
        int exmax = e[0];
#pragma unroll
        for (int s = 1; s < C::WPC; ++s) exmax = max(exmax, e[s]);
        int exj = e[0];    // exponent of the strip that row j of P belongs to
#pragma unroll
        for (int s = 1; s < C::WPC; ++s) exj = (j / C::TS == s) ? e[s] : exj;
        if (h == 0) {
            out[(size_t)c * D + j] = v;
            // dir 0 sums over rows of P, whose scale depends on the row's strip: fold it into the vector
            vec[j] = (dir == 0) ? ldexpf(v, exj - exmax) : v;
        }
        wave_lds_sync();
        float a0 = 0.0f, a1 = 0.0f, a2 = 0.0f, a3 = 0.0f;   // independent chains
#pragma unroll
        for (int r4 = 0; r4 < RPT; r4 += 4) {
            const float4 x = *reinterpret_cast<const float4*>(vec + h * RPT + r4);
            a0 = fmaf(x.x, m[r4], a0);
            a1 = fmaf(x.y, m[r4 + 1], a1);
            a2 = fmaf(x.z, m[r4 + 2], a2);
            a3 = fmaf(x.w, m[r4 + 3], a3);
        }
        wave_lds_sync();
        float acc = (a0 + a1) + (a2 + a3);
        acc += quad_xor1(acc);
        if constexpr (PARTS == 4) acc += quad_xor2(acc);
        // dir 1 produces rows of P: scale by the row's strip
        const float g = (dir == 1) ? ldexpf(acc, exj - exmax) : acc;
        // keep the vector in range with an exact power of two (its scale is irrelevant downstream)
        const float mx = wave_max(g);
        lost = lost || (mx < HOP_LOSS_LIMIT);   // (see HOP_LOSS_LIMIT)
        v = ldexpf(g, -__builtin_amdgcn_frexp_expf(mx));
    };
#pragma unroll
    for (int p = 0; p < PF; ++p) load_mat(p, pm[p], exn[p]);
    const int nfull = nhops / PF * PF;
    for (int it0 = 0; it0 < nfull; it0 += PF) {
#pragma unroll
        for (int p = 0; p < PF; ++p) {
            hop(it0 + p, pm[p], exn[p]);
            load_mat(it0 + p + PF, pm[p], exn[p]);
        }
    }
#pragma unroll
    for (int p = 0; p < PF; ++p)
        if (nfull + p < nhops) hop(nfull + p, pm[p], exn[p]);   // slot p holds hop nfull + p
    if (lost && lane == 0) suspect[seq] = 1;
}

// ---------------------------------------------------------------------------------------------
// Vector recursions inside the chunks.  Lane = (column or row c inside the wave, part h of the
// summation range), with h in the lowest lane bits so that parts are combined with quad
// permutes; A stays in registers.  A chunk of D <= 32 is one wave and needs no workgroup barrier.
template <int D>
HMM_DEV void apply_sync() {
    if constexpr (LargeCfg<D>::VWPC > 1) lds_barrier();
    else wave_lds_sync();
}

template <int D>
HMM_DEV float combine_parts(float acc) {
    using C = LargeCfg<D>;
    acc += quad_xor1(acc);
    if constexpr (C::PARTS == 4) acc += quad_xor2(acc);
    return acc;
}

// Emission factors of a chunk, produced EB steps at a time by all lanes of the chunk and kept in
// double-buffered LDS, so that no global load and no exponential sits on the per-step critical path.
// Steps are numbered in processing order: rev = false walks t0, t0+1, ...; rev = true walks from
// the loop's last step downwards.
template <int D>
struct EmissionBatches {
    using C = LargeCfg<D>;
    static constexpr int EB = 16;
    static constexpr int LPCH = C::VWPC * 64;            // lanes per chunk
    static constexpr int EPT = EB * D / LPCH;            // values per lane per batch
    const float* lseq;
    const float* mseq;
    float* e_lds;    // [2][EB*D] of this chunk
    float* m_lds;    // [2][EB]
    long long t0;
    int nsteps, nloop, Dr, tic;
    bool rev;
    float er[EPT];
    float mr;

    HMM_DEV int step_of(int pos) const { return rev ? nloop - 1 - pos : pos; }
    HMM_DEV void load(int b) {
#pragma unroll
        for (int q = 0; q < EPT; ++q) {
            const int idx = q * LPCH + tic;
            const int sb = idx / D, jj = idx - sb * D;
            const int st = step_of(b * EB + sb);
            float x = -INFINITY, m = 0.0f;
            if (st >= 0 && st < nsteps) {
                m = mseq[t0 + st];
                if (jj < Dr) x = lseq[(size_t)(t0 + st) * Dr + jj];
            }
            m = (m == -INFINITY) ? 0.0f : m;
            er[q] = __builtin_amdgcn_exp2f(fmaf(x, LOG2E, -LOG2E * m));
        }
        mr = 0.0f;
        if (tic < EB) {
            const int st = step_of(b * EB + tic);
            if (st >= 0 && st < nsteps) mr = mseq[t0 + st];
        }
    }
    HMM_DEV void store(int b) {
        float* eb = e_lds + (b & 1) * EB * D;
#pragma unroll
        for (int q = 0; q < EPT; ++q) eb[q * LPCH + tic] = er[q];
        if (tic < EB) m_lds[(b & 1) * EB + tic] = mr;
    }
};

// LDS of the apply kernel, per workgroup
template <int D>
struct ApplyLds {
    using C = LargeCfg<D>;
    __align__(16) float vbuf[2 * C::VCPW * D];
    float wsum[2 * C::VCPW * C::VWPC];
    __align__(16) float e[C::VCPW * 2 * 16 * D];
    float m[C::VCPW * 2 * 16];
};

// Forward potentials (Theorem 1): f_k = (f_{k-1} A) o e_k, written normalised (= p(x_k | y_{1:k})),
// plus the chunk's log evidence log p(y_chunk | y_before).
template <int D>
HMM_DEV void forward_chunk(const float* __restrict__ prior, const float* __restrict__ A, const float* __restrict__ ll,
                           const float* __restrict__ rowmax, long long T, int Dr, int Lc, int cps, long long nchunks,
                           int shared_model, const float* __restrict__ fin, float* __restrict__ F,
                           double* __restrict__ part, long long chunk0, ApplyLds<D>& L) {
    using C = LargeCfg<D>;
    using EBt = EmissionBatches<D>;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int cl = wave / C::VWPC, wv = wave % C::VWPC;
    const int h = lane % C::PARTS;
    const int j = C::CPWV * wv + lane / C::PARTS;
    const long long chunk = chunk0 + cl;
    const ChunkCoord cc = chunk_coord(chunk, nchunks, cps, T, Lc);
    const float* Am = A + (shared_model ? 0 : (size_t)cc.seq * Dr * Dr);
    float areg[C::RPP];
#pragma unroll
    for (int r = 0; r < C::RPP; ++r) {
        const int i = h * C::RPP + r;
        areg[r] = (i == j) ? 1.0f : 0.0f;
        if (i < Dr && j < Dr) areg[r] = Am[(size_t)i * Dr + j];
    }
    float* Fseq = F + (size_t)cc.seq * T * Dr;
    const bool first_chunk = (chunk % cps) == 0;
    const int nloop = (C::VWPC > 1) ? Lc : cc.nsteps;   // with workgroup barriers every wave runs the full count
    EBt eb;
    eb.lseq = ll + (size_t)cc.seq * T * Dr;
    eb.mseq = rowmax + (size_t)cc.seq * T;
    eb.e_lds = L.e + cl * 2 * EBt::EB * D;
    eb.m_lds = L.m + cl * 2 * EBt::EB;
    eb.t0 = cc.t0; eb.nsteps = cc.nsteps; eb.nloop = nloop; eb.Dr = Dr; eb.rev = false;
    eb.tic = threadIdx.x - cl * EBt::LPCH;
    float* fbuf = L.vbuf;
    float* wsum = L.wsum;
    // carry into the chunk; every chunk but the sequence's first starts from a vector summing to one
    float f0 = 0.0f;
    if (cc.nsteps > 0) {
        if (first_chunk) f0 = (j < Dr) ? prior[(shared_model ? 0 : (size_t)cc.seq * Dr) + j] : 0.0f;
        else f0 = fin[(size_t)chunk * D + j];
    }
    if (h == 0) fbuf[cl * D + j] = f0;
    {
        const float s = wave_sum(h == 0 ? f0 : 0.0f);
        if (lane == 0) wsum[cl * C::VWPC + wv] = s;
    }
    const int nb = (nloop + EBt::EB - 1) / EBt::EB;
    if (nb > 0) { eb.load(0); eb.store(0); }
    apply_sync<D>();
    float inv = 1.0f;
    if (!first_chunk) {
        float tot = 0.0f;
#pragma unroll
        for (int w = 0; w < C::VWPC; ++w) tot += wsum[cl * C::VWPC + w];
        inv = __builtin_amdgcn_rcpf(tot);
    }
    double dacc = 0.0;
    int cur = 0;
    for (int b = 0; b < nb; ++b) {
        if (b + 1 < nb) eb.load(b + 1);
        const float* ebuf = eb.e_lds + (b & 1) * EBt::EB * D;
        const float* mbuf = eb.m_lds + (b & 1) * EBt::EB;
        const int send = min(EBt::EB, nloop - b * EBt::EB);
        for (int sb = 0; sb < send; ++sb) {
            const int s = b * EBt::EB + sb;
            const bool active = s < cc.nsteps;
            const float* fc = fbuf + (cur * C::VCPW + cl) * D;
            float* fn = fbuf + ((cur ^ 1) * C::VCPW + cl) * D;
            float* wn = wsum + ((cur ^ 1) * C::VCPW + cl) * C::VWPC;
            float gval = 0.0f;
            if (active) {
                const float e = ebuf[sb * D + j];
                if (cc.t0 + s == 0) {
                    gval = fc[j] * e;   // psi_1 = prior o e_1: no transition
                } else {
                    float acc = 0.0f;
#pragma unroll
                    for (int r4 = 0; r4 < C::RPP; r4 += 4) {
                        const float4 f4 = *reinterpret_cast<const float4*>(fc + h * C::RPP + r4);
                        acc = fmaf(f4.x, areg[r4], acc);
                        acc = fmaf(f4.y, areg[r4 + 1], acc);
                        acc = fmaf(f4.z, areg[r4 + 2], acc);
                        acc = fmaf(f4.w, areg[r4 + 3], acc);
                    }
                    acc = combine_parts<D>(acc);
                    gval = acc * inv * e;
                }
                if (h == 0) fn[j] = gval;
                const float sw = wave_sum(h == 0 ? gval : 0.0f);
                if (lane == 0) wn[wv] = sw;
            }
            if (sb == send - 1 && b + 1 < nb) eb.store(b + 1);
            apply_sync<D>();
            if (active) {
                float tot = 0.0f;
#pragma unroll
                for (int w = 0; w < C::VWPC; ++w) tot += wn[w];
                inv = __builtin_amdgcn_rcpf(tot);
                if (h == 0 && j < Dr) Fseq[(size_t)(cc.t0 + s) * Dr + j] = gval * inv;
                if (lane == 0 && wv == 0) dacc += (double)mbuf[sb] + (double)__logf(tot);
            }
            cur ^= 1;
        }
    }
    if (cc.nsteps > 0 && lane == 0 && wv == 0) part[chunk] = dacc;
}

// Backward potentials (Theorem 2): b_{k-1} = A (e_k o b_k), stored with an arbitrary positive
// scale per step (the marginal is normalised afterwards).
template <int D>
HMM_DEV void backward_chunk(const float* __restrict__ A, const float* __restrict__ ll,
                            const float* __restrict__ rowmax, long long T, int Dr, int Lc, int cps, long long nchunks,
                            int shared_model, const float* __restrict__ bout, float* __restrict__ Bv,
                            long long chunk0, ApplyLds<D>& L) {
    using C = LargeCfg<D>;
    using EBt = EmissionBatches<D>;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int cl = wave / C::VWPC, wv = wave % C::VWPC;
    const int h = lane % C::PARTS;
    const int i = C::CPWV * wv + lane / C::PARTS;
    const long long chunk = chunk0 + cl;
    const ChunkCoord cc = chunk_coord(chunk, nchunks, cps, T, Lc);
    const float* Am = A + (shared_model ? 0 : (size_t)cc.seq * Dr * Dr);
    float areg[C::RPP];
#pragma unroll
    for (int r = 0; r < C::RPP; ++r) {
        const int jj = h * C::RPP + r;
        areg[r] = (i == jj) ? 1.0f : 0.0f;
        if (i < Dr && jj < Dr) areg[r] = Am[(size_t)i * Dr + jj];
    }
    float* Bseq = Bv + (size_t)cc.seq * T * Dr;
    const int nloop = (C::VWPC > 1) ? Lc : cc.nsteps;
    EBt eb;
    eb.lseq = ll + (size_t)cc.seq * T * Dr;
    eb.mseq = rowmax + (size_t)cc.seq * T;
    eb.e_lds = L.e + cl * 2 * EBt::EB * D;
    eb.m_lds = L.m + cl * 2 * EBt::EB;
    eb.t0 = cc.t0; eb.nsteps = cc.nsteps; eb.nloop = nloop; eb.Dr = Dr; eb.rev = true;
    eb.tic = threadIdx.x - cl * EBt::LPCH;
    float* ubuf = L.vbuf;
    float* wsum = L.wsum;
    // b at the chunk's last step; without carries (sequences of one chunk) that is the all-ones vector
    float b = 0.0f;
    if (cc.nsteps > 0) b = bout != nullptr ? bout[(size_t)chunk * D + i] : (i < Dr ? 1.0f : 0.0f);
    float inv = 1.0f;
    int cur = 0;
    const int nb = (nloop + EBt::EB - 1) / EBt::EB;
    if (nb > 0) { eb.load(0); eb.store(0); }
    apply_sync<D>();
    for (int bb = 0; bb < nb; ++bb) {
        if (bb + 1 < nb) eb.load(bb + 1);
        const float* ebuf = eb.e_lds + (bb & 1) * EBt::EB * D;
        const int send = min(EBt::EB, nloop - bb * EBt::EB);
        for (int sb = 0; sb < send; ++sb) {
            const int s = nloop - 1 - (bb * EBt::EB + sb);
            const bool active = s < cc.nsteps;
            float* un = ubuf + ((cur ^ 1) * C::VCPW + cl) * D;
            float* wn = wsum + ((cur ^ 1) * C::VCPW + cl) * C::VWPC;
            if (active) {
                const float bs = b * inv;   // scaled by the previous step's normaliser: any positive scale will do
                if (h == 0 && i < Dr) Bseq[(size_t)(cc.t0 + s) * Dr + i] = bs;
                if (h == 0) un[i] = ebuf[sb * D + i] * bs;
                const float sw = wave_sum(h == 0 ? bs : 0.0f);
                if (lane == 0) wn[wv] = sw;
            }
            if (sb == send - 1 && bb + 1 < nb) eb.store(bb + 1);
            apply_sync<D>();
            if (active && s > 0) {
                float tot = 0.0f;
#pragma unroll
                for (int w = 0; w < C::VWPC; ++w) tot += wn[w];
                inv = __builtin_amdgcn_rcpf(tot);
                float acc = 0.0f;
#pragma unroll
                for (int r4 = 0; r4 < C::RPP; r4 += 4) {
                    const float4 u4 = *reinterpret_cast<const float4*>(un + h * C::RPP + r4);
                    acc = fmaf(u4.x, areg[r4], acc);
                    acc = fmaf(u4.y, areg[r4 + 1], acc);
                    acc = fmaf(u4.z, areg[r4 + 2], acc);
                    acc = fmaf(u4.w, areg[r4 + 3], acc);
                }
                b = combine_parts<D>(acc);
            }
            cur ^= 1;
        }
    }
}

// One launch for both directions: the first half of the grid runs the forward recursion of its
// chunks, the second half the backward recursion of the same chunks, concurrently.
template <int D>
__global__ __launch_bounds__(256) void ld_apply_kernel(const float* __restrict__ prior, const float* __restrict__ A,
                                                       const float* __restrict__ ll, const float* __restrict__ rowmax,
                                                       long long T, int Dr, int Lc, int cps, long long nchunks,
                                                       int shared_model, const float* __restrict__ fin,
                                                       const float* __restrict__ bout, float* __restrict__ F,
                                                       float* __restrict__ Bv, double* __restrict__ part, int half) {
    using C = LargeCfg<D>;
    __shared__ ApplyLds<D> L;
    if ((int)blockIdx.x < half)
        forward_chunk<D>(prior, A, ll, rowmax, T, Dr, Lc, cps, nchunks, shared_model, fin, F, part,
                         (long long)blockIdx.x * C::VCPW, L);
    else
        backward_chunk<D>(A, ll, rowmax, T, Dr, Lc, cps, nchunks, shared_model, bout, Bv,
                          (long long)(blockIdx.x - half) * C::VCPW, L);
}

// ---------------------------------------------------------------------------------------------
// The same vector recursions for D <= 32 with one chunk per DPP row of 16 lanes and no LDS at all.
// Lane l of a row holds components l (and 16 + l for D = 32) of the vector; the product with A is
// systolic: the term f(i) A(i,j) with i = (l - r) mod 16 reaches lane l as the row's vector rotated
// by r lanes (a DPP modifier), multiplied by a register that is constant per (r, block pair).
// Sixteen chunks advance per workgroup, independently; the normaliser of a step is computed beside
// the next step's products and applied one step late, so a step's dependent chain is the products
// and two multiplications.  FUSED (enough chunks to fill the machine with one row each): a row first
// runs the forward recursion of its chunk, which leaves the filtering distributions in F, then the
// backward recursion, which reads them back (every lane the values it stored itself) and writes the
// marginals f_k b_k / Z_k, so that backward potentials never reach memory.  Otherwise the two recursions
// of a chunk run concurrently in different workgroups (first half of the grid forward, second half
// backward, writing the backward potentials) and a separate pass forms the marginals.
template <int D, bool BACKWARD, bool FUSED, bool FULL>
HMM_DEV void apply_row_pass(const float* __restrict__ Am, const float* __restrict__ lseq,
                            const float* __restrict__ mseq, const ChunkCoord& cc, int Dr, int Lc, bool first_chunk,
                            const float (&start)[D / 16], float* fseq, float* __restrict__ gseq, double* part_out) {
    constexpr int NQ = D / 16;
    constexpr int PFD = 8;                                  // steps of log-likelihoods in flight
    const int l = threadIdx.x & 15;
    // forward: a[(qs, qd, r)] = A(16 qs + (l - r) mod 16, 16 qd + l); backward: A(16 qd + l, 16 qs + (l - r) mod 16)
    float a[NQ * NQ * 16];
#pragma unroll
    for (int qs = 0; qs < NQ; ++qs)
#pragma unroll
        for (int qd = 0; qd < NQ; ++qd)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int src = 16 * qs + ((l - r) & 15), dst = 16 * qd + l;
                const int i = BACKWARD ? dst : src, j = BACKWARD ? src : dst;
                float v = (i == j) ? 1.0f : 0.0f;
                if (i < Dr && j < Dr) v = Am[(size_t)i * Dr + j];
                a[(qs * NQ + qd) * 16 + r] = v;
            }
    // step order: forward s = 0, 1, ...; backward s = nsteps-1, nsteps-2, ...  (pos = position in that order)
    auto step_at = [&](int pos) { return BACKWARD ? cc.nsteps - 1 - pos : pos; };
    float xq[PFD][NQ], mq[PFD], fq[PFD][NQ];
    // Running pointers instead of index arithmetic per step.  Fetches are unconditional (the compiler
    // can then count outstanding loads exactly); past the chunk's end they repeat its last position.
    const int s_first = cc.nsteps > 0 ? step_at(0) : 0;
    const long long stride = BACKWARD ? -(long long)Dr : (long long)Dr;
    const float* lp = lseq + (size_t)(cc.t0 + s_first) * Dr;
    const float* mp = mseq + (cc.t0 + s_first);
    const float* fp = fseq + (size_t)(cc.t0 + s_first) * Dr;
    float* op = (BACKWARD ? gseq : fseq) + (size_t)(cc.t0 + s_first) * Dr;
    int colq[NQ];
#pragma unroll
    for (int q = 0; q < NQ; ++q) colq[q] = (16 * q + l) < Dr ? 16 * q + l : 0;
    int fetched = 0;
    auto fetch = [&](float (&x)[NQ], float (&f)[NQ], float& m) {
        m = *mp;
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            x[q] = lp[colq[q]];
            if constexpr (BACKWARD && FUSED) f[q] = fp[colq[q]];
        }
        ++fetched;
        // FULL: the caller fetches exactly the chunk's positions; the pointers end one position outside it, unused
        if (FULL || fetched < cc.nsteps) {
            lp += stride;
            fp += stride;
            mp += BACKWARD ? -1 : 1;
        }
    };
    float h[NQ];
#pragma unroll
    for (int q = 0; q < NQ; ++q) h[q] = start[q];
#pragma unroll
    for (int p = 0; p < PFD; ++p) fetch(xq[p], fq[p], mq[p]);
    float hs = h[0];
#pragma unroll
    for (int q = 1; q < NQ; ++q) hs += h[q];
    // forward: every chunk but the sequence's first starts from a vector summing to one; backward: any scale
    float inv = (!BACKWARD && first_chunk) ? 1.0f : __builtin_amdgcn_rcpf(row_allsum(hs));
    // chunk evidence: sum of the steps' emission maxima, and the product of the steps' normalisers kept as
    // mantissa and binary exponent (one logarithm per chunk instead of one per step)
    float msum = 0.0f, cmant = 1.0f;
    int cexp = 0;
    // FULL (decided for the whole wavefront): every row's chunk has exactly Lc steps, Lc is a multiple of 2 PFD and the
    // model is not padded -- no step is inactive, no lane idle, the sequence's first step can only be a chunk's
    // position 0, and the last PFD steps fetch nothing.
    // A group consumes the PFD positions fetched into (xc, fc, mc) and fetches, PFD positions ahead, into (xn, fn, mn):
    // the same arrays (refilled in place), or a second set -- then nothing waits for a load younger than the one it
    // needs, and a position's data has a whole group's time to arrive.
    auto group = [&](int p0, auto do_fetch, float (&xc)[PFD][NQ], float (&fc)[PFD][NQ], float (&mc)[PFD],
                     float (&xn)[PFD][NQ], float (&fn)[PFD][NQ], float (&mn)[PFD]) {
        const bool at_t0 = FULL && first_chunk && p0 == (BACKWARD ? Lc - PFD : 0);
#pragma unroll
        for (int p = 0; p < PFD; ++p) {
            const int pos = p0 + p;
            const bool active = FULL || pos < cc.nsteps;
            const long long t = cc.t0 + step_at(pos);
            // is this the sequence's first step?
            const bool is_t0 = FULL ? (at_t0 && p == (BACKWARD ? PFD - 1 : 0)) : (t == 0);
            const float mm = (mc[p] == -INFINITY) ? 0.0f : mc[p];
            float e[NQ], fk[NQ];
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                const bool real = FULL || (16 * q + l) < Dr;
                const float x = real ? xc[p][q] : -INFINITY;
                e[q] = __builtin_amdgcn_exp2f(fmaf(x, LOG2E, -LOG2E * mm));
                fk[q] = (BACKWARD && FUSED && real) ? fc[p][q] : 0.0f;
            }
            if constexpr (decltype(do_fetch)::value) fetch(xn[p], fn[p], mn[p]);
            if constexpr (!BACKWARD) {
                float g[NQ];
                float acc[NQ][4];
                row_matvec_terms<NQ>(h, a, acc);
#pragma unroll
                for (int q = 0; q < NQ; ++q) {
                    const float moved = ((acc[q][0] + acc[q][1]) + (acc[q][2] + acc[q][3])) * inv;
                    // psi_1 = prior o e_1: no transition at the first step (FULL: only a group's first step can be it)
                    if constexpr (FULL) g[q] = ((p == 0 && is_t0) ? h[q] : moved) * e[q];
                    else g[q] = (is_t0 ? h[q] : moved) * e[q];
                }
                float gs = g[0];
#pragma unroll
                for (int q = 1; q < NQ; ++q) gs += g[q];
                const float c = row_allsum(gs);            // p(y_t | y_{<t}) e^{-m_t} (times the prior's mass at t = 0)
                const float ic = __builtin_amdgcn_rcpf(c);
                if (active) {
#pragma unroll
                    for (int q = 0; q < NQ; ++q) {
                        if (FULL || 16 * q + l < Dr) op[16 * q + l] = g[q] * ic;   // p(x_t | y_{1:t})
                        h[q] = g[q];
                    }
                    op += stride;
                    inv = ic;
                    msum += mm;
                    const float cp = cmant * c;
                    cmant = __builtin_amdgcn_frexp_mantf(cp);
                    cexp += __builtin_amdgcn_frexp_expf(cp);
                }
            } else {
                float bs[NQ], u[NQ], gam[NQ];
#pragma unroll
                for (int q = 0; q < NQ; ++q) {
                    bs[q] = h[q] * inv;        // any positive scale will do: the marginal is normalised below
                    u[q] = e[q] * bs[q];
                    gam[q] = fk[q] * bs[q];
                }
                float ss = bs[0], gs = gam[0];
#pragma unroll
                for (int q = 1; q < NQ; ++q) {
                    ss += bs[q];
                    gs += gam[q];
                }
                const float ic = __builtin_amdgcn_rcpf(row_allsum(ss));
                const float ig = __builtin_amdgcn_rcpf(row_allsum(gs));   // 1 / Z_k in this scaling
                float acc[NQ][4];
                row_matvec_terms<NQ>(u, a, acc);
                if (active) {
#pragma unroll
                    for (int q = 0; q < NQ; ++q) {
                        if (FULL || 16 * q + l < Dr) op[16 * q + l] = FUSED ? gam[q] * ig : bs[q];   // p(x_t | y_{1:T}), or b_t
                        // (FULL: after the sequence's first step, the last one this direction visits, h is not read again)
                        if (FULL || !is_t0) h[q] = (acc[q][0] + acc[q][1]) + (acc[q][2] + acc[q][3]);
                    }
                    op += stride;
                    inv = ic;
                }
            }
        }
    };
    if constexpr (FULL) {
        float xr[PFD][NQ], mr[PFD], fr[PFD][NQ];   // Lc is a multiple of 2 PFD: groups alternate between the two sets
        for (int p0 = 0; p0 < Lc - 2 * PFD; p0 += 2 * PFD) {
            group(p0, std::true_type{}, xq, fq, mq, xr, fr, mr);
            group(p0 + PFD, std::true_type{}, xr, fr, mr, xq, fq, mq);
        }
        group(Lc - 2 * PFD, std::true_type{}, xq, fq, mq, xr, fr, mr);
        group(Lc - PFD, std::false_type{}, xr, fr, mr, xq, fq, mq);
    } else {
        for (int p0 = 0; p0 < Lc; p0 += PFD) group(p0, std::true_type{}, xq, fq, mq, xq, fq, mq);
    }
    if constexpr (!BACKWARD) {
        if (cc.nsteps > 0 && l == 0)
            *part_out = (double)msum + (double)logf(cmant) + 0.6931471805599453 * (double)cexp;
    }
}

// out: the marginals (FUSED) or the backward potentials; half: workgroups per direction (not FUSED)
template <int D, bool FUSED>
__global__ __launch_bounds__(256) void ld_apply_row_kernel(const float* __restrict__ prior, const float* __restrict__ A,
                                                           const float* __restrict__ ll,
                                                           const float* __restrict__ rowmax, long long T, int Dr,
                                                           int Lc, int cps, long long nchunks, int shared_model,
                                                           const float* __restrict__ fin,
                                                           const float* __restrict__ bout, float* F,
                                                           float* __restrict__ out, double* __restrict__ part,
                                                           int half) {
    static_assert(D == 16 || D == 32, "one DPP row per chunk");
    constexpr int NQ = D / 16;
    const int l = threadIdx.x & 15;
    const bool backward = !FUSED && (int)blockIdx.x >= half;
    const long long chunk = (long long)(backward ? blockIdx.x - half : blockIdx.x) * 16 + (threadIdx.x >> 4);
    const ChunkCoord cc = chunk_coord(chunk, nchunks, cps, T, Lc);
    const float* Am = A + (shared_model ? 0 : (size_t)cc.seq * Dr * Dr);
    const float* lseq = ll + (size_t)cc.seq * T * Dr;
    const float* mseq = rowmax + (size_t)cc.seq * T;
    float* fseq = F + (size_t)cc.seq * T * Dr;
    float* gseq = out + (size_t)cc.seq * T * Dr;
    const bool first_chunk = cc.nsteps > 0 && (chunk % cps) == 0;
    float hf[NQ], hb[NQ];
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        const int j = 16 * q + l;
        hf[q] = hb[q] = 0.0f;
        if (cc.nsteps > 0) {
            if (first_chunk) hf[q] = (j < Dr) ? prior[(shared_model ? 0 : (size_t)cc.seq * Dr) + j] : 0.0f;
            else hf[q] = fin[(size_t)chunk * D + j];
            hb[q] = bout != nullptr ? bout[(size_t)chunk * D + j] : (j < Dr ? 1.0f : 0.0f);   // one chunk per sequence: all ones
        }
    }
    // the usual case, decided per wavefront: whole chunks of an unpadded model (see apply_row_pass)
    const bool full = Dr == D && Lc % 16 == 0 && __builtin_amdgcn_ballot_w64(cc.nsteps != Lc) == 0;
    if (full) {
        if (!backward) apply_row_pass<D, false, FUSED, true>(Am, lseq, mseq, cc, Dr, Lc, first_chunk, hf, fseq, gseq, part + chunk);
        if (FUSED || backward) apply_row_pass<D, true, FUSED, true>(Am, lseq, mseq, cc, Dr, Lc, first_chunk, hb, fseq, gseq, nullptr);
    } else {
        if (!backward) apply_row_pass<D, false, FUSED, false>(Am, lseq, mseq, cc, Dr, Lc, first_chunk, hf, fseq, gseq, part + chunk);
        if (FUSED || backward) apply_row_pass<D, true, FUSED, false>(Am, lseq, mseq, cc, Dr, Lc, first_chunk, hb, fseq, gseq, nullptr);
    }
}

// ---------------------------------------------------------------------------------------------
// p(x_k) = f_k b_k / Z_k.  Four consecutive states per lane; a row is reduced inside a wave; a wave
// takes STREAM_UNROLL groups of rows with all loads issued first, 16-byte accesses when D is a multiple of four.
__global__ __launch_bounds__(256) void ld_combine_kernel(const float* __restrict__ F, const float* __restrict__ Bv,
                                                         long long rows, int Dr, float* __restrict__ marg) {
    const int lpr = (Dr + 3) / 4;                  // lanes per row
    int width = 1;
    while (width < lpr) width <<= 1;               // power of two <= 32 for Dr <= 128
    const int rows_per_wave = 64 / width;
    const int lane = threadIdx.x & 63;
    const long long wave = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int sub = lane % width;
    const long long row0 = wave * (STREAM_UNROLL * rows_per_wave) + lane / width;
    float g[STREAM_UNROLL][4];
    bool live[STREAM_UNROLL];
    if ((Dr & 3) == 0) {
        float4 f[STREAM_UNROLL], b[STREAM_UNROLL];
#pragma unroll
        for (int u = 0; u < STREAM_UNROLL; ++u) {
            const long long row = row0 + u * rows_per_wave;
            live[u] = row < rows && sub < lpr;
            f[u] = b[u] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
            if (live[u]) {
                const v4f fv = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(F + row * Dr + 4 * sub));
                const v4f bv = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(Bv + row * Dr + 4 * sub));
                f[u] = make_float4(fv.x, fv.y, fv.z, fv.w);
                b[u] = make_float4(bv.x, bv.y, bv.z, bv.w);
            }
        }
#pragma unroll
        for (int u = 0; u < STREAM_UNROLL; ++u) {
            g[u][0] = f[u].x * b[u].x; g[u][1] = f[u].y * b[u].y; g[u][2] = f[u].z * b[u].z; g[u][3] = f[u].w * b[u].w;
        }
    } else {
#pragma unroll
        for (int u = 0; u < STREAM_UNROLL; ++u) {
            const long long row = row0 + u * rows_per_wave;
            live[u] = row < rows && sub < lpr;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int j = 4 * sub + q;
                g[u][q] = (live[u] && j < Dr) ? F[row * Dr + j] * Bv[row * Dr + j] : 0.0f;
            }
        }
    }
#pragma unroll
    for (int u = 0; u < STREAM_UNROLL; ++u) {
        const long long row = row0 + u * rows_per_wave;
        float s = g[u][0] + g[u][1] + g[u][2] + g[u][3];
        for (int d = 1; d < width; d <<= 1) s += __shfl_xor(s, d, 64);
        if (live[u]) {
            const float inv = 1.0f / s;
            if ((Dr & 3) == 0) {
                const v4f out = {g[u][0] * inv, g[u][1] * inv, g[u][2] * inv, g[u][3] * inv};
                __builtin_nontemporal_store(out, reinterpret_cast<v4f*>(marg + row * Dr + 4 * sub));
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int j = 4 * sub + q;
                    if (j < Dr) marg[row * Dr + j] = g[u][q] * inv;
                }
            }
        }
    }
}

// out[seq] = ordered sum of the chunk evidences of one sequence
__global__ __launch_bounds__(256) void ld_finalize_kernel(const double* __restrict__ part, int cps,
                                                          double* __restrict__ out) {
    __shared__ double sh[256];
    const int seq = blockIdx.x;
    double acc = 0.0;
    for (int c = threadIdx.x; c < cps; c += 256) acc += part[(size_t)seq * cps + c];
    sh[threadIdx.x] = acc;
    __syncthreads();
    for (int d = 128; d >= 1; d >>= 1) {
        if ((int)threadIdx.x < d) sh[threadIdx.x] += sh[threadIdx.x + d];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[seq] = sh[0];
}

// ---------------------------------------------------------------------------------------------
// Block-wise element (Sec. V-B) of a whole block from its single remaining aggregate: strips brought
// to one power-of-two scale, largest entry in [0.5, 1), padding dropped;
// log_scale = sum of the steps' emission maxima + ln 2 * (binary exponent).  One workgroup per sequence.
template <int D>
__global__ __launch_bounds__(256) void ld_element_finish_kernel(const float* __restrict__ agg, const int* __restrict__ exps,
                                                                const float* __restrict__ rowmax, long long T, int Dr,
                                                                float* __restrict__ element, double* __restrict__ log_scale) {
    using C = LargeCfg<D>;
    __shared__ double dred[4];
    __shared__ float fred[4];
    const int seq = blockIdx.x, tid = threadIdx.x;
    const float* M = agg + (size_t)seq * D * D;
    const int* ex = exps + (size_t)seq * C::WPC;
    double ms = 0.0;
    {
        // eight independent loads in flight per lane: one workgroup adds up the whole block's maxima
        const float* rm = rowmax + (size_t)seq * T;
        constexpr int U = 8;
        long long t = tid;
        for (; t + (U - 1) * 256 < T; t += U * 256) {
            float v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) v[u] = rm[t + u * 256];
#pragma unroll
            for (int u = 0; u < U; ++u) ms += (v[u] == -INFINITY) ? 0.0 : (double)v[u];
        }
        for (; t < T; t += 256) {
            const float m = rm[t];
            ms += (m == -INFINITY) ? 0.0 : (double)m;
        }
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) ms += __shfl_down(ms, d, 64);
    int exmax = ex[0];
#pragma unroll
    for (int w = 1; w < C::WPC; ++w) exmax = max(exmax, ex[w]);
    float lm = 0.0f;
    for (int idx = tid; idx < Dr * Dr; idx += 256) {
        const int i = idx / Dr, j = idx - i * Dr;
        lm = fmaxf(lm, ldexpf(M[(size_t)i * D + j], max(ex[i / C::TS] - exmax, -200)));
    }
    lm = wave_max(lm);
    if ((tid & 63) == 0) { dred[tid >> 6] = ms; fred[tid >> 6] = lm; }
    __syncthreads();
    const float m = fmaxf(fmaxf(fred[0], fred[1]), fmaxf(fred[2], fred[3]));
    const int ex2 = __builtin_amdgcn_frexp_expf(m);
    for (int idx = tid; idx < Dr * Dr; idx += 256) {
        const int i = idx / Dr, j = idx - i * Dr;
        element[(size_t)seq * Dr * Dr + idx] = ldexpf(M[(size_t)i * D + j], max(ex[i / C::TS] - exmax - ex2, -200));
    }
    if (tid == 0) {
        const double total = dred[0] + dred[1] + dred[2] + dred[3];
        log_scale[seq] = (m > 0.0f) ? total + 0.6931471805599453 * ((double)exmax + (double)ex2) : -INFINITY;
    }
}

// ---------------------------------------------------------------------------------------------
// Repair pass.  The aggregates above carry one scale per strip of rows; where the rows of an aggregate have
// drifted apart by more than that can hold (models with zero transitions under evidence that contradicts the
// states the chain can still be in), a carry that sits on the small rows loses them.  Such sequences were
// marked on the way (suspect[seq], raised by the carries; or a log-likelihood that is not a number) and are
// redone here by the classical recursion itself, step by step in single precision with a rescaling at every
// step (Alg. 1; forward potentials scaled to sum one, backward ones to maximum one): slow, one workgroup
// per sequence walking its T steps twice, but it is by definition what the scans have to agree with.
// Sequences that were not marked leave at once.  The forward potentials wait in `marg` itself until the
// backward sweep overwrites them with the marginals.
constexpr int REPAIR_THREADS = 128;   // one thread per state (D <= 128)
constexpr int REPAIR_ASTR = 129;      // row stride of A in LDS: conflict-free by rows and by columns
constexpr int REPAIR_BIAS = 50;       // potentials are held near 2^50 (two of them multiplied and summed over 128 states stay finite)

HMM_DEV float repair_block_sum(float v, float* red) {   // all REPAIR_THREADS threads; two barriers
    const float w = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = w;
    __syncthreads();
    return red[0] + red[1];
}
HMM_DEV float repair_block_max(float v, float* red) {
    const float w = wave_max(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = w;
    __syncthreads();
    return fmaxf(red[0], red[1]);
}

__global__ __launch_bounds__(REPAIR_THREADS) void ld_repair_kernel(
    const double* __restrict__ part, int cps, const int* __restrict__ suspect, const float* __restrict__ prior, const float* __restrict__ A, const float* __restrict__ ll,
    const float* __restrict__ rowmax, long long T, int Dr, int shared_model, float* __restrict__ marg,
    float* __restrict__ filt, double* __restrict__ loglik_out) {
    __shared__ float Al[128 * REPAIR_ASTR];
    __shared__ float vec[128];
    __shared__ float red[2];
    const int seq = blockIdx.x;
    const int j = threadIdx.x;
    // log Z of the scans first: the ordered sum of the chunk evidences (what ld_finalize does where this
    // kernel is not launched)
    __shared__ double ev[REPAIR_THREADS];
    {
        // eight loads in flight per thread (a long sequence has thousands of chunks and one workgroup to add them up)
        const double* pseq = part + (size_t)seq * cps;
        constexpr int U = 8;
        double acc = 0.0;
        int c = j;
        for (; c + (U - 1) * REPAIR_THREADS < cps; c += U * REPAIR_THREADS) {
            double v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) v[u] = pseq[c + u * REPAIR_THREADS];
#pragma unroll
            for (int u = 0; u < U; ++u) acc += v[u];
        }
        for (; c < cps; c += REPAIR_THREADS) acc += pseq[c];
        ev[j] = acc;
        __syncthreads();
        for (int d = REPAIR_THREADS / 2; d >= 1; d >>= 1) {
            if (j < d) ev[j] += ev[j + d];
            __syncthreads();
        }
    }
    const double logz = ev[0];
    // marked on the way, or a result that is not a number
    const bool redo = suspect[seq] != 0 || !(logz == logz);
    if (j == 0 && !redo) loglik_out[seq] = logz;
    if (!__syncthreads_or(redo ? 1 : 0)) return;

    const bool live = j < Dr;
    const float* Am = A + (shared_model ? 0 : (size_t)seq * Dr * Dr);
    for (int idx = j; idx < Dr * Dr; idx += REPAIR_THREADS) Al[(idx / Dr) * REPAIR_ASTR + idx % Dr] = Am[idx];
    const float* lseq = ll + (size_t)seq * T * Dr;
    const float* mseq = rowmax + (size_t)seq * T;
    float* F = filt != nullptr ? filt + (size_t)seq * T * Dr : nullptr;
    float* G_ = marg + (size_t)seq * T * Dr;
    auto factor = [&](long long t) {   // e_t(j), largest one at 1 (as in the aggregate kernels)
        float m = mseq[t];
        m = (m == -INFINITY) ? 0.0f : m;
        return live ? __builtin_amdgcn_exp2f(fmaf(lseq[(size_t)t * Dr + j], LOG2E, -LOG2E * m)) : 0.0f;
    };
    // Both potentials are held far above one (sums / maxima near 2^REPAIR_BIAS, by exact powers of two): an entry
    // 2^-126 below the largest is then still a normal number, and the state that later evidence vindicates
    // is usually such an entry.
    double L = 0.0;
    float S_prev = 1.0f;   // sum of the stored forward vector of the previous step (the prior sums to one)
    __syncthreads();
    // forward sweep: u_t = f_t * 2^k_t into marg (and f_t itself into filt if asked for)
    for (long long t = 0; t < T; ++t) {
        float pred = 0.0f;
        if (live) {
            if (t == 0) {
                pred = prior[(shared_model ? 0 : (size_t)seq * Dr) + j];
            } else {
                for (int i = 0; i < Dr; ++i) pred = fmaf(vec[i], Al[i * REPAIR_ASTR + j], pred);
            }
        }
        const float g = pred * factor(t);
        const float s = repair_block_sum(g, red);   // (its barriers also order the reads of vec above before the write below)
        const int k = REPAIR_BIAS - __builtin_amdgcn_frexp_expf(s);
        const float u = ldexpf(g, k);
        if (live) {
            vec[j] = u;
            G_[(size_t)t * Dr + j] = u;
            if (filt != nullptr) F[(size_t)t * Dr + j] = g / s;
        }
        if (j == 0) {
            float m = mseq[t];
            m = (m == -INFINITY) ? 0.0f : m;
            L += (double)m + log((double)s) - log((double)S_prev);
        }
        S_prev = ldexpf(s, k);   // = the sum of u: scaling by a power of two commutes with the rounding of the sum
        __syncthreads();
    }
    if (j == 0) loglik_out[seq] = L;
    // backward sweep: marginals over the stored u_t
    float b = live ? 1.0f : 0.0f;
    for (long long t = T - 1; t >= 0; --t) {
        const float uj = live ? G_[(size_t)t * Dr + j] : 0.0f;
        const float gam = uj * b;
        const float z = repair_block_sum(gam, red);
        if (live) G_[(size_t)t * Dr + j] = gam / z;
        if (t == 0) break;
        if (live) vec[j] = factor(t) * b;
        __syncthreads();
        float r = 0.0f;
        if (live)
            for (int q = 0; q < Dr; ++q) r = fmaf(Al[j * REPAIR_ASTR + q], vec[q], r);
        const float mx = repair_block_max(r, red);
        b = ldexpf(r, REPAIR_BIAS - __builtin_amdgcn_frexp_expf(mx));
    }
}

// =============================================================================================
// Host side
// =============================================================================================
static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

LargePlan large_plan(int Dr, long long T, int batch) {
    LargePlan p;
    p.DP = Dr <= 16 ? 16 : Dr <= 32 ? 32 : Dr <= 64 ? 64 : 128;
    // chunks: enough to occupy every matrix core (smaller states need more, shorter chunks).  The
    // carry between the chunks of one sequence is sequential, and so are the steps inside a chunk:
    // with a hop costing about as much as one (D >= 64) or half a (D <= 32) step of the in-chunk
    // recursions, their sum is smallest near sqrt(T) resp. sqrt(2T) chunks per sequence, which bounds
    // the count from above.
    const long long target = p.DP >= 128 ? 256 : p.DP >= 64 ? 512 : p.DP >= 32 ? 2048 : 8192;
    long long cps = (target + batch - 1) / batch;
    if (cps < 1) cps = 1;
    long long most = (long long)sqrt((p.DP >= 64 ? 1.0 : 2.0) * (double)T);
    if (most < 256) most = 256;
    if (most > 8192) most = 8192;
    if (cps > most) cps = most;
    long long Lc = (T + cps - 1) / cps;
    Lc = (Lc + 15) / 16 * 16;
    if (Lc < 32) Lc = 32;
    p.Lc = (int)(Lc > 0x3fffffff ? 0x3fffffff : Lc);
    p.cps = (int)((T + p.Lc - 1) / p.Lc);
    p.nchunks = (long long)p.cps * batch;
    return p;
}

// Plan of the smoother: enough chunks for two workgroups per compute unit at D >= 64 (the in-chunk
// recursions are latency-bound, so shorter chunks pay as long as the carries stay cheap), chunks of at
// most 256 (D >= 64) or 128 steps, so that a long sequence gets more chunks rather than longer ones, and above 96 chunks per sequence a second scan level: groups
// of g chunks whose aggregates are formed by ld_product.  With a product hop costing about 8.4
// (D >= 64) or 5.4 (D <= 32) vector hops, g + chunks/g vector hops and g product hops are fewest in
// total near g = sqrt(0.106 chunks) resp. sqrt(0.156 chunks).  Up to 32 states and from 1024 chunks per sequence
// a third level: groups of g2 groups (ld_product applied to the group aggregates), carries over those, then inside
// them over the groups, then inside the groups over the chunks -- 2 g product hops, 2 g + chunks / g^2 vector hops and
// two more launches, fewest near g = cbrt(chunks / 6): a third to a half of the two-level plan's sequential time.
struct SmoothPlan { int DP, Lc, cps; long long nchunks; int g, G, g2, G2; bool two_level, three_level, fused_apply; };

static SmoothPlan smooth_plan(int Dr, long long T, int batch) {
    SmoothPlan p;
    p.DP = Dr <= 16 ? 16 : Dr <= 32 ? 32 : Dr <= 64 ? 64 : 128;
    const long long target = p.DP >= 128 ? 512 : p.DP >= 64 ? 1024 : p.DP >= 32 ? 2048 : 8192;
    long long cps = (target + batch - 1) / batch;
    if (cps < 1) cps = 1;
    const long long lmax = p.DP >= 64 ? 256 : 128;
    long long Lc = (T + cps - 1) / cps;
    Lc = (Lc + 15) / 16 * 16;
    if (Lc < 32) Lc = 32;
    if (Lc > lmax) Lc = lmax;
    p.Lc = (int)Lc;
    p.cps = (int)((T + p.Lc - 1) / p.Lc);
    p.nchunks = (long long)p.cps * batch;
    // D <= 32: forward, backward and marginals in one pass per chunk once that alone gives every SIMD a wave
    // (four chunks per wave); below that the two directions run side by side
    p.fused_apply = p.DP <= 32 && p.nchunks >= 4096;
    p.two_level = p.cps > 96;
    p.three_level = p.DP <= 32 && p.cps >= 1024;
    p.g2 = 1;
    p.G2 = 1;
    if (p.three_level) {
        int g = (int)(cbrt((double)p.cps / 6.0) + 0.5);
        p.g = g < 2 ? 2 : g;
        p.G = (p.cps + p.g - 1) / p.g;
        p.g2 = p.g;
        p.G2 = (p.G + p.g2 - 1) / p.g2;
    } else if (p.two_level) {
        int g = (int)sqrt((p.DP >= 64 ? 0.106 : 0.156) * (double)p.cps);
        p.g = g < 2 ? 2 : g;
        p.G = (p.cps + p.g - 1) / p.g;
    } else {
        p.g = p.cps;
        p.G = 1;
    }
    return p;
}

struct LargeSmoothWs { size_t rowmax, agg, aggT, exps, fin, bout, gagg, gaggT, gexps, gfin, gbout, sagg, saggT, sexps, sfin, sbout, F, Bv, part, suspect, total; };

static LargeSmoothWs large_smooth_ws(int Dr, long long T, int batch, bool own_F) {
    const SmoothPlan p = smooth_plan(Dr, T, batch);
    const size_t D = p.DP, nc = (size_t)p.nchunks, rows = (size_t)T * batch;
    const size_t ng = p.two_level ? (size_t)p.G * batch : 0;
    const size_t ns = p.three_level ? (size_t)p.G2 * batch : 0;   // groups of groups
    LargeSmoothWs w;
    size_t o = 0;
    w.rowmax = o; o = align_up(o + rows * sizeof(float), 256);
    w.agg = o;    o = align_up(o + nc * D * D * sizeof(float), 256);
    w.aggT = o;   o = align_up(o + nc * D * D * sizeof(float), 256);
    w.exps = o;   o = align_up(o + nc * 8 * sizeof(int), 256);
    w.fin = o;    o = align_up(o + nc * D * sizeof(float), 256);
    w.bout = o;   o = align_up(o + nc * D * sizeof(float), 256);
    w.gagg = o;   o = align_up(o + ng * D * D * sizeof(float), 256);
    w.gaggT = o;  o = align_up(o + ng * D * D * sizeof(float), 256);
    w.gexps = o;  o = align_up(o + ng * 8 * sizeof(int), 256);
    w.gfin = o;   o = align_up(o + ng * D * sizeof(float), 256);
    w.gbout = o;  o = align_up(o + ng * D * sizeof(float), 256);
    w.sagg = o;   o = align_up(o + ns * D * D * sizeof(float), 256);
    w.saggT = o;  o = align_up(o + ns * D * D * sizeof(float), 256);
    w.sexps = o;  o = align_up(o + ns * 8 * sizeof(int), 256);
    w.sfin = o;   o = align_up(o + ns * D * sizeof(float), 256);
    w.sbout = o;  o = align_up(o + ns * D * sizeof(float), 256);
    w.F = o;      o = align_up(o + (own_F ? rows * Dr * sizeof(float) : 0), 256);
    w.Bv = o;     o = align_up(o + (p.fused_apply ? 0 : rows * Dr * sizeof(float)), 256);
    w.part = o;   o = align_up(o + nc * sizeof(double), 256);
    w.suspect = o; o = align_up(o + (size_t)batch * sizeof(int), 256);
    w.total = o;
    return w;
}

size_t large_d_smooth_ws_bytes(int Dr, long long T, int batch) {
    return large_smooth_ws(Dr, T, batch, true).total;   // sized for the case without a filtered output
}

template <int D>
static void launch_carry(hipStream_t st, const LargeArgs& a, int cps, const float* agg, const float* aggT,
                         const int* exps, float* fin, float* bout, int seglen, int nseg, const float* start_f,
                         const float* start_b, int* suspect) {
    const unsigned blocks = 2u * (unsigned)a.batch * (unsigned)nseg;
    if constexpr (D <= 32)
        launch("ld_carry", ld_carry_wave_kernel<D>, dim3(blocks), dim3(64), st, a.prior, a.D, cps, a.shared_model, agg,
               aggT, exps, fin, bout, seglen, nseg, start_f, start_b, suspect);
    else
        launch("ld_carry", ld_carry_kernel<D>, dim3(blocks), dim3(256), st, a.prior, a.D, cps, a.shared_model, agg, aggT,
               exps, fin, bout, seglen, nseg, start_f, start_b, suspect);
}

template <int D>
static int large_smooth_impl(const LargeArgs& a, float* marg, float* filt, double* loglik_out) {
    using C = LargeCfg<D>;
    const SmoothPlan p = smooth_plan(a.D, a.T, a.batch);
    const LargeSmoothWs w = large_smooth_ws(a.D, a.T, a.batch, true);
    if (a.ws_bytes < w.total) return 3;
    const long long rows = a.T * a.batch;
    if (rows > 0x7fffffffLL * 4 || p.nchunks > 0x3fffffffLL) return 2;
    char* ws = static_cast<char*>(a.ws);
    float* rowmax = reinterpret_cast<float*>(ws + w.rowmax);
    float* agg = reinterpret_cast<float*>(ws + w.agg);
    float* aggT = reinterpret_cast<float*>(ws + w.aggT);
    int* exps = reinterpret_cast<int*>(ws + w.exps);
    float* fin = reinterpret_cast<float*>(ws + w.fin);
    float* bout = reinterpret_cast<float*>(ws + w.bout);
    float* gagg = reinterpret_cast<float*>(ws + w.gagg);
    float* gaggT = reinterpret_cast<float*>(ws + w.gaggT);
    int* gexps = reinterpret_cast<int*>(ws + w.gexps);
    float* gfin = reinterpret_cast<float*>(ws + w.gfin);
    float* gbout = reinterpret_cast<float*>(ws + w.gbout);
    float* sagg = reinterpret_cast<float*>(ws + w.sagg);
    float* saggT = reinterpret_cast<float*>(ws + w.saggT);
    int* sexps = reinterpret_cast<int*>(ws + w.sexps);
    float* sfin = reinterpret_cast<float*>(ws + w.sfin);
    float* sbout = reinterpret_cast<float*>(ws + w.sbout);
    float* F = filt ? filt : reinterpret_cast<float*>(ws + w.F);
    float* Bv = reinterpret_cast<float*>(ws + w.Bv);
    double* part = reinterpret_cast<double*>(ws + w.part);
    int* suspect = reinterpret_cast<int*>(ws + w.suspect);
    hipStream_t st = a.stream;
    const dim3 block(256);
    // up to 32 states the aggregate kernel forms the row maxima on its way (when there is one: cps > 1)
    const bool fold_rowmax = D <= 32 && p.cps > 1;
    if (!fold_rowmax) {
        int width = 1;
        while (width < (a.D + 3) / 4) width <<= 1;
        const long long rpb = 4LL * STREAM_UNROLL * (64 / width);   // rows per workgroup
        launch("ld_rowmax", ld_rowmax_kernel, dim3((unsigned)((rows + rpb - 1) / rpb)), block, st, a.ll, rows, a.D, rowmax, suspect, a.batch);
    }
    if (p.cps == 1) {
        // a sequence is one chunk: it starts from the prior and ends with the all-ones vector; no aggregates, no carries
        fin = nullptr;
        bout = nullptr;
    } else {
        launch("ld_aggregate", ld_aggregate_kernel<D>, dim3((unsigned)((p.nchunks + C::CPW - 1) / C::CPW)), block, st, a.A,
               a.ll, rowmax, fold_rowmax ? 1 : 0, a.T, a.D, p.Lc, p.cps, p.nchunks, a.shared_model, agg, aggT, exps,
               fold_rowmax ? suspect : (int*)nullptr, a.batch);
    }
    if (p.cps > 1 && p.two_level) {
        const long long ngroups = (long long)p.G * a.batch;
        launch("ld_product", ld_product_kernel<D>, dim3((unsigned)((ngroups + C::CPW - 1) / C::CPW)), block, st,
               (const float*)aggT, (const int*)exps, p.cps, p.g, p.G, ngroups, gagg, gaggT, gexps);
        if (p.three_level) {
            // the same once more over the groups; carries at the boundaries of the groups of groups, then inside each
            // of them at the group boundaries
            const long long nsuper = (long long)p.G2 * a.batch;
            launch("ld_product", ld_product_kernel<D>, dim3((unsigned)((nsuper + C::CPW - 1) / C::CPW)), block, st,
                   (const float*)gaggT, (const int*)gexps, p.G, p.g2, p.G2, nsuper, sagg, saggT, sexps);
            launch_carry<D>(st, a, p.G2, sagg, saggT, sexps, sfin, sbout, p.G2, 1, nullptr, nullptr, suspect);
            launch_carry<D>(st, a, p.G, gagg, gaggT, gexps, gfin, gbout, p.g2, p.G2, sfin, sbout, suspect);
        } else {
            // carries at the group boundaries
            launch_carry<D>(st, a, p.G, gagg, gaggT, gexps, gfin, gbout, p.G, 1, nullptr, nullptr, suspect);
        }
        // inside every group from the carries at its boundaries
        launch_carry<D>(st, a, p.cps, agg, aggT, exps, fin, bout, p.g, p.G, gfin, gbout, suspect);
    } else if (p.cps > 1) {
        launch_carry<D>(st, a, p.cps, agg, aggT, exps, fin, bout, p.cps, 1, nullptr, nullptr, suspect);
    }
    const int half = (int)((p.nchunks + C::VCPW - 1) / C::VCPW);
    bool marginals_done = false;
    if constexpr (D <= 32) {
        const int rhalf = (int)((p.nchunks + 15) / 16);
        if (p.fused_apply) {
            // both recursions and the marginals in one pass over the chunks
            launch("ld_apply", ld_apply_row_kernel<D, true>, dim3((unsigned)rhalf), block, st, a.prior, a.A, a.ll, rowmax,
                   a.T, a.D, p.Lc, p.cps, p.nchunks, a.shared_model, fin, bout, F, marg, part, rhalf);
            marginals_done = true;
        } else {
            launch("ld_apply", ld_apply_row_kernel<D, false>, dim3(2u * (unsigned)rhalf), block, st, a.prior, a.A, a.ll,
                   rowmax, a.T, a.D, p.Lc, p.cps, p.nchunks, a.shared_model, fin, bout, F, Bv, part, rhalf);
        }
    } else {
        launch("ld_apply", ld_apply_kernel<D>, dim3(2u * (unsigned)half), block, st, a.prior, a.A, a.ll, rowmax, a.T, a.D,
               p.Lc, p.cps, p.nchunks, a.shared_model, fin, bout, F, Bv, part, half);
    }
    if (!marginals_done) {
        const int lpr = (a.D + 3) / 4;
        int width = 1;
        while (width < lpr) width <<= 1;
        const long long rows_per_block = 4LL * STREAM_UNROLL * (64 / width);
        launch("ld_combine", ld_combine_kernel, dim3((unsigned)((rows + rows_per_block - 1) / rows_per_block)), block, st, F,
               Bv, rows, a.D, marg);
    }
    if (p.cps == 1)
        launch("ld_finalize", ld_finalize_kernel, dim3((unsigned)a.batch), block, st, part, p.cps, loglik_out);
    else   // the sum of the chunk evidences, and the sequences that the carries marked
        launch("ld_repair", ld_repair_kernel, dim3((unsigned)a.batch), dim3(REPAIR_THREADS), st, (const double*)part, p.cps,
               (const int*)suspect, a.prior, a.A, a.ll,
               (const float*)rowmax, a.T, a.D, a.shared_model, marg, filt, loglik_out);
    return hipGetLastError() == hipSuccess ? 0 : 4;
}

// Chunking of the block-element path (both operators): the smoother's chunk lengths, no second-level plan.
LargePlan element_plan(int Dr, long long T, int batch) {
    const SmoothPlan sp = smooth_plan(Dr, T, batch);
    LargePlan p;
    p.DP = sp.DP; p.Lc = sp.Lc; p.cps = sp.cps; p.nchunks = sp.nchunks;
    return p;
}

// Sum-product block element: rowmax -> chunk aggregates -> products of g aggregates at a time until one
// is left per sequence -> finish.
struct ElementSpWs { size_t rowmax, agg, aggT, exps, lvl[2][3], total; int g; };

static ElementSpWs element_sp_ws(int Dr, long long T, int batch) {
    const LargePlan p = element_plan(Dr, T, batch);
    const size_t D = p.DP, nc = (size_t)p.nchunks, rows = (size_t)T * batch;
    ElementSpWs w;
    w.g = p.DP >= 64 ? 4 : 8;
    size_t o = 0;
    w.rowmax = o; o = align_up(o + rows * sizeof(float), 256);
    w.agg = o;    o = align_up(o + nc * D * D * sizeof(float), 256);
    w.aggT = o;   o = align_up(o + nc * D * D * sizeof(float), 256);
    w.exps = o;   o = align_up(o + nc * 8 * sizeof(int), 256);
    size_t n = (size_t)p.cps;
    for (int l = 0; l < 2; ++l) {
        n = (n + w.g - 1) / w.g;
        const size_t cnt = n * batch;
        w.lvl[l][0] = o; o = align_up(o + cnt * D * D * sizeof(float), 256);
        w.lvl[l][1] = o; o = align_up(o + cnt * D * D * sizeof(float), 256);
        w.lvl[l][2] = o; o = align_up(o + cnt * 8 * sizeof(int), 256);
    }
    w.total = o;
    return w;
}

size_t large_d_element_sp_ws_bytes(int Dr, long long T, int batch) { return element_sp_ws(Dr, T, batch).total; }

template <int D>
static int large_element_sp_impl(const LargeArgs& a, float* element, double* log_scale) {
    using C = LargeCfg<D>;
    const LargePlan p = element_plan(a.D, a.T, a.batch);
    const ElementSpWs w = element_sp_ws(a.D, a.T, a.batch);
    if (a.ws_bytes < w.total) return 3;
    const long long rows = a.T * a.batch;
    if (rows > 0x7fffffffLL * 4 || p.nchunks > 0x3fffffffLL) return 2;
    char* ws = static_cast<char*>(a.ws);
    float* rowmax = reinterpret_cast<float*>(ws + w.rowmax);
    float* agg = reinterpret_cast<float*>(ws + w.agg);
    float* aggT = reinterpret_cast<float*>(ws + w.aggT);
    int* exps = reinterpret_cast<int*>(ws + w.exps);
    hipStream_t st = a.stream;
    const dim3 block(256);
    {
        int width = 1;
        while (width < (a.D + 3) / 4) width <<= 1;
        const long long rpb = 4LL * STREAM_UNROLL * (64 / width);
        launch("ld_rowmax", ld_rowmax_kernel, dim3((unsigned)((rows + rpb - 1) / rpb)), block, st, a.ll, rows, a.D, rowmax, (int*)nullptr, 0);
    }
    launch("ld_aggregate", ld_aggregate_kernel<D>, dim3((unsigned)((p.nchunks + C::CPW - 1) / C::CPW)), block, st, a.A,
           a.ll, rowmax, 0, a.T, a.D, p.Lc, p.cps, p.nchunks, a.shared_model, agg, aggT, exps, (int*)nullptr, 0);
    const float* cur = agg;
    const float* curT = aggT;
    const int* cure = exps;
    int n = p.cps, l = 0;
    while (n > 1) {
        const int G = (n + w.g - 1) / w.g;
        const long long ngroups = (long long)G * a.batch;
        float* o = reinterpret_cast<float*>(ws + w.lvl[l][0]);
        float* oT = reinterpret_cast<float*>(ws + w.lvl[l][1]);
        int* oe = reinterpret_cast<int*>(ws + w.lvl[l][2]);
        launch("ld_product", ld_product_kernel<D>, dim3((unsigned)((ngroups + C::CPW - 1) / C::CPW)), block, st, curT, cure, n,
               w.g, G, ngroups, o, oT, oe);
        cur = o; curT = oT; cure = oe;
        n = G;
        l ^= 1;
    }
    launch("ld_element_finish", ld_element_finish_kernel<D>, dim3((unsigned)a.batch), block, st, cur, cure,
           (const float*)rowmax, a.T, a.D, element, log_scale);
    return hipGetLastError() == hipSuccess ? 0 : 4;
}

int large_d_element_sp(const LargeArgs& a, float* element, double* log_scale) {
    switch (element_plan(a.D, a.T, a.batch).DP) {
        case 16: return large_element_sp_impl<16>(a, element, log_scale);
        case 32: return large_element_sp_impl<32>(a, element, log_scale);
        case 64: return large_element_sp_impl<64>(a, element, log_scale);
        case 128: return large_element_sp_impl<128>(a, element, log_scale);
        default: return 2;
    }
}

int large_d_smooth(const LargeArgs& a, float* marg, float* filt, double* loglik_out) {
    const int DP = large_plan(a.D, a.T, a.batch).DP;
    switch (DP) {
        case 16: return large_smooth_impl<16>(a, marg, filt, loglik_out);
        case 32: return large_smooth_impl<32>(a, marg, filt, loglik_out);
        case 64: return large_smooth_impl<64>(a, marg, filt, loglik_out);
        case 128: return large_smooth_impl<128>(a, marg, filt, loglik_out);
        default: return 2;
    }
}

}  // namespace hmm
