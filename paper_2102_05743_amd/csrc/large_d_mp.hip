// Viterbi / MAP decoding for large state spaces (9 <= D <= 128, padded to 16 / 32 / 64 / 128).
//
// Max-product operator of Definition 5 on logarithms, (a v b)(i,k) = max_j [a(i,j) + b(j,k)]:
// no matrix-core form exists for (max,+), so chunk aggregates are built on the vector ALUs.
//   aggregate  chunk aggregates P_c = psi_{k0} v ... v psi_{k1-1}, psi_k(i,j) = log A(i,j) + ll_k(j)
//   carry      V at chunk boundaries: v <- v v P_c along the chunks of a sequence; long sequences get a
//              second scan level (aggregates of groups of chunks by a tree of pairwise products, a walk
//              over the groups, then walks inside all groups at once)
//   forward    V_k and back-pointers u_{k-1}(x_k) inside each chunk (Sec. IV-A), the chunk's
//              back-pointer map (state at its last step -> state at the previous chunk's last
//              step), x*_T = argmax V_T in the sequence's last chunk, chunk-local log-probability
//   suffix     reversed all-prefix-sums under composition over the chunk maps, collapsed to the
//              single state it is applied to: the state at every chunk's last step (grouped the same
//              way for long sequences); log-probability
//   path       back-pointer walk inside each chunk
// Aggregates and carries are scale-free (offsets are dropped); the log-probability is the sum of the
// chunk-local growths of max_j V, each measured from a carry renormalised to max 0.
//
// The same aggregates and carries, run in both directions, also serve the paper's parallel
// max-product algorithm as printed (Algorithm 5): maximum forward and backward potentials inside
// the chunks and Theorem 4's per-step combination (lm_apply, lm_combine, lm_finalize below).
// Aggregates that keep their offsets and the tree of products also give the block-wise elements of
// Sec. V-B under this operator (lv_aggregate_offsets, lv_tree_product, lv_element_finish).
// For D <= 32 the in-chunk recursions have row-parallel variants (one chunk per DPP row of 16 lanes).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "ktimer.hpp"
#include "large_d.hpp"
#include "large_d_device.hpp"

namespace hmm {

template <int D>
struct MpCfg {
    static constexpr int WPC = (D >= 32) ? 4 : 1;        // waves per chunk in the aggregate kernel
    static constexpr int CPW = 4 / WPC;                  // chunks per workgroup
};

HMM_DEV float max3f(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }

template <int D>
HMM_DEV void chunk_sync() {
    if constexpr (MpCfg<D>::WPC == 4) lds_barrier();
    else __builtin_amdgcn_wave_barrier();
}

HMM_DEV float safe_log(float p) { return p > 0.0f ? logf(p) : -INFINITY; }

// ---------------------------------------------------------------------------------------------
// Chunk aggregates without any operand broadcast: a systolic arrangement inside each
// DPP row of 16 lanes.  A row of lanes owns 16 columns j = 16*cb + l of P' and works through its
// share of the rows i of P.  For one row i, lane l holds P(i, 16q + l) for every q; the term
// P(i,k) + log A(k,j) needs k = 16q + (l - r) mod 16 at rotation r, which is exactly what a DPP
// row rotation by r delivers as an operand of the add, and the matching log A(k,j) sits in a
// register fixed per (q, r).  Every add therefore reads one rotated register and one constant
// register: 1.5 vector instructions per term (add + half a three-way max), no LDS traffic, no
// scalar loads, no data movement instruction in the inner loop.
template <int R>
HMM_DEV float row_rotate(float v) {
    if constexpr (R == 0) return v;
    else return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x120 + R, 0xF, 0xF, true));
}

template <int D, int Q, int R>
HMM_DEV void systolic_terms(const float (&pr)[D / 16], const float (&la)[D], float& acc) {
    if constexpr (R < 16) {
        const float t0 = row_rotate<R>(pr[Q]) + la[Q * 16 + R];
        const float t1 = row_rotate<R + 1>(pr[Q]) + la[Q * 16 + R + 1];
        acc = max3f(acc, t0, t1);
        systolic_terms<D, Q, R + 2>(pr, la, acc);
    } else if constexpr (Q + 1 < D / 16) {
        systolic_terms<D, Q + 1, 0>(pr, la, acc);
    }
}

template <int D, bool WITH_OFFSETS>
HMM_DEV void lv_aggregate_systolic_body(const float* __restrict__ A, const float* __restrict__ ll, long long T, int Dr,
                                        int Lc, int cps, long long nchunks, int shared_model, float* __restrict__ agg,
                                        float* __restrict__ agg_other, double* __restrict__ agg_off) {
    constexpr int NQ = D / 16;             // column blocks = registers per lane for one row of P
    constexpr int WPCH = MpCfg<D>::WPC;    // waves per chunk: a workgroup for D >= 32, else one wave
    constexpr int CPWG = 4 / WPCH;         // chunks per workgroup
    constexpr int RSPLIT = 4 * WPCH / NQ;  // row ranges (DPP rows of the chunk / column blocks)
    constexpr int RPD = D / RSPLIT;        // rows of P per DPP row
    __shared__ __align__(16) float pbuf[CPWG * 2 * D * D];   // P, double-buffered: [i][l][q] with k = 16q + l
    __shared__ float wmax[2 * 4];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int cl = wave / WPCH;                                  // chunk inside the workgroup
    const int drow = (wave % WPCH) * 4 + lane / 16;              // DPP row inside the chunk
    const int l = lane & 15;
    const int cb = drow % NQ, rs = drow / NQ;
    const int j = 16 * cb + l;
    const long long chunk = (long long)blockIdx.x * CPWG + cl;
    const ChunkCoord cc = chunk_coord(chunk, nchunks, cps, T, Lc);
    const float* Am = A + (shared_model ? 0 : (size_t)cc.seq * Dr * Dr);
    float la[D];   // la[16q + r] = log A(16q + (l - r) mod 16, j)
#pragma unroll
    for (int q = 0; q < NQ; ++q)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int k = 16 * q + ((l - r) & 15);
            float v = (k == j) ? 0.0f : -INFINITY;
            if (k < Dr && j < Dr) v = safe_log(Am[(size_t)k * Dr + j]);
            la[16 * q + r] = v;
        }
    const float* lseq = ll + (size_t)cc.seq * T * Dr;
    if constexpr (D == 16) {
        // One column block: the row P(i, .) that a DPP row of lanes rotates is exactly what its lanes hold,
        // so P never leaves the registers (four rows per DPP row of lanes), and its maximum is taken off
        // every fourth step only.
        float pr[RPD];
        float xn = -INFINITY;
        if (j < Dr && cc.nsteps > 0) xn = lseq[(size_t)cc.t0 * Dr + j];
        // the sequence's first element has no transition part: the aggregate after it is that step's log-likelihoods
        // on the diagonal, which is written here in place of the neutral element (0 on the diagonal)
        const int s_begin = (cc.t0 == 0 && cc.nsteps > 0) ? 1 : 0;
        {
            const float diag = s_begin ? xn : 0.0f;
#pragma unroll
            for (int r = 0; r < RPD; ++r) pr[r] = (rs * RPD + r == j) ? diag : -INFINITY;
            if (s_begin && s_begin < cc.nsteps && j < Dr) xn = lseq[(size_t)(cc.t0 + 1) * Dr + j];
        }
        float off = 0.0f;
        double offsum = 0.0;
        auto take_off_maximum = [&]() {
            float lmax = pr[0];
#pragma unroll
            for (int r = 1; r < RPD; ++r) lmax = fmaxf(lmax, pr[r]);
            const float m = wave_max(lmax);
            off = (m == -INFINITY) ? 0.0f : m;
            offsum += (double)off;
        };
        if (s_begin && cc.nsteps == 1) take_off_maximum();   // a chunk that is only that first element
        for (int s = s_begin; s < cc.nsteps; ++s) {
            const float add = xn - off;
            if (s + 1 < cc.nsteps && j < Dr) xn = lseq[(size_t)(cc.t0 + s + 1) * Dr + j];
#pragma unroll
            for (int r = 0; r < RPD; ++r) {
                const float one[1] = {pr[r]};
                float acc = -INFINITY;
                systolic_terms<D, 0, 0>(one, la, acc);
                pr[r] = acc + add;
            }
            off = 0.0f;
            if ((s & 3) == 3 || s == cc.nsteps - 1) take_off_maximum();
        }
        if (cc.nsteps > 0) {
            if constexpr (WITH_OFFSETS) {
                if (lane == 0) agg_off[chunk] = offsum;
            }
            float* dst = agg + (size_t)chunk * D * D;
#pragma unroll
            for (int r = 0; r < RPD; ++r) {
                const int i = rs * RPD + r;
                const float val = pr[r] - off;
                dst[(size_t)j * D + i] = val;   // stored transposed, as the one-wave carry reads it
                if (agg_other != nullptr) agg_other[(size_t)chunk * D * D + (size_t)i * D + j] = val;
            }
        }
        return;
    }
    float* p0 = pbuf + cl * 2 * D * D;
    float* p1 = p0 + D * D;
    // The sequence's first element has no transition part: the aggregate after it is that step's log-likelihoods on
    // the diagonal.  It is written here, in place of the neutral element (0 on the diagonal, -inf elsewhere), so that
    // the step loop needs no case for it.  Element (i, k) lives at i*D + (k%16)*NQ + k/16.
    const int s_begin = (cc.t0 == 0 && cc.nsteps > 0) ? 1 : 0;
    float xn = -INFINITY;
    if (j < Dr && cc.nsteps > 0) xn = lseq[(size_t)cc.t0 * Dr + j];
    {
        const float diag = s_begin ? xn : 0.0f;
        for (int r = 0; r < RPD; ++r) {
            const int i = rs * RPD + r;
            p0[i * D + l * NQ + cb] = (i == j) ? diag : -INFINITY;
        }
        if (s_begin && s_begin < cc.nsteps && j < Dr) xn = lseq[(size_t)(cc.t0 + 1) * Dr + j];
    }
    chunk_sync<D>();
    float off = 0.0f;
    double offsum = 0.0;
    int cur = 0;
    if (s_begin == cc.nsteps && s_begin) {
        // a chunk that is only that first element (uniform over the chunk's waves): its maximum is taken off here
        float m = wave_max(xn);
        if constexpr (WPCH == 4) {
            if (lane == 0) wmax[wave] = m;
            lds_barrier();
            m = fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3]));
        }
        off = (m == -INFINITY) ? 0.0f : m;
        if constexpr (WITH_OFFSETS) offsum += (double)off;
    }
    for (int s = s_begin; s < cc.nsteps; ++s) {
        const float x = xn;
        if (s + 1 < cc.nsteps && j < Dr) xn = lseq[(size_t)(cc.t0 + s + 1) * Dr + j];
        const float* po = cur ? p1 : p0;
        float* pn = cur ? p0 : p1;
        const float add = x - off;
        float lmax = -INFINITY;
#pragma unroll(RPD <= 4 ? RPD : 1)
        for (int r = 0; r < RPD; ++r) {
            const int i = rs * RPD + r;
            float pr[NQ];
            const float* src = po + i * D + l * NQ;
            if constexpr (NQ >= 4) {
#pragma unroll
                for (int q4 = 0; q4 < NQ; q4 += 4) {
                    const float4 v4 = *reinterpret_cast<const float4*>(src + q4);
                    pr[q4] = v4.x; pr[q4 + 1] = v4.y; pr[q4 + 2] = v4.z; pr[q4 + 3] = v4.w;
                }
            } else if constexpr (NQ == 2) {
                const float2 v2 = *reinterpret_cast<const float2*>(src);
                pr[0] = v2.x; pr[1] = v2.y;
            } else {
                pr[0] = src[0];
            }
            float acc = -INFINITY;
            systolic_terms<D, 0, 0>(pr, la, acc);
            acc += add;
            lmax = fmaxf(lmax, acc);
            pn[i * D + l * NQ + cb] = acc;
        }
        // the running maximum is taken off every fourth step (and after the last one), one step late
        const bool take = (s & 3) == 3 || s == cc.nsteps - 1;   // uniform over the workgroup
        float m = 0.0f;
        if (take) m = wave_max(lmax);
        if constexpr (WPCH == 4) {
            if (take && lane == 0) wmax[(cur ^ 1) * 4 + wave] = m;
            lds_barrier();
            if (take)
                m = fmaxf(fmaxf(wmax[(cur ^ 1) * 4], wmax[(cur ^ 1) * 4 + 1]),
                          fmaxf(wmax[(cur ^ 1) * 4 + 2], wmax[(cur ^ 1) * 4 + 3]));
        } else {
            chunk_sync<D>();
        }
        off = (m == -INFINITY) ? 0.0f : m;
        if constexpr (WITH_OFFSETS) offsum += (double)off;
        cur ^= 1;
    }
    if (cc.nsteps > 0) {
        // what the rescalings removed, for callers that need the aggregate's absolute level
        if constexpr (WITH_OFFSETS) {
            if ((wave % WPCH) == 0 && lane == 0) agg_off[chunk] = offsum;
        }
        const float* pf = cur ? p1 : p0;
        float* dst = agg + (size_t)chunk * D * D;
        for (int r = 0; r < RPD; ++r) {
            const int i = rs * RPD + r;
            const float val = pf[i * D + l * NQ + cb] - off;
            // D <= 32: stored transposed, the one-wave carry reads the terms of a column contiguously
            dst[(D <= 32) ? ((size_t)j * D + i) : ((size_t)i * D + j)] = val;
            // the backward carry of the two-filter plan wants the other orientation
            if (agg_other != nullptr)
                agg_other[(size_t)chunk * D * D + ((D <= 32) ? ((size_t)i * D + j) : ((size_t)j * D + i))] = val;
        }
    }
}

template <int D>
__global__ __launch_bounds__(256) void lv_aggregate_systolic_kernel(const float* __restrict__ A,
                                                                    const float* __restrict__ ll, long long T, int Dr,
                                                                    int Lc, int cps, long long nchunks,
                                                                    int shared_model, float* __restrict__ agg,
                                                                    float* __restrict__ agg_other) {
    lv_aggregate_systolic_body<D, false>(A, ll, T, Dr, Lc, cps, nchunks, shared_model, agg, agg_other, nullptr);
}

// The same, also recording per chunk what the rescalings removed (block-wise elements need the
// aggregates' absolute level).
template <int D>
__global__ __launch_bounds__(256) void lv_aggregate_offsets_kernel(const float* __restrict__ A, const float* __restrict__ ll,
                                                                   long long T, int Dr, int Lc, int cps, long long nchunks,
                                                                   int shared_model, float* __restrict__ agg,
                                                                   double* __restrict__ agg_off) {
    lv_aggregate_systolic_body<D, true>(A, ll, T, Dr, Lc, cps, nchunks, shared_model, agg, nullptr, agg_off);
}

// ---------------------------------------------------------------------------------------------
// V at chunk boundaries.  One workgroup per sequence; lane = (column j, part q of the max over i).
// vin[c] = V just before chunk c (log prior for c = 0, afterwards shifted to max 0).
template <int D>
__global__ __launch_bounds__(256) void lv_carry_kernel(const float* __restrict__ prior, int Dr, int cps,
                                                       int shared_model, const float* __restrict__ agg,
                                                       float* __restrict__ vin, const float* __restrict__ agg_other,
                                                       float* __restrict__ bout, int seglen, int nseg,
                                                       const float* __restrict__ start,
                                                       const float* __restrict__ start_b) {
    // With bout given the grid is doubled: odd workgroups run the backward direction, the same
    // recursion on the aggregates' other orientation, over the chunks right to left, from the zero
    // vector: bout[c] = backward potential at chunk c's last step.
    // The chunks of a sequence may be cut into nseg segments of seglen chunks, walked independently (one
    // workgroup per segment and direction) from start[segment] = V just before the segment, resp.
    // start_b[segment] = backward potential at the segment's last step.
    constexpr int Q = 256 / D;
    constexpr int RPT = D / Q;
    __shared__ float vec[D];
    __shared__ float partial[Q * D];
    __shared__ float max_lds;
    const bool two = bout != nullptr;
    const int unit = two ? blockIdx.x >> 1 : blockIdx.x;
    const int dir = two ? (blockIdx.x & 1) : 0;
    const int seq = unit / nseg, seg = unit % nseg;
    const int c_begin = seg * seglen, c_end = min(cps, c_begin + seglen);
    const int nhops = c_end - c_begin;
    const int j = threadIdx.x % D, q = threadIdx.x / D;
    const float* mats = (dir ? agg_other : agg) + (size_t)seq * cps * D * D;
    float* out = (dir ? bout : vin) + (size_t)seq * cps * D;
    float v;
    if (dir) v = (start_b != nullptr) ? start_b[(size_t)unit * D + j] : ((j < Dr) ? 0.0f : -INFINITY);
    else if (start != nullptr) v = start[(size_t)unit * D + j];
    else v = (j < Dr) ? safe_log(prior[(shared_model ? 0 : (size_t)seq * Dr) + j]) : -INFINITY;
    float pv[RPT];
    auto load_mat = [&](int it) {
        const float* Mx = mats + (size_t)(dir ? c_end - 1 - it : c_begin + it) * D * D;
#pragma unroll
        for (int r = 0; r < RPT; ++r) pv[r] = Mx[(size_t)(q * RPT + r) * D + j];
    };
    if (nhops > 0) load_mat(0);
    for (int it = 0; it < nhops; ++it) {
        const int c = dir ? c_end - 1 - it : c_begin + it;
        if (q == 0) {
            out[(size_t)c * D + j] = v;
            vec[j] = v;
        }
        lds_barrier();
        float acc = -INFINITY;
#pragma unroll
        for (int r = 0; r < RPT; ++r) acc = fmaxf(acc, vec[q * RPT + r] + pv[r]);
        if (it + 1 < nhops) load_mat(it + 1);
        partial[q * D + j] = acc;
        lds_barrier();
        float g = -INFINITY;
        if (q == 0) {
#pragma unroll
            for (int p = 0; p < Q; ++p) g = fmaxf(g, partial[p * D + j]);
        }
        if (threadIdx.x < 64) {
            float m = -INFINITY;
            for (int jj = threadIdx.x; jj < D; jj += 64) {
#pragma unroll
                for (int p = 0; p < Q; ++p) m = fmaxf(m, partial[p * D + jj]);
            }
            m = wave_max(m);
            if (threadIdx.x == 0) max_lds = (m == -INFINITY) ? 0.0f : m;
        }
        lds_barrier();
        v = g - max_lds;
    }
}

// The same for D <= 32 by a single wave per sequence (lane = (column j, part h of the max over i),
// parts combined with quad permutes, wave-level ordering only, aggregates prefetched PF hops ahead):
// a hop costs a few hundred cycles, which is what bounds a long sequence.
template <int D>
__global__ __launch_bounds__(64) void lv_carry_wave_kernel(const float* __restrict__ prior, int Dr, int cps,
                                                           int shared_model, const float* __restrict__ agg,
                                                           float* __restrict__ vin,
                                                           const float* __restrict__ agg_other,
                                                           float* __restrict__ bout, int seglen, int nseg,
                                                           const float* __restrict__ start,
                                                           const float* __restrict__ start_b) {
    // With bout given the grid is doubled and odd workgroups run the backward direction; forward walks may
    // be cut into segments with their own start vectors (see lv_carry_kernel).
    static_assert(D <= 32, "one wave covers the columns");
    constexpr int PARTS = 64 / D;
    constexpr int RPT = D / PARTS;
    constexpr int PF = 8;
    __shared__ __align__(16) float vec[D];
    const bool two = bout != nullptr;
    const int unit = two ? blockIdx.x >> 1 : blockIdx.x;
    const int dir = two ? (blockIdx.x & 1) : 0;
    const int seq = unit / nseg, seg = unit % nseg;
    const int c_begin = seg * seglen, c_end = min(cps, c_begin + seglen);
    const int nhops = c_end - c_begin;
    if (nhops <= 0) return;   // uniform over the wave
    const int lane = threadIdx.x;
    const int h = lane % PARTS, j = lane / PARTS;
    const float* mats = (dir ? agg_other : agg) + (size_t)seq * cps * D * D;
    float* out = (dir ? bout : vin) + (size_t)seq * cps * D;
    float v;
    if (dir) v = (start_b != nullptr) ? start_b[(size_t)unit * D + j] : ((j < Dr) ? 0.0f : -INFINITY);
    else if (start != nullptr) v = start[(size_t)unit * D + j];
    else v = (j < Dr) ? safe_log(prior[(shared_model ? 0 : (size_t)seq * Dr) + j]) : -INFINITY;
    settle_loaded(v);
    float pv[PF][RPT];
    // unconditional loads (clamped hop index): the compiler can count outstanding loads exactly
    auto load_mat = [&](int it, float (&m)[RPT]) {
        const int itc = it < nhops ? it : nhops - 1;
        const int c = dir ? c_end - 1 - itc : c_begin + itc;
        const float* Mx = mats + (size_t)c * D * D + (size_t)j * D + h * RPT;   // the lane's terms are contiguous
#pragma unroll
        for (int r4 = 0; r4 < RPT; r4 += 4) {
            const float4 x = *reinterpret_cast<const float4*>(Mx + r4);
            m[r4] = x.x; m[r4 + 1] = x.y; m[r4 + 2] = x.z; m[r4 + 3] = x.w;
        }
    };
    auto hop = [&](int it, const float (&m)[RPT]) {
        const int c = dir ? c_end - 1 - it : c_begin + it;
        if (h == 0) {
            out[(size_t)c * D + j] = v;
            vec[j] = v;
        }
        wave_lds_sync();
        float a0 = -INFINITY, a1 = -INFINITY;   // independent chains
#pragma unroll
        for (int r4 = 0; r4 < RPT; r4 += 4) {
            const float4 x = *reinterpret_cast<const float4*>(vec + h * RPT + r4);
            a0 = max3f(a0, x.x + m[r4], x.y + m[r4 + 1]);
            a1 = max3f(a1, x.z + m[r4 + 2], x.w + m[r4 + 3]);
        }
        wave_lds_sync();
        float acc = fmaxf(a0, a1);
        acc = fmaxf(acc, quad_xor1(acc));
        if constexpr (PARTS == 4) acc = fmaxf(acc, quad_xor2(acc));
        const float mx = wave_max(acc);
        v = acc - ((mx == -INFINITY) ? 0.0f : mx);
    };
#pragma unroll
    for (int p = 0; p < PF; ++p) load_mat(p, pv[p]);
    const int nfull = nhops / PF * PF;
    for (int c0 = 0; c0 < nfull; c0 += PF) {
#pragma unroll
        for (int p = 0; p < PF; ++p) {
            hop(c0 + p, pv[p]);
            load_mat(c0 + p + PF, pv[p]);
        }
    }
#pragma unroll
    for (int p = 0; p < PF; ++p)
        if (nfull + p < nhops) hop(nfull + p, pv[p]);   // slot p holds hop nfull + p
}

// ---------------------------------------------------------------------------------------------
// Forward max-plus recursion with back-pointers inside the chunks, the chunk's back-pointer map
// and log-probability growth.  Lane = (column j inside the wave, part h of the max over i), log A
// in registers; back-pointers are kept in LDS for the map composition and copied to the workspace.
template <int D>
__global__ __launch_bounds__(256) void lv_forward_kernel(const float* __restrict__ prior, const float* __restrict__ A,
                                                         const float* __restrict__ ll, long long T, int Dr, int Lc,
                                                         int cps, long long nchunks, int shared_model,
                                                         const float* __restrict__ vin, uint8_t* __restrict__ bp,
                                                         uint8_t* __restrict__ cmap, int* __restrict__ xstar,
                                                         double* __restrict__ part) {
    using C = LargeCfg<D>;
    extern __shared__ __align__(16) unsigned char dyn_lds[];   // back-pointers of the workgroup's chunks
    __shared__ __align__(16) float vbuf[2 * C::VCPW * D];
    __shared__ float wmaxs[2 * C::VCPW * C::VWPC];
    __shared__ float red_v[C::VCPW * 4];
    __shared__ int red_i[C::VCPW * 4];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int cl = wave / C::VWPC, wv = wave % C::VWPC;
    const int jl = lane % C::CPWV, h = lane / C::CPWV;
    const int j = C::CPWV * wv + jl;
    const long long chunk = (long long)blockIdx.x * C::VCPW + cl;
    const ChunkCoord cc = chunk_coord(chunk, nchunks, cps, T, Lc);
    const float* Am = A + (shared_model ? 0 : (size_t)cc.seq * Dr * Dr);
    uint8_t* bpl = dyn_lds + (size_t)cl * Lc * D;
    float lareg[C::RPP];
#pragma unroll
    for (int r = 0; r < C::RPP; ++r) {
        const int i = h * C::RPP + r;
        float v = (i == j) ? 0.0f : -INFINITY;
        if (i < Dr && j < Dr) v = safe_log(Am[(size_t)i * Dr + j]);
        lareg[r] = v;
    }
    const float* lseq = ll + (size_t)cc.seq * T * Dr;
    const bool first_chunk = (chunk % cps) == 0;
    float v0 = -INFINITY;
    if (cc.nsteps > 0) {
        if (first_chunk) v0 = (j < Dr) ? safe_log(prior[(shared_model ? 0 : (size_t)cc.seq * Dr) + j]) : -INFINITY;
        else v0 = vin[(size_t)chunk * D + j];
    }
    if (h == 0) vbuf[cl * D + j] = v0;
    {
        const float m = wave_max(v0);
        if (lane == 0) wmaxs[cl * C::VWPC + wv] = m;
    }
    __syncthreads();
    // level the chunk starts from: 0 for the log prior (nothing is removed at the first step), else the
    // carry's maximum (0 up to rounding, since the carry kernel shifts it there)
    float start = 0.0f;
    if (!first_chunk) {
        start = wmaxs[cl * C::VWPC];
#pragma unroll
        for (int w = 1; w < C::VWPC; ++w) start = fmaxf(start, wmaxs[cl * C::VWPC + w]);
        start = (start == -INFINITY) ? 0.0f : start;
    }
    __syncthreads();
    // offset applied one step late
    float off = start;
    double osum = 0.0;
    int cur = 0;
    float xn = -INFINITY;
    if (cc.nsteps > 0 && j < Dr) xn = lseq[(size_t)cc.t0 * Dr + j];
    float vlast = v0;
    for (int s = 0; s < Lc; ++s) {
        const bool active = s < cc.nsteps;
        const float x = xn;
        if (s + 1 < cc.nsteps && j < Dr) xn = lseq[(size_t)(cc.t0 + s + 1) * Dr + j];
        const float* vc = vbuf + (cur * C::VCPW + cl) * D;
        float* vn = vbuf + ((cur ^ 1) * C::VCPW + cl) * D;
        float* wn = wmaxs + ((cur ^ 1) * C::VCPW + cl) * C::VWPC;
        float gval = -INFINITY;
        if (active) {
            int arg = j;
            if (cc.t0 + s == 0) {
                gval = vc[j] + x;   // V_1 = log prior + ll_1
            } else {
                // D <= 32: groups of four candidates are ranked independently and merged in index order (short
                // dependent chains); strict comparisons throughout, so the lowest index wins ties
                float best = -INFINITY;
                int bi = h * C::RPP;
#pragma unroll
                for (int r4 = 0; r4 < C::RPP; r4 += 4) {
                    const float4 v4 = *reinterpret_cast<const float4*>(vc + h * C::RPP + r4);
                    const float c0 = v4.x + lareg[r4], c1 = v4.y + lareg[r4 + 1];
                    const float c2 = v4.z + lareg[r4 + 2], c3 = v4.w + lareg[r4 + 3];
                    if constexpr (C::VWPC == 1) {
                        float ba = c0, bb = c2;
                        int ia = h * C::RPP + r4, ib = h * C::RPP + r4 + 2;
                        if (c1 > ba) { ba = c1; ia = h * C::RPP + r4 + 1; }
                        if (c3 > bb) { bb = c3; ib = h * C::RPP + r4 + 3; }
                        if (bb > ba) { ba = bb; ia = ib; }
                        if (r4 == 0 || ba > best) { best = ba; bi = ia; }
                    } else {   // long rows (D >= 64): one chain, fewer instructions (measured faster there)
                        if (c0 > best) { best = c0; bi = h * C::RPP + r4; }
                        if (c1 > best) { best = c1; bi = h * C::RPP + r4 + 1; }
                        if (c2 > best) { best = c2; bi = h * C::RPP + r4 + 2; }
                        if (c3 > best) { best = c3; bi = h * C::RPP + r4 + 3; }
                    }
                }
                // combine the parts: a higher part wins only if strictly better
#pragma unroll
                for (int d = C::CPWV; d < 64; d <<= 1) {
                    const float ob = __shfl_xor(best, d, 64);
                    const int oi = __shfl_xor(bi, d, 64);
                    const bool take = (ob > best) || (ob == best && oi < bi);
                    best = take ? ob : best;
                    bi = take ? oi : bi;
                }
                gval = best + (x - off);
                arg = bi;
            }
            if (h == 0) {
                vn[j] = gval;
                bpl[(size_t)s * D + j] = (uint8_t)arg;
            }
            const float mw = wave_max(gval);
            if (lane == 0) wn[wv] = mw;
        }
        if constexpr (C::VWPC > 1) lds_barrier();   // a chunk of D <= 32 is one wave: its LDS traffic is ordered as issued
        else wave_lds_sync();
        if (active) {
            float m = wn[0];
#pragma unroll
            for (int w = 1; w < C::VWPC; ++w) m = fmaxf(m, wn[w]);
            // V_s as stored equals the true V_s minus the offsets removed so far; its max is the next offset
            osum += (double)((cc.t0 + s == 0) ? 0.0f : off);
            off = (m == -INFINITY) ? 0.0f : m;
            vlast = gval;
        }
        cur ^= 1;
    }
    // chunk-local growth of max_j V: offsets removed plus what is left in the last stored vector
    const bool live = cc.nsteps > 0;
    if (live && lane == 0 && wv == 0) part[chunk] = osum + (double)off - (double)start;
    __syncthreads();
    // copy the chunk's back-pointers to the workspace (coalesced)
    if (live) {
        uint8_t* dst = bp + ((size_t)cc.seq * T + cc.t0) * D;
        const int nbytes = cc.nsteps * D;
        const int tic = threadIdx.x - cl * C::VWPC * 64;
        for (int idx = tic * 4; idx < nbytes; idx += C::VWPC * 64 * 4)
            *reinterpret_cast<uint32_t*>(dst + idx) = *reinterpret_cast<const uint32_t*>(bpl + idx);
    }
    // x*_T in the sequence's last chunk: argmax over j of the last V, lowest index on ties
    const bool last_chunk = live && (chunk % cps) == cps - 1;
    int xs = 0;
    if (last_chunk) {
        float bv = (h == 0) ? vlast : -INFINITY;
        int bi = j;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const float ob = __shfl_xor(bv, d, 64);
            const int oi = __shfl_xor(bi, d, 64);
            const bool take = (ob > bv) || (ob == bv && oi < bi);
            bv = take ? ob : bv;
            bi = take ? oi : bi;
        }
        if (lane == 0) { red_v[cl * 4 + wv] = bv; red_i[cl * 4 + wv] = bi; }
    }
    __syncthreads();
    if (last_chunk) {
        float bv = red_v[cl * 4];
        xs = red_i[cl * 4];
#pragma unroll
        for (int w = 1; w < C::VWPC; ++w) {
            const float ob = red_v[cl * 4 + w];
            const int oi = red_i[cl * 4 + w];
            if (ob > bv || (ob == bv && oi < xs)) { bv = ob; xs = oi; }
        }
        if (lane == 0 && wv == 0) xstar[cc.seq] = xs;
    }
    // chunk map: hmap(j) = state at the step before the chunk given state j at its last step
    if (live && h == 0) {
        int hm = j;
        for (int s = cc.nsteps - 1; s >= 0; --s) hm = bpl[(size_t)s * D + hm];
        if (last_chunk) {
            // every state maps to the image of x*_T
            int hx = xs;
            for (int s = cc.nsteps - 1; s >= 0; --s) hx = bpl[(size_t)s * D + hx];
            hm = hx;
        }
        cmap[(size_t)chunk * D + j] = (uint8_t)hm;
    }
}

// t[r] = V((l - r) mod 16) + la[r] for the sixteen rotations of a DPP row
template <int R>
HMM_DEV void row_candidates(float v, const float (&la)[16], float (&t)[16]) {
    if constexpr (R < 16) {
        t[R] = row_rotate<R>(v) + la[R];
        row_candidates<R + 1>(v, la, t);
    }
}

// ---------------------------------------------------------------------------------------------
// The same for D = 16 with one chunk per DPP row of 16 lanes (sixteen chunks per workgroup) and no
// barrier: lane l holds V(l) of its chunk, the candidates V(k) + log A(k, l) with k = (l - r) mod 16
// arrive as the row's vector rotated by r lanes (an operand modifier of the add), their maximum is a
// chain of three-way maxima, and the back-pointer is the lowest k among the candidates that equal it.
// The row's maximum (the next step's offset) is four rotate-and-max steps off the critical path.
// Log-likelihoods are prefetched PFD steps ahead through a running pointer that stops at the
// chunk's last step.
template <int D>
__global__ __launch_bounds__(256) void lv_forward_row_kernel(const float* __restrict__ prior, const float* __restrict__ A,
                                                             const float* __restrict__ ll, long long T, int Dr, int Lc,
                                                             int cps, long long nchunks, int shared_model,
                                                             const float* __restrict__ vin, uint8_t* __restrict__ bp,
                                                             uint8_t* __restrict__ cmap, int* __restrict__ xstar,
                                                             double* __restrict__ part) {
    static_assert(D == 16, "one DPP row per chunk");
    constexpr int PFD = 8;
    extern __shared__ __align__(16) unsigned char dyn_lds[];   // back-pointers: [16 chunks][Lc][16]
    const int l = threadIdx.x & 15, cl = threadIdx.x >> 4;
    const long long chunk = (long long)blockIdx.x * 16 + cl;
    const ChunkCoord cc = chunk_coord(chunk, nchunks, cps, T, Lc);
    const float* Am = A + (shared_model ? 0 : (size_t)cc.seq * Dr * Dr);
    uint8_t* bpl = dyn_lds + (size_t)cl * Lc * D;
    float la[16];
    unsigned kr[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int k = (l - r) & 15;
        float v = (k == l) ? 0.0f : -INFINITY;
        if (k < Dr && l < Dr) v = safe_log(Am[(size_t)k * Dr + l]);
        la[r] = v;
        kr[r] = (unsigned)k;
    }
    const bool live = cc.nsteps > 0;
    const bool first_chunk = (chunk % cps) == 0;
    float v = -INFINITY;
    if (live) {
        if (first_chunk) v = (l < Dr) ? safe_log(prior[(shared_model ? 0 : (size_t)cc.seq * Dr) + l]) : -INFINITY;
        else v = vin[(size_t)chunk * D + l];
    }
    // level the chunk starts from: 0 for the log prior, else the carry's maximum
    float start = 0.0f;
    if (!first_chunk) {
        start = row_allmax(v);
        start = (start == -INFINITY) ? 0.0f : start;
    }
    float off = start;
    double osum = 0.0;
    const float* lp = ll + ((size_t)cc.seq * T + cc.t0) * Dr + (l < Dr ? l : 0);
    int fetched = 0;
    float xq[PFD];
    // FULL (decided for the whole wavefront): every row's chunk has exactly Lc steps, Lc is a multiple of PFD and the
    // model is not padded -- no step is inactive, no lane idle, only a chunk's step 0 can be the sequence's first,
    // and the last PFD steps fetch nothing.
    const bool full = Dr == D && Lc % PFD == 0 && Lc >= 2 * PFD && __builtin_amdgcn_ballot_w64(cc.nsteps != Lc) == 0;
    auto run = [&](auto full_tag) {
        constexpr bool FULL = decltype(full_tag)::value;
        auto fetch = [&](float& x) {
            x = *lp;
            ++fetched;
            if (FULL || fetched < cc.nsteps) lp += Dr;
        };
#pragma unroll
        for (int p = 0; p < PFD; ++p) fetch(xq[p]);
        auto group = [&](int s0, auto do_fetch) {
#pragma unroll
            for (int p = 0; p < PFD; ++p) {
                const int s = s0 + p;
                const bool active = FULL || s < cc.nsteps;
                const float x = (FULL || l < Dr) ? xq[p] : -INFINITY;
                if constexpr (decltype(do_fetch)::value) fetch(xq[p]);
                float t[16];
                row_candidates<0>(v, la, t);
                float best = max3f(t[0], t[1], t[2]);
#pragma unroll
                for (int r = 3; r < 15; r += 2) best = max3f(best, t[r], t[r + 1]);
                best = fmaxf(best, t[15]);
                unsigned arg = 255u;
#pragma unroll
                for (int r = 0; r < 16; ++r) arg = min(arg, (t[r] == best) ? kr[r] : 255u);   // lowest state among the maximisers
                // V_1 = log prior + ll_1: no transition, no offset
                const bool seq_start = FULL ? (p == 0 && first_chunk && s0 == 0) : (cc.t0 + s == 0);
                const float gval = seq_start ? v + x : best + (x - off);
                if (active) {
                    bpl[(size_t)s * D + l] = (uint8_t)(seq_start ? (unsigned)l : arg);
                    const float m = row_allmax(gval);
                    osum += (double)(seq_start ? 0.0f : off);
                    off = (m == -INFINITY) ? 0.0f : m;
                    v = gval;
                }
            }
        };
        if constexpr (FULL) {
            for (int s0 = 0; s0 < Lc - PFD; s0 += PFD) group(s0, std::true_type{});
            group(Lc - PFD, std::false_type{});
        } else {
            for (int s0 = 0; s0 < Lc; s0 += PFD) group(s0, std::true_type{});
        }
    };
    if (full) run(std::true_type{});
    else run(std::false_type{});
    if (live && l == 0) part[chunk] = osum + (double)off - (double)start;
    wave_lds_sync();   // the chunk's back-pointers were written by its own row of lanes
    if (live) {
        uint8_t* dst = bp + ((size_t)cc.seq * T + cc.t0) * D;
        const int nbytes = cc.nsteps * D;
        for (int idx = l * 4; idx < nbytes; idx += 64)
            *reinterpret_cast<uint32_t*>(dst + idx) = *reinterpret_cast<const uint32_t*>(bpl + idx);
    }
    // x*_T in the sequence's last chunk: argmax over the row, lowest index on ties
    const bool last_chunk = live && (chunk % cps) == cps - 1;
    float bv = v;
    int bi = l;
#pragma unroll
    for (int d = 1; d < 16; d <<= 1) {
        const float ob = __shfl_xor(bv, d, 64);
        const int oi = __shfl_xor(bi, d, 64);
        const bool take = (ob > bv) || (ob == bv && oi < bi);
        bv = take ? ob : bv;
        bi = take ? oi : bi;
    }
    if (last_chunk && l == 0) xstar[cc.seq] = bi;
    // chunk map: state at the step before the chunk given state l at its last step (in the last chunk every
    // state maps to the image of x*_T)
    if (live) {
        int hm = last_chunk ? bi : l;
        for (int s = cc.nsteps - 1; s >= 0; --s) hm = bpl[(size_t)s * D + hm];
        cmap[(size_t)chunk * D + l] = (uint8_t)hm;
    }
}

// ---------------------------------------------------------------------------------------------
// State at every chunk's last step (chunk maps applied right to left from x*_T) and the
// sequence's log-probability.  One workgroup per sequence; the maps are chased through LDS.
template <int D>
__global__ __launch_bounds__(256) void lv_suffix_kernel(const uint8_t* __restrict__ cmap, const int* __restrict__ xstar,
                                                        int cps, int* __restrict__ xend,
                                                        const double* __restrict__ part, int nparts,
                                                        double* __restrict__ logprob) {
    constexpr int PIECE = 128;                       // chunk maps staged per round
    __shared__ __align__(16) uint8_t maps[PIECE * D];
    __shared__ double sh[256];
    __shared__ int xcur;
    const int seq = blockIdx.x;
    if (threadIdx.x == 0) xcur = xstar[seq];
    for (int hi = cps; hi > 0; hi -= PIECE) {
        const int lo = hi > PIECE ? hi - PIECE : 0;
        const int n = (hi - lo) * D;
        const uint8_t* src = cmap + ((size_t)seq * cps + lo) * D;
        for (int idx = threadIdx.x * 4; idx < n; idx += 256 * 4)
            *reinterpret_cast<uint32_t*>(maps + idx) = *reinterpret_cast<const uint32_t*>(src + idx);
        __syncthreads();
        if (threadIdx.x == 0) {
            int x = xcur;
            for (int c = hi - 1; c >= lo; --c) {
                xend[(size_t)seq * cps + c] = x;
                x = maps[(c - lo) * D + x];
            }
            xcur = x;
        }
        __syncthreads();
    }
    double acc = 0.0;
    for (int c = threadIdx.x; c < nparts; c += 256) acc += part[(size_t)seq * nparts + c];
    sh[threadIdx.x] = acc;
    __syncthreads();
    for (int d = 128; d >= 1; d >>= 1) {
        if ((int)threadIdx.x < d) sh[threadIdx.x] += sh[threadIdx.x + d];
        __syncthreads();
    }
    if (threadIdx.x == 0) logprob[seq] = sh[0];
}

// ---------------------------------------------------------------------------------------------
// Second level of the reversed scan over chunk maps for long sequences: the composed map of every
// group of g consecutive chunks (state at the group's last step -> state before its first chunk), so
// that lv_suffix walks groups instead of chunks, and then, for all groups in parallel, the walk
// through each group's own chunks from the state lv_suffix found at its end.  The group's maps are
// staged in LDS: a chain of dependent byte look-ups.
template <int D>
__global__ __launch_bounds__(128) void lv_group_maps_kernel(const uint8_t* __restrict__ cmap, int cps, int g, int G,
                                                            uint8_t* __restrict__ gmap) {
    extern __shared__ __align__(16) unsigned char dyn_lds[];
    const int seq = blockIdx.x / G, grp = blockIdx.x % G;
    const int c0 = grp * g, c1 = min(cps, c0 + g);
    const uint8_t* src = cmap + ((size_t)seq * cps + c0) * D;
    const int n = (c1 - c0) * D;
    for (int idx = threadIdx.x * 4; idx < n; idx += 128 * 4)
        *reinterpret_cast<uint32_t*>(dyn_lds + idx) = *reinterpret_cast<const uint32_t*>(src + idx);
    __syncthreads();
    if ((int)threadIdx.x < D) {
        int x = threadIdx.x;
        for (int c = c1 - 1; c >= c0; --c) x = dyn_lds[(c - c0) * D + x];
        gmap[((size_t)seq * G + grp) * D + threadIdx.x] = (uint8_t)x;
    }
}

template <int D>
__global__ __launch_bounds__(128) void lv_group_chase_kernel(const uint8_t* __restrict__ cmap, const int* __restrict__ xg,
                                                             int cps, int g, int G, int* __restrict__ xend) {
    extern __shared__ __align__(16) unsigned char dyn_lds[];
    const int seq = blockIdx.x / G, grp = blockIdx.x % G;
    const int c0 = grp * g, c1 = min(cps, c0 + g);
    const uint8_t* src = cmap + ((size_t)seq * cps + c0) * D;
    const int n = (c1 - c0) * D;
    for (int idx = threadIdx.x * 4; idx < n; idx += 128 * 4)
        *reinterpret_cast<uint32_t*>(dyn_lds + idx) = *reinterpret_cast<const uint32_t*>(src + idx);
    __syncthreads();
    if (threadIdx.x == 0) {
        int x = xg[(size_t)seq * G + grp];
        for (int c = c1 - 1; c >= c0; --c) {
            xend[(size_t)seq * cps + c] = x;
            x = dyn_lds[(c - c0) * D + x];
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Back-pointer walk inside each chunk from the state at its last step; coalesced path write.  One wave
// per chunk (the walk itself is a chain of dependent LDS look-ups by one lane; several chunks per
// workgroup keep more of those chains in flight per compute unit), cpw chunks per workgroup.
template <int D>
__global__ __launch_bounds__(256) void lv_path_kernel(long long T, int Lc, int cps, long long nchunks, int cpw,
                                                      const uint8_t* __restrict__ bp, const int* __restrict__ xend,
                                                      int32_t* __restrict__ path) {
    extern __shared__ __align__(16) unsigned char dyn_lds[];   // per chunk: [Lc*D] back-pointers, then [Lc] path (int32)
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    if (wave >= cpw) return;                                   // uniform over the wave; no workgroup barrier below
    const long long chunk = (long long)blockIdx.x * cpw + wave;
    const ChunkCoord cc = chunk_coord(chunk, nchunks, cps, T, Lc);
    if (cc.nsteps == 0) return;
    unsigned char* base = dyn_lds + (size_t)wave * ((size_t)Lc * D + (size_t)Lc * sizeof(int32_t));
    uint8_t* bpl = base;
    int32_t* pl = reinterpret_cast<int32_t*>(base + (size_t)Lc * D);
    const uint8_t* src = bp + ((size_t)cc.seq * T + cc.t0) * D;
    const int nbytes = cc.nsteps * D;
    // 16-byte pieces, four loads in flight per lane (the wave copies its chunk alone)
    for (int idx = lane * 16; idx < nbytes; idx += 4 * 64 * 16) {
        uint4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int o = idx + u * 64 * 16;
            v[u] = *reinterpret_cast<const uint4*>(src + (o < nbytes ? o : idx));
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int o = idx + u * 64 * 16;
            if (o < nbytes) *reinterpret_cast<uint4*>(bpl + o) = v[u];
        }
    }
    wave_lds_sync();
    if (lane == 0) {
        int x = xend[chunk];
        for (int s = cc.nsteps - 1; s >= 0; --s) {
            pl[s] = x;
            x = bpl[(size_t)s * D + x];
        }
    }
    wave_lds_sync();
    int32_t* dst = path + (size_t)cc.seq * T + cc.t0;
    for (int s = lane; s < cc.nsteps; s += 64) dst[s] = pl[s];
}

// =============================================================================================
// The paper's parallel max-product algorithm as printed (Algorithm 5): maximum forward and backward
// potentials (the lemma of Sec. IV-C) inside the chunks, then Theorem 4's per-step combination.
// =============================================================================================

// First half of the grid: psi~^f_k inside each chunk from the forward carry, every step stored
// shifted to max 0, plus the chunk-local growth of the log of the best joint weight.  Second half:
// psi~^b_k inside each chunk from the backward carry, stored with an arbitrary shift per step (the
// combination removes it).  Lane = (component inside the wave, part h of the max), log A in
// registers (a column for the forward, a row for the backward recursion), the vector through
// double-buffered LDS, its maximum removed one step late: one barrier per step.
template <int D>
__global__ __launch_bounds__(256) void lm_apply_kernel(const float* __restrict__ prior, const float* __restrict__ A,
                                                       const float* __restrict__ ll, long long T, int Dr, int Lc,
                                                       int cps, long long nchunks, int shared_model,
                                                       const float* __restrict__ vin, const float* __restrict__ bout,
                                                       float* __restrict__ F, float* __restrict__ Bv,
                                                       double* __restrict__ part, int half) {
    using C = LargeCfg<D>;
    __shared__ __align__(16) float vbuf[2 * C::VCPW * D];
    __shared__ float wmaxs[2 * C::VCPW * C::VWPC];
    const bool backward = (int)blockIdx.x >= half;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int cl = wave / C::VWPC, wv = wave % C::VWPC;
    const int jl = lane % C::CPWV, h = lane / C::CPWV;
    const int j = C::CPWV * wv + jl;                      // component owned (replicated over the parts h)
    const long long chunk = (long long)(backward ? blockIdx.x - half : blockIdx.x) * C::VCPW + cl;
    const ChunkCoord cc = chunk_coord(chunk, nchunks, cps, T, Lc);
    const float* Am = A + (shared_model ? 0 : (size_t)cc.seq * Dr * Dr);
    float lareg[C::RPP];   // forward: log A(i, j) over the part's i; backward: log A(j, i') over the part's i'
#pragma unroll
    for (int r = 0; r < C::RPP; ++r) {
        const int i = h * C::RPP + r;
        float v = (i == j) ? 0.0f : -INFINITY;
        if (i < Dr && j < Dr) v = safe_log(backward ? Am[(size_t)j * Dr + i] : Am[(size_t)i * Dr + j]);
        lareg[r] = v;
    }
    const float* lseq = ll + (size_t)cc.seq * T * Dr;
    float* oseq = (backward ? Bv : F) + (size_t)cc.seq * T * Dr;
    const bool first_chunk = (chunk % cps) == 0;
    auto block_max = [&](const float* w) {
        float m = w[0];
#pragma unroll
        for (int q = 1; q < C::VWPC; ++q) m = fmaxf(m, w[q]);
        return (m == -INFINITY) ? 0.0f : m;
    };
    auto part_max = [&](float best) {   // combine the parts h of a component
#pragma unroll
        for (int d = C::CPWV; d < 64; d <<= 1) best = fmaxf(best, __shfl_xor(best, d, 64));
        return best;
    };
    if (!backward) {
        float v0 = -INFINITY;
        if (cc.nsteps > 0) {
            if (first_chunk) v0 = (j < Dr) ? safe_log(prior[(shared_model ? 0 : (size_t)cc.seq * Dr) + j]) : -INFINITY;
            else v0 = vin[(size_t)chunk * D + j];
        }
        if (h == 0) vbuf[cl * D + j] = v0;
        {
            const float m = wave_max(v0);
            if (lane == 0) wmaxs[cl * C::VWPC + wv] = m;
        }
        __syncthreads();
        // level the chunk starts from: 0 for the log prior (used as given), else the carry's maximum
        const float start = first_chunk ? 0.0f : block_max(wmaxs + cl * C::VWPC);
        __syncthreads();
        float off = start;
        double osum = 0.0;
        int cur = 0;
        float xn = -INFINITY;
        if (cc.nsteps > 0 && j < Dr) xn = lseq[(size_t)cc.t0 * Dr + j];
        for (int s = 0; s < Lc; ++s) {
            const bool active = s < cc.nsteps;
            const float x = xn;
            if (s + 1 < cc.nsteps && j < Dr) xn = lseq[(size_t)(cc.t0 + s + 1) * Dr + j];
            const float* vc = vbuf + (cur * C::VCPW + cl) * D;
            float* vn = vbuf + ((cur ^ 1) * C::VCPW + cl) * D;
            float* wn = wmaxs + ((cur ^ 1) * C::VCPW + cl) * C::VWPC;
            float gval = -INFINITY;
            if (active) {
                if (cc.t0 + s == 0) {
                    gval = vc[j] + x;   // psi~^f_1 = log prior + ll_1
                } else {
                    float b0 = -INFINITY, b1 = -INFINITY;
#pragma unroll
                    for (int r4 = 0; r4 < C::RPP; r4 += 4) {
                        const float4 v4 = *reinterpret_cast<const float4*>(vc + h * C::RPP + r4);
                        b0 = max3f(b0, v4.x + lareg[r4], v4.y + lareg[r4 + 1]);
                        b1 = max3f(b1, v4.z + lareg[r4 + 2], v4.w + lareg[r4 + 3]);
                    }
                    gval = part_max(fmaxf(b0, b1)) + (x - off);
                }
                if (h == 0) vn[j] = gval;
                const float mw = wave_max(gval);
                if (lane == 0) wn[wv] = mw;
            }
            lds_barrier();
            if (active) {
                const float m = block_max(wn);
                if (h == 0 && j < Dr) oseq[(size_t)(cc.t0 + s) * Dr + j] = gval - m;
                osum += (double)((cc.t0 + s == 0) ? 0.0f : off);
                off = m;
            }
            cur ^= 1;
        }
        if (cc.nsteps > 0 && lane == 0 && wv == 0) part[chunk] = osum + (double)off - (double)start;
    } else {
        // u = psi~^b at the current step, component j, shifted by the previous step's maximum
        // without carries (sequences of one chunk) the backward potential at the last step is the operator's unit
        float u = -INFINITY;
        if (cc.nsteps > 0) u = bout != nullptr ? bout[(size_t)chunk * D + j] : (j < Dr ? 0.0f : -INFINITY);
        int cur = 0;
        float xn = -INFINITY;
        if (cc.nsteps > 0 && j < Dr) xn = lseq[(size_t)(cc.t0 + cc.nsteps - 1) * Dr + j];
        for (int sp = 0; sp < Lc; ++sp) {
            const int s = Lc - 1 - sp;
            const bool active = s < cc.nsteps;
            float* vn = vbuf + ((cur ^ 1) * C::VCPW + cl) * D;
            float* wn = wmaxs + ((cur ^ 1) * C::VCPW + cl) * C::VWPC;
            if (active) {
                const float x = xn;
                if (s >= 1 && j < Dr) xn = lseq[(size_t)(cc.t0 + s - 1) * Dr + j];
                if (h == 0) {
                    if (j < Dr) oseq[(size_t)(cc.t0 + s) * Dr + j] = u;
                    vn[j] = x + u;          // log psi_{s} 's emission part + psi~^b_s: what step s-1 maximises over
                }
                const float mw = wave_max(u);
                if (lane == 0) wn[wv] = mw;
            }
            lds_barrier();
            if (active && s > 0) {
                const float m = block_max(wn);
                float b0 = -INFINITY, b1 = -INFINITY;
#pragma unroll
                for (int r4 = 0; r4 < C::RPP; r4 += 4) {
                    const float4 t4 = *reinterpret_cast<const float4*>(vn + h * C::RPP + r4);
                    b0 = max3f(b0, t4.x + lareg[r4], t4.y + lareg[r4 + 1]);
                    b1 = max3f(b1, t4.z + lareg[r4 + 2], t4.w + lareg[r4 + 3]);
                }
                u = part_max(fmaxf(b0, b1)) - m;
            }
            cur ^= 1;
        }
    }
}

// The same for D <= 32 with one chunk per DPP row of 16 lanes (sixteen chunks per workgroup), no LDS and no
// barrier: lane l holds components 16 q + l of the vector, the candidates of the maximum arrive as the
// row's vector rotated by r lanes (an operand modifier of the add) against constants
// la[qd][16 qs + r] = log A(16 qs + (l - r) mod 16, 16 qd + l)   (forward; transposed for the backward pass),
// and the row's maximum takes four rotate-and-max steps.  Log-likelihoods are prefetched PFD steps ahead.
// FUSED (enough chunks to fill the machine with one row each): a row runs the forward pass of its chunk,
// which leaves log psi~^f in F, then the backward pass, which reads it back (every lane the values it stored
// itself) and writes Theorem 4's combination -- max-marginals and their lowest maximiser -- directly.
// Otherwise the two passes of a chunk run in different workgroups (first half of the grid forward, second
// half backward, writing log psi~^b) and lm_combine follows.
template <int D, bool BACKWARD, bool FUSED>
HMM_DEV void lm_row_pass(const float* __restrict__ Am, const float* __restrict__ lseq, const ChunkCoord& cc, int Dr, int Lc,
                         bool first_chunk, const float (&start_v)[D / 16], float* fseq, float* __restrict__ gseq,
                         int32_t* __restrict__ pseq, double* part_out) {
    constexpr int NQ = D / 16;
    constexpr int PFD = 8;
    const int l = threadIdx.x & 15;
    float la[NQ][D];
#pragma unroll
    for (int qd = 0; qd < NQ; ++qd)
#pragma unroll
        for (int qs = 0; qs < NQ; ++qs)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int src = 16 * qs + ((l - r) & 15), dst = 16 * qd + l;
                const int i = BACKWARD ? dst : src, j = BACKWARD ? src : dst;
                float v = (i == j) ? 0.0f : -INFINITY;
                if (i < Dr && j < Dr) v = safe_log(Am[(size_t)i * Dr + j]);
                la[qd][16 * qs + r] = v;
            }
    const bool live = cc.nsteps > 0;
    bool have[NQ];
    int col[NQ];
#pragma unroll
    for (int q = 0; q < NQ; ++q) { have[q] = 16 * q + l < Dr; col[q] = have[q] ? 16 * q + l : 0; }
    const long long s_first = BACKWARD ? (long long)cc.nsteps - 1 : 0;
    const long long stride = BACKWARD ? -(long long)Dr : (long long)Dr;
    const long long at = cc.t0 + (live ? s_first : 0);
    const float* lp = lseq + (size_t)at * Dr;
    const float* fp = fseq + (size_t)at * Dr;
    float* op = (BACKWARD ? gseq : fseq) + (size_t)at * Dr;
    int32_t* pp = pseq ? pseq + at : nullptr;
    int fetched = 0;
    float xq[PFD][NQ], fq[PFD][NQ];
    auto fetch = [&](float (&x)[NQ], float (&f)[NQ]) {
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            x[q] = lp[col[q]];
            if constexpr (BACKWARD && FUSED) f[q] = fp[col[q]];
        }
        ++fetched;
        if (fetched < cc.nsteps) {
            lp += stride;
            fp += stride;
        }
    };
    auto row_max_of = [&](const float (&v)[NQ]) {
        float m = v[0];
#pragma unroll
        for (int q = 1; q < NQ; ++q) m = fmaxf(m, v[q]);
        m = row_allmax(m);
        return (m == -INFINITY) ? 0.0f : m;
    };
    float v[NQ];
#pragma unroll
    for (int q = 0; q < NQ; ++q) v[q] = start_v[q];
#pragma unroll
    for (int p = 0; p < PFD; ++p) fetch(xq[p], fq[p]);
    if constexpr (!BACKWARD) {
        // level the chunk starts from: 0 for the log prior (used as given), else the carry's maximum
        const float start = first_chunk ? 0.0f : row_max_of(v);
        float off = start;
        double osum = 0.0;
        for (int s0 = 0; s0 < Lc; s0 += PFD) {
#pragma unroll
            for (int p = 0; p < PFD; ++p) {
                const int s = s0 + p;
                const bool active = s < cc.nsteps;
                float x[NQ];
#pragma unroll
                for (int q = 0; q < NQ; ++q) x[q] = have[q] ? xq[p][q] : -INFINITY;
                fetch(xq[p], fq[p]);
                const bool seq_start = (cc.t0 + s == 0);   // psi~^f_1 = log prior + ll_1
                float g[NQ];
#pragma unroll
                for (int qd = 0; qd < NQ; ++qd) {
                    float best = -INFINITY;
                    systolic_terms<D, 0, 0>(v, la[qd], best);
                    g[qd] = seq_start ? v[qd] + x[qd] : best + (x[qd] - off);
                }
                if (active) {
                    const float m = row_max_of(g);
#pragma unroll
                    for (int q = 0; q < NQ; ++q) {
                        if (have[q]) op[16 * q + l] = g[q] - m;
                        v[q] = g[q];
                    }
                    op += stride;
                    osum += (double)(seq_start ? 0.0f : off);
                    off = m;
                }
            }
        }
        if (live && l == 0) *part_out = osum + (double)off - (double)start;
    } else {
        // v = psi~^b at the current step, shifted by the previous step's maximum
        for (int s0 = 0; s0 < Lc; s0 += PFD) {
#pragma unroll
            for (int p = 0; p < PFD; ++p) {
                const int pos = s0 + p;
                const bool active = pos < cc.nsteps;
                const int s = cc.nsteps - 1 - pos;
                float t[NQ], gm[NQ];
#pragma unroll
                for (int q = 0; q < NQ; ++q) {
                    t[q] = (have[q] ? xq[p][q] : -INFINITY) + v[q];   // emission part of psi_s + psi~^b_s
                    gm[q] = (FUSED && have[q]) ? fq[p][q] + v[q] : -INFINITY;   // Theorem 4: log psi~^f_s + log psi~^b_s
                }
                fetch(xq[p], fq[p]);
                float nv[NQ];
                const float m = row_max_of(v);
#pragma unroll
                for (int qd = 0; qd < NQ; ++qd) {
                    float best = -INFINITY;
                    systolic_terms<D, 0, 0>(t, la[qd], best);
                    nv[qd] = best - m;
                }
                float gbest = 0.0f, garg = 0.0f;
                if constexpr (FUSED) {
                    gbest = gm[0];
#pragma unroll
                    for (int q = 1; q < NQ; ++q) gbest = fmaxf(gbest, gm[q]);
                    gbest = row_allmax(gbest);
                    garg = 1.0e9f;                       // lowest state reaching the maximum (states are exact in float)
#pragma unroll
                    for (int q = NQ - 1; q >= 0; --q)
                        if (have[q] && gm[q] == gbest) garg = (float)(16 * q + l);
                    garg = row_allmin(garg);
                }
                if (active) {
                    const float shift = (gbest == -INFINITY) ? 0.0f : gbest;
#pragma unroll
                    for (int q = 0; q < NQ; ++q) {
                        if (have[q]) op[16 * q + l] = FUSED ? gm[q] - shift : v[q];
                        if (s > 0) v[q] = nv[q];
                    }
                    op += stride;
                    if constexpr (FUSED) {
                        if (pp != nullptr) {
                            if (l == 0) *pp = (int32_t)garg;
                            --pp;
                        }
                    }
                }
            }
        }
    }
}

// out: the max-marginals (FUSED; path: their maximisers, may be null) or log psi~^b; half: workgroups per direction
// (not FUSED)
template <int D, bool FUSED>
__global__ __launch_bounds__(256) void lm_apply_row_kernel(const float* __restrict__ prior, const float* __restrict__ A,
                                                           const float* __restrict__ ll, long long T, int Dr, int Lc,
                                                           int cps, long long nchunks, int shared_model,
                                                           const float* __restrict__ vin, const float* __restrict__ bout,
                                                           float* F, float* __restrict__ out,
                                                           int32_t* __restrict__ path, double* __restrict__ part,
                                                           int half) {
    static_assert(D == 16 || D == 32, "one DPP row per chunk");
    constexpr int NQ = D / 16;
    const bool backward = !FUSED && (int)blockIdx.x >= half;
    const int l = threadIdx.x & 15;
    const long long chunk = (long long)(backward ? blockIdx.x - half : blockIdx.x) * 16 + (threadIdx.x >> 4);
    const ChunkCoord cc = chunk_coord(chunk, nchunks, cps, T, Lc);
    const float* Am = A + (shared_model ? 0 : (size_t)cc.seq * Dr * Dr);
    const float* lseq = ll + (size_t)cc.seq * T * Dr;
    float* fseq = F + (size_t)cc.seq * T * Dr;
    float* gseq = out + (size_t)cc.seq * T * Dr;
    int32_t* pseq = (FUSED && path != nullptr) ? path + (size_t)cc.seq * T : nullptr;
    const bool live = cc.nsteps > 0;
    const bool first_chunk = (chunk % cps) == 0;
    float vf[NQ], vb[NQ];
#pragma unroll
    for (int q = 0; q < NQ; ++q) {
        const int j = 16 * q + l;
        vf[q] = vb[q] = -INFINITY;
        if (live) {
            if (first_chunk) vf[q] = (j < Dr) ? safe_log(prior[(shared_model ? 0 : (size_t)cc.seq * Dr) + j]) : -INFINITY;
            else vf[q] = vin[(size_t)chunk * D + j];
            vb[q] = bout != nullptr ? bout[(size_t)chunk * D + j] : (j < Dr ? 0.0f : -INFINITY);   // one chunk per sequence: the unit
        }
    }
    if (!backward) lm_row_pass<D, false, FUSED>(Am, lseq, cc, Dr, Lc, first_chunk, vf, fseq, gseq, pseq, part + chunk);
    if (FUSED || backward) lm_row_pass<D, true, FUSED>(Am, lseq, cc, Dr, Lc, first_chunk, vb, fseq, gseq, pseq, nullptr);
}

// Theorem 4: max-marginal log psi~^f_k + log psi~^b_k, shifted so that the step's largest entry is 0,
// and its maximiser (lowest state on ties).  A power-of-two group of lanes per step; a wave takes
// COMBINE_UNROLL groups of steps with all loads issued first (16-byte accesses when D is a multiple of four).
constexpr int COMBINE_UNROLL = 4;

__global__ __launch_bounds__(256) void lm_combine_kernel(const float* __restrict__ F, const float* __restrict__ Bv,
                                                         long long rows, int Dr, float* __restrict__ mm,
                                                         int32_t* __restrict__ path) {
    const int lpr = (Dr + 3) / 4;                  // lanes per step
    int width = 1;
    while (width < lpr) width <<= 1;
    const int rows_per_wave = 64 / width;
    const int lane = threadIdx.x & 63;
    const long long wave = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int sub = lane % width;
    const long long row0 = wave * (COMBINE_UNROLL * rows_per_wave) + lane / width;
    float g[COMBINE_UNROLL][4];
    bool live[COMBINE_UNROLL];
    const bool vec = (Dr & 3) == 0;
#pragma unroll
    for (int u = 0; u < COMBINE_UNROLL; ++u) {
        const long long row = row0 + u * rows_per_wave;
        live[u] = row < rows && sub < lpr;
#pragma unroll
        for (int q = 0; q < 4; ++q) g[u][q] = -INFINITY;
        if (live[u]) {
            if (vec) {
                const v4f f = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(F + row * Dr + 4 * sub));
                const v4f b = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(Bv + row * Dr + 4 * sub));
                g[u][0] = f.x + b.x; g[u][1] = f.y + b.y; g[u][2] = f.z + b.z; g[u][3] = f.w + b.w;
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int j = 4 * sub + q;
                    if (j < Dr) g[u][q] = F[row * Dr + j] + Bv[row * Dr + j];
                }
            }
        }
    }
#pragma unroll
    for (int u = 0; u < COMBINE_UNROLL; ++u) {
        const long long row = row0 + u * rows_per_wave;
        float best = g[u][0];
        int arg = 4 * sub;
#pragma unroll
        for (int q = 1; q < 4; ++q)
            if (g[u][q] > best) { best = g[u][q]; arg = 4 * sub + q; }
        for (int d = 1; d < width; d <<= 1) {
            const float ob = __shfl_xor(best, d, 64);
            const int oi = __shfl_xor(arg, d, 64);
            const bool take = (ob > best) || (ob == best && oi < arg);
            best = take ? ob : best;
            arg = take ? oi : arg;
        }
        if (live[u]) {
            const float m = (best == -INFINITY) ? 0.0f : best;
            if (vec) {
                const v4f out = {g[u][0] - m, g[u][1] - m, g[u][2] - m, g[u][3] - m};
                __builtin_nontemporal_store(out, reinterpret_cast<v4f*>(mm + row * Dr + 4 * sub));
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int j = 4 * sub + q;
                    if (j < Dr) mm[row * Dr + j] = g[u][q] - m;
                }
            }
            if (sub == 0 && path != nullptr) path[row] = arg;
        }
    }
}

// out[seq] = sum of the chunk partials of one sequence (one wave)
__global__ __launch_bounds__(64) void lm_finalize_kernel(const double* __restrict__ part, int cps,
                                                         double* __restrict__ out) {
    double acc = 0.0;
    for (int c = threadIdx.x; c < cps; c += 64) acc += part[(size_t)blockIdx.x * cps + c];
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) acc += __shfl_down(acc, d, 64);
    if (threadIdx.x == 0) out[blockIdx.x] = acc;
}

// ---------------------------------------------------------------------------------------------
// Block-wise elements (Sec. V-B) under the max-product operator: the ordered product of a block's chunk
// aggregates by a binary tree, one level per launch: out[o] = in[2o] v in[2o+1] (a copy if there is no
// right neighbour).  A workgroup forms a slab of sixteen rows of one result; lane = (column j, a share
// of the slab's rows), the slab of the left operand in LDS.  Shifting a result to maximum 0 needs all
// of its slabs, so it is left to the reader: every slab records its own maximum (tmax), and a level
// reads its operands as (value - largest slab maximum), adding what it took off to the result's offset.
// Without tmax the inputs are the chunk aggregates, which have maximum 0 already.
// `swap`: the matrices are stored transposed, so the operands trade places.
template <int D>
__global__ __launch_bounds__(256) void lv_tree_product_kernel(const float* __restrict__ in, const double* __restrict__ in_off,
                                                              const float* __restrict__ in_tmax, int n_in, int n_out,
                                                              int swap, float* __restrict__ out,
                                                              double* __restrict__ out_off, float* __restrict__ out_tmax) {
    constexpr int NT = D / 16;        // slabs per matrix
    constexpr int NRG = 256 / D;      // row groups
    constexpr int RPT = 16 / NRG;     // rows per lane
    __shared__ float xs[16 * D];
    __shared__ float red[4];
    const int tid = threadIdx.x;
    const int slab = blockIdx.x % NT;
    const int res = blockIdx.x / NT;                 // seq * n_out + o
    const int seq = res / n_out, o = res % n_out;
    const size_t ia = (size_t)seq * n_in + 2 * o;
    const bool pair = 2 * o + 1 < n_in;
    auto shift_of = [&](size_t idx) {
        if (in_tmax == nullptr) return 0.0f;
        float m = -INFINITY;
#pragma unroll
        for (int t = 0; t < NT; ++t) m = fmaxf(m, in_tmax[idx * NT + t]);
        return (m == -INFINITY) ? 0.0f : m;
    };
    const float ma = shift_of(ia), mb = pair ? shift_of(ia + 1) : 0.0f;
    const float* Ma = in + ia * D * D;
    const float* Mb = Ma + D * D;
    float* Z = out + (size_t)res * D * D;
    const int j = tid % D, rg = tid / D;
    const int i0 = 16 * slab;
    float lmax = -INFINITY;
    if (!pair) {
#pragma unroll
        for (int r = 0; r < RPT; ++r) {
            const float v = Ma[(size_t)(i0 + rg * RPT + r) * D + j] - ma;
            Z[(size_t)(i0 + rg * RPT + r) * D + j] = v;
            lmax = fmaxf(lmax, v);
        }
    } else {
        const float* X = swap ? Mb : Ma;
        const float* Y = swap ? Ma : Mb;
        for (int idx = tid; idx < 16 * D; idx += 256) xs[idx] = X[(size_t)i0 * D + idx];
        __syncthreads();
        float acc[RPT];
#pragma unroll
        for (int r = 0; r < RPT; ++r) acc[r] = -INFINITY;
#pragma unroll 4
        for (int k = 0; k < D; ++k) {
            const float y = Y[(size_t)k * D + j];
#pragma unroll
            for (int r = 0; r < RPT; ++r) acc[r] = fmaxf(acc[r], xs[(rg * RPT + r) * D + k] + y);
        }
#pragma unroll
        for (int r = 0; r < RPT; ++r) {
            const float v = acc[r] - (ma + mb);
            Z[(size_t)(i0 + rg * RPT + r) * D + j] = v;
            lmax = fmaxf(lmax, v);
        }
    }
    lmax = wave_max(lmax);
    if ((tid & 63) == 0) red[tid >> 6] = lmax;
    __syncthreads();
    if (tid == 0) {
        out_tmax[(size_t)res * NT + slab] = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        if (slab == 0 && out_off != nullptr)   // callers that only need the product's direction pass no offsets
            out_off[res] = in_off[ia] + (pair ? in_off[ia + 1] : 0.0) + (double)ma + (double)mb;
    }
}

// The block's element from its single remaining aggregate: padding dropped, largest entry 0,
// log_scale = accumulated offset (-inf if no sequence of the block has any weight).
template <int D>
__global__ __launch_bounds__(256) void lv_element_finish_kernel(const float* __restrict__ M, const double* __restrict__ off,
                                                                int Dr, int transposed, float* __restrict__ element,
                                                                double* __restrict__ log_scale) {
    __shared__ float red[4];
    const int seq = blockIdx.x, tid = threadIdx.x;
    const float* X = M + (size_t)seq * D * D;
    float lm = -INFINITY;
    for (int idx = tid; idx < Dr * Dr; idx += 256) {
        const int i = idx / Dr, j = idx - i * Dr;
        lm = fmaxf(lm, X[transposed ? (size_t)j * D + i : (size_t)i * D + j]);
    }
    lm = wave_max(lm);
    if ((tid & 63) == 0) red[tid >> 6] = lm;
    __syncthreads();
    const float m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    const float sh = (m == -INFINITY) ? 0.0f : m;
    for (int idx = tid; idx < Dr * Dr; idx += 256) {
        const int i = idx / Dr, j = idx - i * Dr;
        element[(size_t)seq * Dr * Dr + idx] = X[transposed ? (size_t)j * D + i : (size_t)i * D + j] - sh;
    }
    if (tid == 0) log_scale[seq] = (m == -INFINITY) ? -INFINITY : off[seq] + (double)m;
}

// =============================================================================================
// Host side
// =============================================================================================
static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Chunking for the max-plus path: the back-pointers of a chunk must fit in LDS (Lc * DP <= 48 KiB).
// From D = 32 the aggregate kernel runs one workgroup per chunk, all resident at once: a chunk count
// just above a multiple of the 256 compute units leaves most of them idle while a few work through one
// chunk more (713 chunks take as long as 768).  Shorten the chunks so that the count fills the last round.
static void fill_last_round(LargePlan& p, long long T, int batch) {
    if (p.DP < 32 || p.nchunks <= 256 || p.nchunks % 256 == 0) return;
    const long long target = (p.nchunks + 255) / 256 * 256;
    const long long cps_t = target / batch;
    if (cps_t < 1) return;
    long long Lc = (T + cps_t - 1) / cps_t;
    Lc = (Lc + 7) / 8 * 8;
    if (Lc >= 32 && Lc <= p.Lc) {
        p.Lc = (int)Lc;
        p.cps = (int)((T + p.Lc - 1) / p.Lc);
        p.nchunks = (long long)p.cps * batch;
    }
}

// D = 16 with chunks of at most ROW_FORWARD_MAX_LC steps (batches of sequences, which need few chunks each) runs
// the forward recursion with one chunk per DPP row, sixteen chunks' back-pointers per workgroup.
constexpr int ROW_FORWARD_MAX_LC = 192;

// Long sequences get a second scan level (SCAN2_MIN_CHUNKS chunks per sequence and more): aggregates of
// groups of g = 2^k consecutive chunks by k levels of lv_tree_product, V at the group boundaries by a walk
// over the groups, then V at every chunk by walks inside all groups at once; the reversed scan over the
// chunk maps is grouped the same way.  The sequential depth drops from chunks to about 2 sqrt(chunks), so
// below D = 128 the chunks can be as short as the smoother's (more of them, shorter in-chunk recursions).
constexpr int SCAN2_MIN_CHUNKS = 128;

struct Scan2 { bool on; int g, k, G; };

static Scan2 scan2_of(const LargePlan& p) {
    Scan2 s{false, p.cps, 0, 1};
    if (p.cps < SCAN2_MIN_CHUNKS) return s;
    s.on = true;
    int k = 1;
    while ((1 << (2 * k)) < p.cps) ++k;          // 2^k >= sqrt(chunks)
    if (k > 1 && (1 << (2 * k - 1)) >= p.cps) --k;   // nearer power of two
    s.k = k;
    s.g = 1 << k;
    s.G = (p.cps + s.g - 1) / s.g;
    return s;
}

static LargePlan viterbi_plan(int Dr, long long T, int batch) {
    LargePlan p = large_plan(Dr, T, batch);
    if (p.DP < 128) p = element_plan(Dr, T, batch);
    const int vcpw = p.DP >= 128 ? 1 : p.DP >= 64 ? 2 : 4;   // chunks sharing a workgroup in the forward kernel
    const int cap = (48 * 1024) / (p.DP * vcpw) / 16 * 16;
    if (p.Lc > cap) {
        p.Lc = cap;
        p.cps = (int)((T + p.Lc - 1) / p.Lc);
        p.nchunks = (long long)p.cps * batch;
    }
    fill_last_round(p, T, batch);
    return p;
}

struct LargeViterbiWs { size_t agg, vin, bp, cmap, xend, xstar, part, lvl[2][2], gvin, gmap, xg, total; };

static LargeViterbiWs large_viterbi_ws(int Dr, long long T, int batch) {
    const LargePlan p = viterbi_plan(Dr, T, batch);
    const size_t D = p.DP, nc = (size_t)p.nchunks, rows = (size_t)T * batch;
    LargeViterbiWs w;
    size_t o = 0;
    w.agg = o;   o = align_up(o + nc * D * D * sizeof(float), 256);
    w.vin = o;   o = align_up(o + nc * D * sizeof(float), 256);
    w.bp = o;    o = align_up(o + rows * D + 16, 256);
    w.cmap = o;  o = align_up(o + nc * D, 256);
    w.xend = o;  o = align_up(o + nc * sizeof(int), 256);
    w.xstar = o; o = align_up(o + (size_t)batch * sizeof(int), 256);
    w.part = o;  o = align_up(o + nc * sizeof(double), 256);
    const Scan2 s2 = scan2_of(p);
    size_t n = (size_t)p.cps;
    for (int l = 0; l < 2; ++l) {   // tree levels alternate between two buffers
        n = (n + 1) / 2;
        const size_t cnt = s2.on ? n * batch : 0;
        w.lvl[l][0] = o; o = align_up(o + cnt * D * D * sizeof(float), 256);
        w.lvl[l][1] = o; o = align_up(o + cnt * 8 * sizeof(float), 256);
    }
    const size_t ng = s2.on ? (size_t)s2.G * batch : 0;
    w.gvin = o;  o = align_up(o + ng * D * sizeof(float), 256);
    w.gmap = o;  o = align_up(o + ng * D, 256);
    w.xg = o;    o = align_up(o + ng * sizeof(int), 256);
    w.total = o;
    return w;
}

size_t large_d_viterbi_ws_bytes(int Dr, long long T, int batch) { return large_viterbi_ws(Dr, T, batch).total; }

template <int D>
static int large_viterbi_impl(const LargeArgs& a, int32_t* path, double* logprob_out) {
    using C = LargeCfg<D>;
    using M = MpCfg<D>;
    const LargePlan p = viterbi_plan(a.D, a.T, a.batch);
    const LargeViterbiWs w = large_viterbi_ws(a.D, a.T, a.batch);
    if (a.ws_bytes < w.total) return 3;
    if (p.nchunks > 0x7fffffffLL) return 2;
    char* ws = static_cast<char*>(a.ws);
    float* agg = reinterpret_cast<float*>(ws + w.agg);
    float* vin = reinterpret_cast<float*>(ws + w.vin);
    uint8_t* bp = reinterpret_cast<uint8_t*>(ws + w.bp);
    uint8_t* cmap = reinterpret_cast<uint8_t*>(ws + w.cmap);
    int* xend = reinterpret_cast<int*>(ws + w.xend);
    int* xstar = reinterpret_cast<int*>(ws + w.xstar);
    double* part = reinterpret_cast<double*>(ws + w.part);
    hipStream_t st = a.stream;
    const dim3 block(256);
    // a sequence of one chunk starts from the prior: no aggregates, no carries
    if (p.cps > 1)
        launch("lv_aggregate", lv_aggregate_systolic_kernel<D>, dim3((unsigned)((p.nchunks + M::CPW - 1) / M::CPW)), block,
               st, a.A, a.ll, a.T, a.D, p.Lc, p.cps, p.nchunks, a.shared_model, agg, static_cast<float*>(nullptr));
    const Scan2 s2 = scan2_of(p);
    auto carry = [&](int cps, const float* mats, float* out, int seglen, int nseg, const float* start) {
        const unsigned blocks = (unsigned)a.batch * (unsigned)nseg;
        if constexpr (D <= 32)
            launch("lv_carry", lv_carry_wave_kernel<D>, dim3(blocks), dim3(64), st, a.prior, a.D, cps, a.shared_model, mats,
                   out, static_cast<const float*>(nullptr), static_cast<float*>(nullptr), seglen, nseg, start,
                   static_cast<const float*>(nullptr));
        else
            launch("lv_carry", lv_carry_kernel<D>, dim3(blocks), block, st, a.prior, a.D, cps, a.shared_model, mats, out,
                   static_cast<const float*>(nullptr), static_cast<float*>(nullptr), seglen, nseg, start,
                   static_cast<const float*>(nullptr));
    };
    if (s2.on) {
        constexpr int transposed = (D <= 32) ? 1 : 0;
        float* gvin = reinterpret_cast<float*>(ws + w.gvin);
        const float* cur = agg;
        const float* curm = nullptr;
        int n = p.cps;
        for (int l = 0; l < s2.k; ++l) {
            const int n_out = (n + 1) / 2;
            float* o = reinterpret_cast<float*>(ws + w.lvl[l & 1][0]);
            float* om = reinterpret_cast<float*>(ws + w.lvl[l & 1][1]);
            launch("lv_tree_product", lv_tree_product_kernel<D>, dim3((unsigned)((long long)n_out * a.batch * (D / 16))), block,
                   st, cur, static_cast<const double*>(nullptr), curm, n, n_out, transposed, o, static_cast<double*>(nullptr),
                   om);
            cur = o; curm = om;
            n = n_out;
        }
        carry(s2.G, cur, gvin, s2.G, 1, nullptr);            // V before every group
        carry(p.cps, agg, vin, s2.g, s2.G, gvin);             // V before every chunk, all groups at once
    } else if (p.cps > 1) {
        carry(p.cps, agg, vin, p.cps, 1, nullptr);
    }
    bool row_forward = false;
    if constexpr (D == 16) {
        if (p.Lc <= ROW_FORWARD_MAX_LC) {
            row_forward = true;
            launch_dyn("lv_forward", lv_forward_row_kernel<D>, dim3((unsigned)((p.nchunks + 15) / 16)), block,
                       (size_t)16 * p.Lc * D, st, a.prior, a.A, a.ll, a.T, a.D, p.Lc, p.cps, p.nchunks, a.shared_model, vin, bp,
                       cmap, xstar, part);
        }
    }
    if (!row_forward) {
        const size_t fwd_lds = (size_t)C::VCPW * p.Lc * D;
        launch_dyn("lv_forward", lv_forward_kernel<D>, dim3((unsigned)((p.nchunks + C::VCPW - 1) / C::VCPW)), block, fwd_lds,
                   st, a.prior, a.A, a.ll, a.T, a.D, p.Lc, p.cps, p.nchunks, a.shared_model, vin, bp, cmap, xstar, part);
    }
    if (s2.on) {
        uint8_t* gmap = reinterpret_cast<uint8_t*>(ws + w.gmap);
        int* xg = reinterpret_cast<int*>(ws + w.xg);
        const dim3 groups((unsigned)a.batch * (unsigned)s2.G);
        launch_dyn("lv_group_maps", lv_group_maps_kernel<D>, groups, dim3(128), (size_t)s2.g * D, st, (const uint8_t*)cmap,
                   p.cps, s2.g, s2.G, gmap);
        launch("lv_suffix", lv_suffix_kernel<D>, dim3((unsigned)a.batch), block, st, (const uint8_t*)gmap, (const int*)xstar,
               s2.G, xg, (const double*)part, p.cps, logprob_out);
        launch_dyn("lv_group_chase", lv_group_chase_kernel<D>, groups, dim3(128), (size_t)s2.g * D, st, (const uint8_t*)cmap,
                   (const int*)xg, p.cps, s2.g, s2.G, xend);
    } else {
        launch("lv_suffix", lv_suffix_kernel<D>, dim3((unsigned)a.batch), block, st, (const uint8_t*)cmap, (const int*)xstar,
               p.cps, xend, (const double*)part, p.cps, logprob_out);
    }
    const size_t path_lds = (size_t)p.Lc * D + (size_t)p.Lc * sizeof(int32_t);   // per chunk
    const int cpw = path_lds * 4 <= 48 * 1024 ? 4 : path_lds * 2 <= 48 * 1024 ? 2 : 1;
    launch_dyn("lv_path", lv_path_kernel<D>, dim3((unsigned)((p.nchunks + cpw - 1) / cpw)), block, path_lds * cpw, st, a.T,
               p.Lc, p.cps, p.nchunks, cpw, (const uint8_t*)bp, (const int*)xend, path);
    return hipGetLastError() == hipSuccess ? 0 : 4;
}

struct LargeMmWs { size_t agg, agg_other, vin, bout, F, Bv, part, lvl[2][2][2], gvin, gbout, total; };

static LargePlan max_product_plan(int Dr, long long T, int batch) {
    LargePlan p = large_plan(Dr, T, batch);
    if (p.DP < 128) p = element_plan(Dr, T, batch);   // short chunks: long sequences get the second scan level
    fill_last_round(p, T, batch);
    return p;
}

// D <= 32: forward pass, backward pass and combination of a chunk in one workgroup once that alone gives every
// SIMD four waves (four chunks per wave; the chains of maxima are latency-bound, and with fewer waves the two
// passes side by side plus lm_combine are as fast or faster: 102 against 106 us at 8192 chunks of D = 16,
// 203 against 189 us at 16384).
static bool one_pass_apply(const LargePlan& p) { return p.DP <= 32 && p.nchunks >= 16384; }

static LargeMmWs large_mm_ws(int Dr, long long T, int batch) {
    const LargePlan p = max_product_plan(Dr, T, batch);
    const size_t D = p.DP, nc = (size_t)p.nchunks, rows = (size_t)T * batch;
    LargeMmWs w;
    size_t o = 0;
    w.agg = o;       o = align_up(o + nc * D * D * sizeof(float), 256);
    w.agg_other = o; o = align_up(o + nc * D * D * sizeof(float), 256);
    w.vin = o;       o = align_up(o + nc * D * sizeof(float), 256);
    w.bout = o;      o = align_up(o + nc * D * sizeof(float), 256);
    w.F = o;         o = align_up(o + rows * Dr * sizeof(float), 256);
    w.Bv = o;        o = align_up(o + (one_pass_apply(p) ? 0 : rows * Dr * sizeof(float)), 256);
    w.part = o;      o = align_up(o + nc * sizeof(double), 256);
    const Scan2 s2 = scan2_of(p);
    for (int dir = 0; dir < 2; ++dir) {
        size_t n = (size_t)p.cps;
        for (int l = 0; l < 2; ++l) {
            n = (n + 1) / 2;
            const size_t cnt = s2.on ? n * batch : 0;
            w.lvl[dir][l][0] = o; o = align_up(o + cnt * D * D * sizeof(float), 256);
            w.lvl[dir][l][1] = o; o = align_up(o + cnt * 8 * sizeof(float), 256);
        }
    }
    const size_t ng = s2.on ? (size_t)s2.G * batch : 0;
    w.gvin = o;      o = align_up(o + ng * D * sizeof(float), 256);
    w.gbout = o;     o = align_up(o + ng * D * sizeof(float), 256);
    w.total = o;
    return w;
}

size_t large_d_max_product_ws_bytes(int Dr, long long T, int batch) { return large_mm_ws(Dr, T, batch).total; }

template <int D>
static int large_max_product_impl(const LargeArgs& a, float* mm, int32_t* path, double* logprob_out) {
    using C = LargeCfg<D>;
    using M = MpCfg<D>;
    const LargePlan p = max_product_plan(a.D, a.T, a.batch);
    const LargeMmWs w = large_mm_ws(a.D, a.T, a.batch);
    if (a.ws_bytes < w.total) return 3;
    const long long rows = a.T * a.batch;
    if (rows > 0x7fffffffLL * 4 || p.nchunks > 0x3fffffffLL) return 2;
    char* ws = static_cast<char*>(a.ws);
    float* agg = reinterpret_cast<float*>(ws + w.agg);
    float* agg_other = reinterpret_cast<float*>(ws + w.agg_other);
    float* vin = reinterpret_cast<float*>(ws + w.vin);
    float* bout = reinterpret_cast<float*>(ws + w.bout);
    float* F = reinterpret_cast<float*>(ws + w.F);
    float* Bv = reinterpret_cast<float*>(ws + w.Bv);
    double* part = reinterpret_cast<double*>(ws + w.part);
    hipStream_t st = a.stream;
    const dim3 block(256);
    if (p.cps == 1) {
        // a sequence of one chunk starts from the prior and ends with the operator's unit: no aggregates, no carries
        bout = nullptr;
    } else {
        launch("lv_aggregate", lv_aggregate_systolic_kernel<D>, dim3((unsigned)((p.nchunks + M::CPW - 1) / M::CPW)), block,
               st, a.A, a.ll, a.T, a.D, p.Lc, p.cps, p.nchunks, a.shared_model, agg, agg_other);
    }
    const Scan2 s2 = scan2_of(p);
    auto carry = [&](int cps, const float* mats, const float* mats_other, float* out, float* out_b, int seglen, int nseg,
                     const float* start, const float* start_b) {
        const unsigned blocks = 2u * (unsigned)a.batch * (unsigned)nseg;
        if constexpr (D <= 32)
            launch("lm_carry", lv_carry_wave_kernel<D>, dim3(blocks), dim3(64), st, a.prior, a.D, cps, a.shared_model, mats,
                   out, mats_other, out_b, seglen, nseg, start, start_b);
        else
            launch("lm_carry", lv_carry_kernel<D>, dim3(blocks), block, st, a.prior, a.D, cps, a.shared_model, mats, out,
                   mats_other, out_b, seglen, nseg, start, start_b);
    };
    if (s2.on) {
        // group aggregates in both orientations: the other orientation holds transposes, whose ordered product is
        // the transpose of the product in reverse order, so its operands trade places
        constexpr int transposed = (D <= 32) ? 1 : 0;
        float* gvin = reinterpret_cast<float*>(ws + w.gvin);
        float* gbout = reinterpret_cast<float*>(ws + w.gbout);
        const float* top[2] = {agg, agg_other};
        for (int dir = 0; dir < 2; ++dir) {
            const float* cur = top[dir];
            const float* curm = nullptr;
            int n = p.cps;
            for (int l = 0; l < s2.k; ++l) {
                const int n_out = (n + 1) / 2;
                float* o = reinterpret_cast<float*>(ws + w.lvl[dir][l & 1][0]);
                float* om = reinterpret_cast<float*>(ws + w.lvl[dir][l & 1][1]);
                launch("lv_tree_product", lv_tree_product_kernel<D>, dim3((unsigned)((long long)n_out * a.batch * (D / 16))),
                       block, st, cur, static_cast<const double*>(nullptr), curm, n, n_out, dir == 0 ? transposed : 1 - transposed,
                       o, static_cast<double*>(nullptr), om);
                cur = o; curm = om;
                n = n_out;
            }
            top[dir] = cur;
        }
        carry(s2.G, top[0], top[1], gvin, gbout, s2.G, 1, nullptr, nullptr);
        carry(p.cps, agg, agg_other, vin, bout, s2.g, s2.G, gvin, gbout);
    } else if (p.cps > 1) {
        carry(p.cps, agg, agg_other, vin, bout, p.cps, 1, nullptr, nullptr);
    }
    bool combined = false;
    if constexpr (D <= 32) {
        const int half = (int)((p.nchunks + 15) / 16);
        if (one_pass_apply(p)) {
            // both passes and Theorem 4's combination in one pass over the chunks
            launch("lm_apply", lm_apply_row_kernel<D, true>, dim3((unsigned)half), block, st, a.prior, a.A, a.ll, a.T, a.D,
                   p.Lc, p.cps, p.nchunks, a.shared_model, vin, bout, F, mm, path, part, half);
            combined = true;
        } else {
            launch("lm_apply", lm_apply_row_kernel<D, false>, dim3(2u * (unsigned)half), block, st, a.prior, a.A, a.ll, a.T,
                   a.D, p.Lc, p.cps, p.nchunks, a.shared_model, vin, bout, F, Bv, static_cast<int32_t*>(nullptr), part, half);
        }
    } else {
        const int half = (int)((p.nchunks + C::VCPW - 1) / C::VCPW);
        launch("lm_apply", lm_apply_kernel<D>, dim3(2u * (unsigned)half), block, st, a.prior, a.A, a.ll, a.T, a.D, p.Lc,
               p.cps, p.nchunks, a.shared_model, vin, bout, F, Bv, part, half);
    }
    if (!combined) {
        const int lpr = (a.D + 3) / 4;
        int width = 1;
        while (width < lpr) width <<= 1;
        const long long rows_per_block = 4LL * COMBINE_UNROLL * (64 / width);
        launch("lm_combine", lm_combine_kernel, dim3((unsigned)((rows + rows_per_block - 1) / rows_per_block)), block, st, F,
               Bv, rows, a.D, mm, path);
    }
    launch("lm_finalize", lm_finalize_kernel, dim3((unsigned)a.batch), dim3(64), st, part, p.cps, logprob_out);
    return hipGetLastError() == hipSuccess ? 0 : 4;
}

// Max-product block element: chunk aggregates with their offsets -> binary tree of products -> finish.
struct ElementMpWs { size_t agg, off, lvl[2][3], total; };

static ElementMpWs element_mp_ws(int Dr, long long T, int batch) {
    const LargePlan p = element_plan(Dr, T, batch);
    const size_t D = p.DP, nc = (size_t)p.nchunks;
    ElementMpWs w;
    size_t o = 0;
    w.agg = o; o = align_up(o + nc * D * D * sizeof(float), 256);
    w.off = o; o = align_up(o + nc * sizeof(double), 256);
    size_t n = (size_t)p.cps;
    for (int l = 0; l < 2; ++l) {
        n = (n + 1) / 2;
        w.lvl[l][0] = o; o = align_up(o + n * batch * D * D * sizeof(float), 256);
        w.lvl[l][1] = o; o = align_up(o + n * batch * sizeof(double), 256);
        w.lvl[l][2] = o; o = align_up(o + n * batch * 8 * sizeof(float), 256);
    }
    w.total = o;
    return w;
}

size_t large_d_element_mp_ws_bytes(int Dr, long long T, int batch) { return element_mp_ws(Dr, T, batch).total; }

template <int D>
static int large_element_mp_impl(const LargeArgs& a, float* element, double* log_scale) {
    using M = MpCfg<D>;
    const LargePlan p = element_plan(a.D, a.T, a.batch);
    const ElementMpWs w = element_mp_ws(a.D, a.T, a.batch);
    if (a.ws_bytes < w.total) return 3;
    if (p.nchunks > 0x0fffffffLL) return 2;   // the tree's first level launches nchunks / 2 * D / 16 workgroups
    char* ws = static_cast<char*>(a.ws);
    float* agg = reinterpret_cast<float*>(ws + w.agg);
    double* off = reinterpret_cast<double*>(ws + w.off);
    hipStream_t st = a.stream;
    const dim3 block(256);
    launch("lv_aggregate", lv_aggregate_offsets_kernel<D>, dim3((unsigned)((p.nchunks + M::CPW - 1) / M::CPW)), block,
           st, a.A, a.ll, a.T, a.D, p.Lc, p.cps, p.nchunks, a.shared_model, agg, off);
    constexpr int transposed = (D <= 32) ? 1 : 0;   // orientation in which the aggregate kernel stores its results
    const float* cur = agg;
    const double* curo = off;
    const float* curm = nullptr;
    int n = p.cps, l = 0;
    while (n > 1) {
        const int n_out = (n + 1) / 2;
        float* o = reinterpret_cast<float*>(ws + w.lvl[l][0]);
        double* oo = reinterpret_cast<double*>(ws + w.lvl[l][1]);
        float* om = reinterpret_cast<float*>(ws + w.lvl[l][2]);
        launch("lv_tree_product", lv_tree_product_kernel<D>, dim3((unsigned)((long long)n_out * a.batch * (D / 16))), block, st,
               cur, curo, curm, n, n_out, transposed, o, oo, om);
        cur = o; curo = oo; curm = om;
        n = n_out;
        l ^= 1;
    }
    launch("lv_element_finish", lv_element_finish_kernel<D>, dim3((unsigned)a.batch), block, st, cur, curo, a.D, transposed,
           element, log_scale);
    return hipGetLastError() == hipSuccess ? 0 : 4;
}

int large_d_element_mp(const LargeArgs& a, float* element, double* log_scale) {
    switch (element_plan(a.D, a.T, a.batch).DP) {
        case 16: return large_element_mp_impl<16>(a, element, log_scale);
        case 32: return large_element_mp_impl<32>(a, element, log_scale);
        case 64: return large_element_mp_impl<64>(a, element, log_scale);
        case 128: return large_element_mp_impl<128>(a, element, log_scale);
        default: return 2;
    }
}

int large_d_max_product(const LargeArgs& a, float* mm, int32_t* path, double* logprob_out) {
    const int DP = large_plan(a.D, a.T, a.batch).DP;
    switch (DP) {
        case 16: return large_max_product_impl<16>(a, mm, path, logprob_out);
        case 32: return large_max_product_impl<32>(a, mm, path, logprob_out);
        case 64: return large_max_product_impl<64>(a, mm, path, logprob_out);
        case 128: return large_max_product_impl<128>(a, mm, path, logprob_out);
        default: return 2;
    }
}

int large_d_viterbi(const LargeArgs& a, int32_t* path, double* logprob_out) {
    const int DP = large_plan(a.D, a.T, a.batch).DP;
    switch (DP) {
        case 16: return large_viterbi_impl<16>(a, path, logprob_out);
        case 32: return large_viterbi_impl<32>(a, path, logprob_out);
        case 64: return large_viterbi_impl<64>(a, path, logprob_out);
        case 128: return large_viterbi_impl<128>(a, path, logprob_out);
        default: return 2;
    }
}

}  // namespace hmm
