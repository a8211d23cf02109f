// Kernels and launch logic of the register-resident path for ONE state-space size
// D = HMM_SMALL_D (this file is compiled once per D in 1..8).
//
// Two launch plans compute the same thing with the same per-lane arithmetic:
//   * single-launch ("fused"): every tile is one co-resident workgroup; tile aggregates (and, for
//     Viterbi, tile back-pointer maps) are exchanged through tagged words in the workspace, so the
//     log-likelihoods are read from HBM once, nothing but the outputs is written back and a call is
//     one kernel;
//   * multi-launch: reduce -> carry -> apply (-> suffix -> path) kernels with no inter-workgroup
//     waiting, for shapes with more tiles than the GPU can hold resident at once.
// Sequences of at most 64 chunks are packed several to a workgroup and exchange nothing at all.
//
// The evidence outputs (log Z of Sec. II; the best joint log-weight of Corollary 1) are read off the
// aggregate of the whole sequence, whose scale is tracked exactly (semiring.hpp), by one lane per
// sequence; the per-step recursions carry no scale.
#include <hip/hip_runtime.h>

#include <type_traits>
#include <stdint.h>
#include <stdlib.h>

#include "ktimer.hpp"
#include "small_d.hpp"
#include "small_d_device.hpp"

#ifndef HMM_SMALL_D
#error "compile with -DHMM_SMALL_D=<1..8>"
#endif

namespace hmm {

// An exchange record in the workspace: the AggImage words of a tile's aggregate as tagged words, stored word
// by word across tiles -- word w of tile t at [w * XCH_MAX_TILES + t] -- so that the lanes of a wavefront,
// each fetching the records of two neighbouring tiles, read consecutive addresses.  Every word validates
// itself (no ordering between stores is relied upon); the tile's seal, a tagged word in a separate array
// written after the record, only tells readers when reading the record is worth while, so that the wait
// polls one word per tile instead of whole records.
template <int D>
struct SlotRecord {
    static constexpr int W = AggImage<D>::WORDS;
};
constexpr size_t XCH_WORD_STRIDE = XCH_MAX_TILES;   // 64-bit words from one word of a record to the next

// Seals and tile maps are what every workgroup polls while it waits, all of them the same few cache lines:
// the polls of 256 workgroups queue up at one memory channel, and the stores they are waiting for queue up
// behind them.  So each seal and each map is published XCH_COPIES times, in arrays that lie apart, and
// workgroup b polls copy b mod XCH_COPIES.  (Records are read once per workgroup, after the seals: one copy.)
constexpr int XCH_COPIES = 8;
constexpr size_t XCH_COPY_WORDS = XCH_MAX_TILES;   // 64-bit words from one copy of the seals / maps to the next
// The tile maps are published by all workgroups at nearly the same moment, and nothing is visible elsewhere
// sooner than a microsecond later: the first poll waits this long (s_sleep units of 64 clocks).
constexpr int MAPS_HEAD_START = 25;
constexpr int POLL_BACKOFF = 4;   // s_sleep units between two polls of a wait

// Products of the four wave totals in wagg, formed row by row by the first wavefront: a group of D lanes owns
// one product, lane i of the group its row i (rows of a product depend on the left factor's row only), so a
// product costs D^2 multiply-adds per lane instead of a whole matrix product in one lane, and the three
// products of a step run side by side:
//   step 1   group 0: W_0 W_1                     group 1: W_2 W_3
//   step 2   group 0: (W_0 W_1)(W_2 W_3)          group 1: (W_0 W_1) W_2          group 2: W_1 (W_2 W_3)
// The workgroup's aggregate (step 2, group 0) goes to `image` and is returned as the calling lane's row
// (x, xe, c) for publication.  With wp != nullptr the prefixes W_0 .. W_{w-1} go to wp->wpre[w-1] and the
// suffixes W_w .. W_3 to wp->wsuf[w-1], w = 1 .. 3.
// U: uniform mode -- the wave totals must be uniform and the products are kept uniform (all rows take the
// exponent of the largest); `bad` reports where that fails.
template <class S, int D, bool U>
HMM_DEV void wave_products_impl(const float* wagg, float* image, WaveProducts<D>* wp, float* own_lds, float (&x)[D],
                                int& xe, double& c, bool& bad) {
    using C = SmallCfg<D>;
    static_assert(C::NW == 4, "the schedule above is for four waves");
    constexpr int W = AggImage<D>::WORDS;
    constexpr bool UNI = U && !S::is_max_plus;
    const int lane = threadIdx.x & 63;
    const int g = (lane < 3 * D) ? lane / D : 0;   // spare lanes shadow group 0 and never store
    const int i = lane - (lane / D) * D;
    const bool stores = lane < 3 * D;
    // scratch images for the two step-1 products when the caller keeps none
    float* p01 = wp != nullptr ? wp->wpre + 1 * W : own_lds;
    float* p23 = wp != nullptr ? wp->wsuf + 1 * W : own_lds + W;
    auto take_row = [&](const float* src) {
#pragma unroll
        for (int j = 0; j < D; ++j) x[j] = src[i * D + j];
        xe = reinterpret_cast<const int*>(src)[D * D + i];   // SumProd: the row's exponent
        c = *reinterpret_cast<const double*>(src + D * D + D);
        if constexpr (UNI) bad = bad || (xe != reinterpret_cast<const int*>(src)[D * D]);
    };
    auto put_row = [&](float* dst, bool on) {
        if (on) {
#pragma unroll
            for (int j = 0; j < D; ++j) dst[i * D + j] = x[j];
            reinterpret_cast<int*>(dst)[D * D + i] = xe;
            if (i == 0) *reinterpret_cast<double*>(dst + D * D + D) = c;
        }
    };
    // row (op) M, as a row of an aggregate again; the D lanes of a group settle the common scale among themselves
    auto times = [&](const float* src) {
        Agg<S, D> M;
        float r[D];
        agg_load<S, D>(src, M);
        if constexpr (UNI) bad = bad || !agg_is_uniform<D>(M);
        const double sc = vec_agg_m<U, S, D>(x, M, r);
        c += M.c;
        const int g0 = g * D;
        if constexpr (S::is_max_plus) {
            // each row comes out with an offset of its own; an aggregate has one: the largest (rows that are
            // entirely -inf report 0 and stay -inf whatever is added)
            double top = __shfl(sc, g0, 64);
#pragma unroll
            for (int k = 1; k < D; ++k) {
                const double o = __shfl(sc, g0 + k, 64);
                top = o > top ? o : top;
            }
            const float d = (float)(sc - top);
#pragma unroll
            for (int j = 0; j < D; ++j) x[j] = r[j] + d;
            c += top;
        } else if constexpr (UNI) {
            // the row came out at the height of a vector with its own exponent: all rows take the largest
            const int own = xe + (int)sc;
            int top = __shfl(own, g0, 64);
#pragma unroll
            for (int k = 1; k < D; ++k) top = max_of_int(top, __shfl(own, g0 + k, 64));
            bad = bad || (top - own > UNIFORM_SPREAD);
            const int down = max_of_int(own - top, -200);
#pragma unroll
            for (int j = 0; j < D; ++j) x[j] = ldexpf(r[j], ROW_BIAS - VEC_BIAS + down);
            xe = top + (VEC_BIAS - ROW_BIAS);
        } else {
            // vec_agg leaves the row at the height of a vector: back to a row's
            xe += (int)sc + (VEC_BIAS - ROW_BIAS);
#pragma unroll
            for (int j = 0; j < D; ++j) x[j] = ldexpf(r[j], ROW_BIAS - VEC_BIAS);
        }
    };
    auto wave_sync = [&]() {   // this wave's own LDS writes before its reads
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    };
    // step 1 (groups 0 and 1; group 2 repeats group 0's work and stores nothing)
    {
        const int left = (g == 1) ? 2 : 0;
        take_row(wagg + left * W);
        times(wagg + (left + 1) * W);
        put_row(g == 1 ? p23 : p01, stores && g < 2);
    }
    wave_sync();
    // step 2
    {
        const float* xsrc = (g == 2) ? wagg + 1 * W : p01;
        const float* msrc = (g == 1) ? wagg + 2 * W : p23;
        take_row(xsrc);
        times(msrc);
        float* dst = (g == 0) ? image : (g == 1) ? (wp != nullptr ? wp->wpre + 2 * W : nullptr)
                                                 : (wp != nullptr ? wp->wsuf + 0 * W : nullptr);
        put_row(dst, stores && dst != nullptr);
    }
    if (wp != nullptr) {
        // the one-factor ends of both lists: W_0 and W_3 as they are
        if (lane < W) {
            wp->wpre[lane] = wagg[lane];
            wp->wsuf[2 * W + lane] = wagg[3 * W + lane];
        }
        if (W > 64 && lane + 64 < W) {
            wp->wpre[lane + 64] = wagg[lane + 64];
            wp->wsuf[2 * W + lane + 64] = wagg[3 * W + lane + 64];
        }
    }
}

// Call from the whole workgroup after the barrier that makes wagg visible (only the first wavefront works); the
// LDS results are visible to the other waves after the next barrier.  own_lds: 2 AggImage::WORDS floats of LDS
// scratch, needed only when wp == nullptr.  If slots != nullptr the workgroup's aggregate also goes to the tile's
// exchange record, followed by its seal.  AUTO: uniform mode where the wave totals allow it.
template <class S, int D, bool AUTO>
HMM_DEV void wave_products(const float* wagg, float* image, WaveProducts<D>* wp, float* own_lds, unsigned long long* slots,
                           unsigned long long* seal, uint32_t tag) {
    const int wave = threadIdx.x >> 6;
    const int lane = threadIdx.x & 63;
    if (wave != 0) return;
    float x[D];
    int xe;
    double c;
    bool general = true;
    if constexpr (AUTO && !S::is_max_plus) {
        bool bad = false;
        wave_products_impl<S, D, true>(wagg, image, wp, own_lds, x, xe, c, bad);
        general = wave_any(bad);
        if (general) {   // what the uniform pass left in LDS is rewritten from scratch
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
    }
    if (general) {
        bool unused = false;
        wave_products_impl<S, D, false>(wagg, image, wp, own_lds, x, xe, c, unused);
    }
    if (wave == 0 && slots != nullptr && lane < D) {
        const int i = lane;
#pragma unroll
        for (int j = 0; j < D; ++j) publish_word(slots + (i * D + j) * XCH_WORD_STRIDE, x[j], tag);
        publish_word(slots + (D * D + i) * XCH_WORD_STRIDE, (uint32_t)(S::is_max_plus ? 0 : xe), tag);
        if (lane == 0) {
            const unsigned long long cb = (unsigned long long)__double_as_longlong(c);
            publish_word(slots + (D * D + D) * XCH_WORD_STRIDE, (uint32_t)cb, tag);
            publish_word(slots + (D * D + D + 1) * XCH_WORD_STRIDE, (uint32_t)(cb >> 32), tag);
#pragma unroll
            for (int k = 0; k < XCH_COPIES; ++k) publish_word(seal + k * XCH_COPY_WORDS, 1u, tag);
        }
    }
}

// =============================================================================================
// Multi-launch plan
// =============================================================================================

// Kernel 1 (both operators): tile aggregates, as AggImage records
template <class S, int D>
__global__ __launch_bounds__(256) void sd_reduce_kernel(const float* __restrict__ A, const float* __restrict__ ll,
                                                        long long T, int tps, int shared_model,
                                                        float* __restrict__ agg) {
    using C = SmallCfg<D>;
    constexpr int W = AggImage<D>::WORDS;
    __shared__ float lds[C::LDS_FLOATS];
    __shared__ __align__(8) float wagg[C::NW * W];
    __shared__ __align__(8) float wtot[W];
    __shared__ __align__(8) float wtmp[2 * W];
    const TileCoord tc = tile_coord<D>(T, tps);
    load_tile<D>(ll + tc.base * D, tc.nvalid, lds);
    float Am[D * D];
    load_model<S, D>(A + (shared_model ? 0 : (size_t)tc.seq * D * D), Am);
    __syncthreads();
    const int n = min(max(tc.nvalid - (int)threadIdx.x * C::L, 0), C::L);
    Agg<S, D> P, Q;
    chunk_aggregate<S, D, false>(lds + threadIdx.x * C::STRIDE, n, tc.tile == 0 && threadIdx.x == 0, Am, P);
    block_prefix<S, D>(P, Q, wagg);
    __syncthreads();
    wave_products<S, D, false>(wagg, wtot, nullptr, wtmp, nullptr, nullptr, 0u);
    __syncthreads();
    if (threadIdx.x < W) agg[(size_t)blockIdx.x * W + threadIdx.x] = wtot[threadIdx.x];
}

// Kernel 2 (both operators): carries between tiles of one sequence, and the sequence's evidence.  One
// workgroup per sequence; lane t folds R consecutive tile aggregates, the workgroup exchanges the
// folds, then each lane walks its tiles again with vectors.  fin[tile] = forward potential before the
// tile's first step (prior for tile 0); bout[tile] = backward potential at the tile's last step (ones
// at T); out[seq] = log Z (SumProd) / best joint log-weight (MaxPlus) from the product of all tiles.
template <class S, int D, bool BWD>
__global__ __launch_bounds__(256) void sd_carry_kernel(const float* __restrict__ prior, int tps, int shared_model,
                                                       const float* __restrict__ agg, float* __restrict__ fin,
                                                       float* __restrict__ bout, double* __restrict__ out) {
    using C = SmallCfg<D>;
    constexpr int W = AggImage<D>::WORDS;
    __shared__ __align__(8) float wagg[C::NW * W];
    const int seq = blockIdx.x;
    const int R = (tps + C::NT - 1) / C::NT;
    const int t0 = threadIdx.x * R;
    const float* sagg = agg + (size_t)seq * tps * W;
    Agg<S, D> P;
    agg_identity<S, D>(P);
    for (int r = 0; r < R; ++r) {
        const int tile = t0 + r;
        if (tile < tps) {
            Agg<S, D> M, Z;
            agg_load<S, D>(sagg + (size_t)tile * W, M);
            agg_mul<S, D, true>(P, M, Z);
            P = Z;
        }
    }
    float cf[D], cb[D], f[D], b[D];
    const float* pr = prior + (shared_model ? 0 : (size_t)seq * D);
#pragma unroll
    for (int j = 0; j < D; ++j) {
        cf[j] = S::is_max_plus ? logf(pr[j]) : pr[j];
        cb[j] = S::one();
    }
    int bex[D];
    block_exchange<S, D, BWD>(P, cf, cb, f, b, bex, wagg);
    if constexpr (BWD && !S::is_max_plus) backward_plain<D>(b, bex);   // handed on as a plain vector
    if (threadIdx.x == 0) {
        Agg<S, D> X;
        block_total<S, D>(wagg, X);
        out[seq] = sequence_evidence<S, D>(cf, X);
    }
    float* sfin = fin + (size_t)seq * tps * D;
    for (int r = 0; r < R; ++r) {
        const int tile = t0 + r;
        if (tile < tps) {
#pragma unroll
            for (int j = 0; j < D; ++j) sfin[(size_t)tile * D + j] = f[j];
            Agg<S, D> M;
            float g[D];
            agg_load<S, D>(sagg + (size_t)tile * W, M);
            vec_agg<S, D>(f, M, g);   // the prior itself is handed over unscaled; what follows it is rescaled
#pragma unroll
            for (int j = 0; j < D; ++j) f[j] = g[j];
        }
    }
    if constexpr (BWD) {
        float* sbout = bout + (size_t)seq * tps * D;
        for (int r = R - 1; r >= 0; --r) {
            const int tile = t0 + r;
            if (tile < tps) {
#pragma unroll
                for (int j = 0; j < D; ++j) sbout[(size_t)tile * D + j] = b[j];
                Agg<S, D> M;
                float g[D];
                agg_load<S, D>(sagg + (size_t)tile * W, M);
                agg_vec<S, D>(M, b, g);
#pragma unroll
                for (int j = 0; j < D; ++j) b[j] = g[j];
            }
        }
    }
}

// Lane-level two-filter work shared by all plans: forward scan, reversed scan and their per-step
// combination inside the lane's chunk.  SumProd: marginals (Alg. 3).  MaxPlus: max-marginals
// (Alg. 5 / Theorem 4).
template <class S, int D, bool WRITE_FILT, bool COUNTS = false>
HMM_DEV void smooth_chunk(float* row, int n, bool first, const float (&Am)[D * D], float (&f)[D], float (&b)[D],
                          const int (&bex)[D], float* __restrict__ filt_dst, float (&acc)[COUNTS ? D * D : 1]) {
    using C = SmallCfg<D>;
    float F[C::L][D];
    if constexpr (S::is_max_plus) {
        if (!first) renorm<S, D>(f);   // the log prior is used as given; every other carry starts at max 0
        renorm<S, D>(b);
        if (n == C::L) {
            mpv_forward_impl<D, true>(row, n, first, Am, f, F);
            mpv_backward_impl<D, true>(row, n, Am, b, F);
        } else {
            mpv_forward_impl<D, false>(row, n, first, Am, f, F);
            mpv_backward_impl<D, false>(row, n, Am, b, F);
        }
    } else {
        float fin[D];
#pragma unroll
        for (int j = 0; j < D; ++j) fin[j] = f[j];
        if (n == C::L) {
            sp_forward_impl<D, WRITE_FILT, true>(row, n, first, Am, f, F, filt_dst);
            sp_backward_impl<D, true, COUNTS>(row, n, first, Am, b, bex, F, fin, acc);
        } else {
            sp_forward_impl<D, WRITE_FILT, false>(row, n, first, Am, f, F, filt_dst);
            sp_backward_impl<D, false, COUNTS>(row, n, first, Am, b, bex, F, fin, acc);
        }
    }
}
template <class S, int D, bool WRITE_FILT>
HMM_DEV void smooth_chunk(float* row, int n, bool first, const float (&Am)[D * D], float (&f)[D], float (&b)[D],
                          const int (&bex)[D], float* __restrict__ filt_dst) {
    float unused[1];
    smooth_chunk<S, D, WRITE_FILT, false>(row, n, first, Am, f, b, bex, filt_dst, unused);
}

// The lanes' pairwise-posterior sums of a workgroup added up, multiplied by the transition probabilities and
// written as the workgroup's partial sum (D*D floats).  `red`: NW * D * D floats of LDS.  Contains a barrier.
template <class S, int D>
HMM_DEV void store_pair_sums(const float (&acc)[D * D], const float (&Am)[D * D], float* red, float* __restrict__ dst) {
    using C = SmallCfg<D>;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int e = 0; e < D * D; ++e) {
        float v = (Am[e] > 0.0f) ? acc[e] * Am[e] : 0.0f;   // (a forbidden transition's sum is not a posterior: see sp_backward_impl)
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) v += __shfl_down(v, d, 64);
        if (lane == 0) red[wave * D * D + e] = v;
    }
    __syncthreads();
    if ((int)threadIdx.x < D * D) {
        float v = 0.0f;
#pragma unroll
        for (int w = 0; w < C::NW; ++w) v += red[w * D * D + threadIdx.x];
        dst[threadIdx.x] = v;
    }
}

// Kernel 3 (smoother, max-product): forward scan, reversed scan and (max-)marginals inside a tile;
// `argmax`, if given, receives the per-step maximiser (Theorem 4).
// COUNTS (sum-product): each workgroup also leaves the sum of the pairwise posteriors of its steps' transitions,
// times A, in pair_partial[workgroup][D*D] (the expectation step's statistic; added up per sequence afterwards).
template <class S, int D, bool WRITE_FILT, bool COUNTS = false>
__global__ __launch_bounds__(256) void sd_smooth_apply_kernel(const float* __restrict__ A,
                                                              const float* __restrict__ ll, long long T, int tps,
                                                              int shared_model, const float* __restrict__ fin_g,
                                                              const float* __restrict__ bout_g,
                                                              float* __restrict__ marg, float* __restrict__ filt,
                                                              int32_t* __restrict__ argmax,
                                                              float* __restrict__ pair_partial) {
    using C = SmallCfg<D>;
    __shared__ float lds[C::LDS_FLOATS];
    __shared__ __align__(8) float wagg[C::NW * AggImage<D>::WORDS];
    __shared__ float pair_red[COUNTS ? C::NW * D * D : 1];
    const TileCoord tc = tile_coord<D>(T, tps);
    load_tile<D>(ll + tc.base * D, tc.nvalid, lds);
    float Am[D * D];
    load_model<S, D>(A + (shared_model ? 0 : (size_t)tc.seq * D * D), Am);
    float cf[D], cb[D];
#pragma unroll
    for (int j = 0; j < D; ++j) {
        cf[j] = fin_g[(size_t)blockIdx.x * D + j];
        cb[j] = bout_g[(size_t)blockIdx.x * D + j];
    }
    __syncthreads();
    float* row = lds + threadIdx.x * C::STRIDE;
    const int n = min(max(tc.nvalid - (int)threadIdx.x * C::L, 0), C::L);
    const bool first = tc.tile == 0 && threadIdx.x == 0;
    Agg<S, D> P;
    chunk_aggregate<S, D, true>(row, n, first, Am, P);
    float f[D], b[D];
    int bex[D];
    block_exchange<S, D, true>(P, cf, cb, f, b, bex, wagg);
    // (the filtering distributions go to memory lane by lane here: a second staging tile would halve the
    // workgroups per compute unit, which costs more than the scattered stores)
    float* fdst = WRITE_FILT ? filt + (tc.base + (long long)threadIdx.x * C::L) * D : nullptr;
    float acc[COUNTS ? D * D : 1];
#pragma unroll
    for (int e = 0; e < (COUNTS ? D * D : 1); ++e) acc[e] = 0.0f;
    smooth_chunk<S, D, WRITE_FILT, COUNTS>(row, n, first, Am, f, b, bex, fdst, acc);
    __syncthreads();
    store_tile<D>(marg + tc.base * D, tc.nvalid, lds);
    if (argmax != nullptr) store_argmax_tile<D>(argmax + tc.base, tc.nvalid, lds);
    if constexpr (COUNTS) store_pair_sums<S, D>(acc, Am, pair_red, pair_partial + (size_t)blockIdx.x * D * D);
}

// Lane-level Viterbi forward work shared by all plans: h receives the chunk map, xs the final state if
// this lane holds the sequence's last step.
template <int D>
HMM_DEV void viterbi_chunk(const float* row, int n, bool first, bool last, const float (&Am)[D * D], float (&v)[D],
                           uint32_t (&bp)[SmallCfg<D>::W], uint32_t& h, uint32_t& xs) {
    using C = SmallCfg<D>;
    if (!first) renorm<MaxPlus, D>(v);   // the log prior is used as given; other carries start at max 0
    if (n == C::L) mp_forward_impl<D, true>(row, n, first, Am, v, bp);
    else mp_forward_impl<D, false>(row, n, first, Am, v, bp);
    h = chunk_map<D>(bp, n);
    xs = 0u;
    if (last) {   // x*_T = argmax V_T: every later state maps to h(x*_T)
        xs = argmax_state<D>(v);
        h = map_constant<D>(map_apply<D>(h, xs));
    }
}

// Kernel V3: forward max-plus scan inside the tile with back-pointers, each lane's chunk map and the
// tile's map.
template <int D>
__global__ __launch_bounds__(256) void sd_viterbi_forward_kernel(const float* __restrict__ A,
                                                                 const float* __restrict__ ll, long long T,
                                                                 int tps, int shared_model,
                                                                 const float* __restrict__ vin_g,
                                                                 uint32_t* __restrict__ bp_g,
                                                                 uint32_t* __restrict__ cmap_g,
                                                                 uint32_t* __restrict__ tmap_g) {
    using C = SmallCfg<D>;
    using S = MaxPlus;
    __shared__ float lds[C::LDS_FLOATS];
    __shared__ __align__(8) float wagg[C::NW * AggImage<D>::WORDS];
    __shared__ uint32_t wmaps[C::NW];
    const TileCoord tc = tile_coord<D>(T, tps);
    load_tile<D>(ll + tc.base * D, tc.nvalid, lds);
    float Am[D * D];
    load_model<S, D>(A + (shared_model ? 0 : (size_t)tc.seq * D * D), Am);
    float cf[D];
#pragma unroll
    for (int j = 0; j < D; ++j) cf[j] = vin_g[(size_t)blockIdx.x * D + j];
    __syncthreads();
    float* row = lds + threadIdx.x * C::STRIDE;
    const int n = min(max(tc.nvalid - (int)threadIdx.x * C::L, 0), C::L);
    const bool first = tc.tile == 0 && threadIdx.x == 0;
    const bool last = (tc.tile == tps - 1) && n > 0 && ((int)threadIdx.x * C::L + n == tc.nvalid);
    Agg<S, D> P;
    chunk_aggregate<S, D, false>(row, n, first, Am, P);
    float v[D], unused[D];
    int unused_ex[D];
    block_exchange<S, D, false>(P, cf, cf, v, unused, unused_ex, wagg);
    uint32_t bp[C::W], h, xs;
    viterbi_chunk<D>(row, n, first, last, Am, v, bp, h, xs);
    const size_t gl = (size_t)blockIdx.x * C::NT + threadIdx.x;
#pragma unroll
    for (int w = 0; w < C::W; ++w) bp_g[gl * C::W + w] = bp[w];
    cmap_g[gl] = last ? (h | MAP_FINAL_FLAG | (xs << MAP_FINAL_SHIFT)) : h;
    uint32_t excl;
    const uint32_t total = block_map_suffix<D>(h, excl, wmaps);
    if (threadIdx.x == 0) tmap_g[blockIdx.x] = total;
}

// Kernel V4: state at the last step of every tile, by composing tile maps right to left.  One
// workgroup per sequence.
template <int D>
__global__ __launch_bounds__(256) void sd_viterbi_suffix_kernel(const uint32_t* __restrict__ tmap_g, int tps,
                                                                uint32_t* __restrict__ xend_g) {
    using C = SmallCfg<D>;
    __shared__ uint32_t wmaps[C::NW];
    const int seq = blockIdx.x;
    const int R = (tps + C::NT - 1) / C::NT;
    const int t0 = threadIdx.x * R;
    const uint32_t* sm = tmap_g + (size_t)seq * tps;
    uint32_t g = map_identity<D>();
    for (int r = 0; r < R; ++r) {
        const int tile = t0 + r;
        if (tile < tps) g = map_compose<D>(g, sm[tile]);
    }
    uint32_t excl;
    block_map_suffix<D>(g, excl, wmaps);
    uint32_t x = map_apply<D>(excl, 0u);   // the last tile's map is constant, so the seed is immaterial
    for (int r = R - 1; r >= 0; --r) {
        const int tile = t0 + r;
        if (tile < tps) {
            xend_g[(size_t)seq * tps + tile] = x;
            x = map_apply<D>(sm[tile], x);
        }
    }
}

// Kernel V5: walk the back-pointers inside each lane's chunk and write the path.
template <int D>
__global__ __launch_bounds__(256) void sd_viterbi_path_kernel(long long T, int tps,
                                                              const uint32_t* __restrict__ bp_g,
                                                              const uint32_t* __restrict__ cmap_g,
                                                              const uint32_t* __restrict__ xend_g,
                                                              int32_t* __restrict__ path) {
    using C = SmallCfg<D>;
    __shared__ int32_t stage[C::NT * C::PSTRIDE];
    __shared__ uint32_t wmaps[C::NW];
    const TileCoord tc = tile_coord<D>(T, tps);
    const int n = min(max(tc.nvalid - (int)threadIdx.x * C::L, 0), C::L);
    const bool first = tc.tile == 0 && threadIdx.x == 0;
    const size_t gl = (size_t)blockIdx.x * C::NT + threadIdx.x;
    uint32_t bp[C::W];
#pragma unroll
    for (int w = 0; w < C::W; ++w) bp[w] = bp_g[gl * C::W + w];
    const uint32_t stored = cmap_g[gl];
    uint32_t excl;
    block_map_suffix<D>(stored & MAP_BODY, excl, wmaps);
    uint32_t x = map_apply<D>(excl, xend_g[blockIdx.x]);
    if (stored & MAP_FINAL_FLAG) x = (stored >> MAP_FINAL_SHIFT) & C::MASK;
    walk_chunk<D>(bp, n, first, x, stage + threadIdx.x * C::PSTRIDE);
    __syncthreads();
    store_path_tile<D>(path + tc.base, tc.nvalid, stage);
}

// =============================================================================================
// Single-launch plan (all tiles co-resident)
// =============================================================================================

#if HMM_SMALL_D == 1 || defined(HMM_ONLY_SMALL_D)
// Zero fill of the exchange region (hmm_workspace_init): a kernel, so that it can be captured into a graph.
__global__ void sd_zero_kernel(uint32_t* __restrict__ p, size_t n) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}
#endif

struct FusedWs {
    XchHeader* hdr;             // generation, poison flag, finished-sequence counter
    unsigned long long* agg;    // [SlotRecord::W][XCH_MAX_TILES] tagged words: tile aggregates
    unsigned long long* seal;   // [XCH_COPIES][XCH_MAX_TILES] tagged words: the tile's record is complete
    unsigned long long* tmap;   // [XCH_COPIES][XCH_MAX_TILES] tagged words: tile back-pointer maps (Viterbi)
    int batch;                  // sequences in the call
    int spin_limit;             // polls before a wait gives up (every wave terminates whatever the other workgroups do)
};

// LDS scratch of the inter-tile exchange: the per-wave reductions.
template <int D>
struct alignas(8) GridLds {
    static constexpr int W = AggImage<D>::WORDS;
    alignas(8) float red[SmallCfg<D>::NW * W];   // (aggregate images hold a double: 8-byte alignment)
};

// Generation and poison flag of the exchange region.  One thread reads them when the kernel starts and
// hands them to the workgroup through LDS (all threads must agree: barriers depend on it).
struct CallTag {
    uint32_t tag;
    bool poisoned;
};
HMM_DEV void read_call_header(const FusedWs& ws, unsigned long long* shared_word) {   // thread 0, before a barrier
    *shared_word = coherent_load(reinterpret_cast<const unsigned long long*>(ws.hdr));
}
HMM_DEV CallTag call_tag(const unsigned long long* shared_word) {                      // everyone, after the barrier
    const unsigned long long h = *shared_word;
    CallTag t;
    t.tag = (uint32_t)h + 1u;
    t.tag = t.tag == 0u ? 1u : t.tag;   // 0 is what a freshly zeroed region holds
    t.poisoned = (uint32_t)(h >> 32) != 0u;
    return t;
}

// All lanes: wait until `nrec` (<= blockDim.x) consecutive tagged words starting at `src` carry the call's tag,
// one lane per word; lane t < nrec gets word t's value.  Returns false if the bounded wait ran out.
// A poll takes a memory round trip of about a microsecond, and polls that cannot succeed yet only delay the
// stores they wait for: HEAD_START (s_sleep units of 64 clocks) is how long the first poll is held back
// where the caller knows that the words were stored only just now.
template <int HEAD_START>
HMM_DEV bool await_words(const unsigned long long* src, int nrec, uint32_t tag, int spin_limit, uint32_t& value) {
    const bool mine = (int)threadIdx.x < nrec;
    const unsigned long long* p = src + (mine ? (int)threadIdx.x : 0);
    if constexpr (HEAD_START > 0) __builtin_amdgcn_s_sleep(HEAD_START);
    for (int spin = 0; spin < spin_limit; ++spin) {
        const unsigned long long v = coherent_load(p);
        const bool valid = !mine || (uint32_t)(v >> 32) == tag;
        if (__syncthreads_and(valid ? 1 : 0)) {
            value = (uint32_t)v;
            return true;
        }
        __builtin_amdgcn_s_sleep(POLL_BACKOFF);
    }
    return false;
}

// One tile's record into registers (the calling lane's own copy); false if a word does not carry the call's tag.
// Small records are fetched in one round trip; larger ones in batches, so that the words in flight do not
// crowd out the aggregates the caller holds.
template <class S, int D>
HMM_DEV bool fetch_record(const unsigned long long* records, uint32_t tile, uint32_t tag, Agg<S, D>& M) {
    constexpr int W = AggImage<D>::WORDS;
    constexpr int NB = W <= 24 ? W : 16;
    bool valid = true;
    uint32_t clo = 0u, chi = 0u;
    uint32_t lane_off = tile * 8u;
    // (opaque to the optimiser: otherwise it forms one 64-bit address per word ahead of the retry loop and
    // keeps them all alive)
    asm volatile("" : "+v"(lane_off));
#pragma unroll
    for (int base = 0; base < W; base += NB) {
        unsigned long long v[NB];
#pragma unroll
        for (int q = 0; q < NB; ++q)
            if (base + q < W) {
                // a uniform base per word plus one 32-bit lane offset: one address register for the whole record
                const char* wbase = reinterpret_cast<const char*>(records + (base + q) * XCH_WORD_STRIDE);
                v[q] = coherent_load(reinterpret_cast<const unsigned long long*>(wbase + lane_off));
            }
#pragma unroll
        for (int q = 0; q < NB; ++q) {
            const int w = base + q;
            if (w < W) {
                valid = valid && (uint32_t)(v[q] >> 32) == tag;
                const uint32_t bits = (uint32_t)v[q];
                if (w < D * D) M.m[w] = __uint_as_float(bits);
                else if (w < D * D + D) M.ex[w - D * D] = (int)bits;
                else if (w == D * D + D) clo = bits;
                else chi = bits;
            }
        }
        if constexpr (NB < W) __builtin_amdgcn_sched_barrier(0);   // keep the batches apart
    }
    M.c = __longlong_as_double((long long)(((unsigned long long)chi << 32) | clo));
    return valid;
}

// Gather the aggregates of the sequence's tiles and return the vectors entering this tile with the
// scales they were stripped of (bits for SumProd, an offset for MaxPlus):
// cf = forward potential before its first step (start (op) M_0 (op) ... (op) M_{c-1}),
// cb = backward potential at its last step (M_{c+1} (op) ... (op) M_{tps-1} (op) ones).
// The ordered products are masked reductions over the tile slots (tps <= NT): with both directions the first two
// waves reduce the tiles before c and the last two the tiles after c; forward only, all four reduce those before c.
template <class S, int D, bool BWD>
HMM_DEV bool grid_gather(const TileCoord& tc, int tps, const float (&start)[D], const FusedWs& ws, uint32_t tag,
                         GridLds<D>& gl, float (&cf)[D], double& cfs, float (&cb)[D], double& cbs) {
    using C = SmallCfg<D>;
    using G = GridLds<D>;
    static_assert(C::NW == 4, "the split below assumes four waves");
    const int tile0 = blockIdx.x - tc.tile;   // first tile of this sequence
    uint32_t sealed;
    const size_t copy = (size_t)(blockIdx.x % XCH_COPIES) * XCH_COPY_WORDS;   // the copy this workgroup polls
    bool ok = await_words<0>(ws.seal + copy + tile0, tps, tag, ws.spin_limit, sealed);
    // every seal of this sequence seen
    const int wave = threadIdx.x >> 6;
    const int lane = threadIdx.x & 63;
    // With both directions wanted, the first two waves take the tiles before this one and the last two those after
    // it, every lane two neighbouring tiles; forward only, all four waves take the tiles before it, one per lane.
    // Records go straight into registers; after the seals they are normally complete at the first attempt.
    constexpr int NF = BWD ? 2 : 4;                       // waves on the forward side
    const bool fwd_half = wave < NF;
    const int u = (int)threadIdx.x & 127;                 // pair index 0..127 inside a half (both directions)
    const int ta = BWD ? 2 * u : (int)threadIdx.x, tb = 2 * u + 1;
    const bool use_a = ta < tps && (fwd_half ? (ta < tc.tile) : (ta > tc.tile));
    const bool use_b = BWD && tb < tps && (fwd_half ? (tb < tc.tile) : (tb > tc.tile));
    Agg<S, D> Ma, Mb;
    if (ok) {
        ok = false;
        for (int spin = 0; spin <= ws.spin_limit; ++spin) {
            bool valid = true;
            if (use_a) valid = fetch_record<S, D>(ws.agg, (uint32_t)(tile0 + ta), tag, Ma);
            if constexpr (BWD) {
                if (use_b) valid = fetch_record<S, D>(ws.agg, (uint32_t)(tile0 + tb), tag, Mb) && valid;
            }
            if (__syncthreads_and(valid ? 1 : 0)) {
                ok = true;
                break;
            }
        }
    }
    // every tile aggregate in registers
    {
        Agg<S, D> X;
        if (!(ok && use_a)) agg_identity<S, D>(Ma);
        if constexpr (BWD) {
            if (!(ok && use_b)) agg_identity<S, D>(Mb);
        }
        // lane 63 ends with the wave's ordered product
        if constexpr (S::is_max_plus) {
            if constexpr (BWD) agg_mul<S, D, true>(Ma, Mb, X);
            else X = Ma;
            wave_scan_prefix<S, D>(X);
        } else {
            double cs = Ma.c;
            bool general = !agg_is_uniform<D>(Ma);
            if constexpr (BWD) {
                cs += Mb.c;
                general = general || !agg_is_uniform<D>(Mb);
            }
            cs = wave_sum(cs);                            // the common scales just add up: no need to scan them
            general = wave_any(general);
            if (!general) {
                bool bad = false;
                if constexpr (BWD) agg_mul_u<D, false>(Ma, Mb, X, bad);
                else X = Ma;
                wave_scan_up<S, D, false, false, true>(X, bad);
                general = wave_any(bad);
            }
            if (general) {
                if constexpr (BWD) agg_mul<S, D, false>(Ma, Mb, X);
                else X = Ma;
                wave_scan_up<S, D, false, false>(X);
            }
            X.c = cs;
        }
        if (lane == 63) agg_store<S, D>(gl.red + wave * G::W, X);
    }
    __syncthreads();
    // wave products reduced
    // the wave products through the start vector / the vector of ones (every lane does the same work: no branch
    // below diverges)
    Agg<S, D> Wf[NF], Wb[2];
    bool uni = !S::is_max_plus;
#pragma unroll
    for (int w = 0; w < NF; ++w) {
        agg_load<S, D>(gl.red + w * G::W, Wf[w]);
        if constexpr (!S::is_max_plus) uni = uni && agg_is_uniform<D>(Wf[w]);
    }
    if constexpr (BWD) {
        agg_load<S, D>(gl.red + 2 * G::W, Wb[0]);
        agg_load<S, D>(gl.red + 3 * G::W, Wb[1]);
        if constexpr (!S::is_max_plus) uni = uni && agg_is_uniform<D>(Wb[0]) && agg_is_uniform<D>(Wb[1]);
    }
    auto vectors = [&](auto mode) {
        constexpr bool U = decltype(mode)::value;
        float v[D], r[D];
        double vs = 0.0;
#pragma unroll
        for (int j = 0; j < D; ++j) v[j] = start[j];
#pragma unroll
        for (int w = 0; w < NF; ++w) {
            vs += Wf[w].c + vec_agg_m<U, S, D>(v, Wf[w], r);
#pragma unroll
            for (int j = 0; j < D; ++j) v[j] = r[j];
        }
        // the first tile starts from the prior exactly as given; every later tile's carry is rescaled
#pragma unroll
        for (int j = 0; j < D; ++j) cf[j] = (tc.tile == 0) ? start[j] : v[j];
        cfs = (tc.tile == 0) ? 0.0 : vs;
#pragma unroll
        for (int j = 0; j < D; ++j) cb[j] = S::one();
        cbs = 0.0;
        if constexpr (BWD) {
#pragma unroll
            for (int w = 1; w >= 0; --w) {
                cbs += Wb[w].c + agg_vec_m<U, S, D>(Wb[w], cb, r);
#pragma unroll
                for (int j = 0; j < D; ++j) cb[j] = r[j];
            }
        }
    };
    if (!wave_any(!uni)) vectors(std::true_type{});
    else vectors(std::false_type{});
    if (!ok && threadIdx.x == 0) coherent_store(&ws.hdr->poison, 1u);
    return ok;   // false: the bounded wait ran out (the tiles were not all resident)
}

// End of a sequence's work in the single-launch plan, by one thread of the workgroup that reports the
// sequence's evidence: writes it, and once every sequence of the call has reported, advances the
// exchange region's generation (all workgroups of a sequence have read the old one before any of them
// got past its gather).  A failed call leaves the region poisoned instead.
HMM_DEV void finish_sequence(const FusedWs& ws, uint32_t tag, bool ok, double evidence, double* __restrict__ out, int seq) {
    out[seq] = ok ? evidence : __builtin_nan("");
    if (!ok) {
        coherent_store(&ws.hdr->poison, 1u);
        return;
    }
    bool last = true;
    if (ws.batch > 1) {
        const uint32_t done = __hip_atomic_fetch_add(&ws.hdr->seq_done, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        last = done + 1u == (uint32_t)ws.batch;
        if (last) coherent_store(&ws.hdr->seq_done, 0u);
    }
    if (last) coherent_store(&ws.hdr->generation, tag);
}

template <class S, int D, bool WRITE_FILT, bool COUNTS = false>
__global__ __launch_bounds__(256) void sd_smooth_fused_kernel(const float* __restrict__ prior,
                                                              const float* __restrict__ A,
                                                              const float* __restrict__ ll, long long T, int tps,
                                                              int shared_model, float* __restrict__ marg,
                                                              float* __restrict__ filt, int32_t* __restrict__ argmax,
                                                              double* __restrict__ loglik_out, FusedWs ws,
                                                              float* __restrict__ pair_partial) {
    using C = SmallCfg<D>;
    constexpr int W = AggImage<D>::WORDS;
    __shared__ float lds[C::LDS_FLOATS];
    // the filtering distributions of the tile are staged like the marginals, in a tile of their own
    __shared__ float flds[WRITE_FILT ? C::LDS_FLOATS : 1];
    __shared__ float pair_red[COUNTS ? C::NW * D * D : 1];   // (COUNTS: see sd_smooth_apply_kernel)
    __shared__ GridLds<D> gl;
    __shared__ __align__(8) float wagg[C::NW * W];
    __shared__ __align__(8) float wtot[W];
    __shared__ WaveProducts<D> wprod;
    // phase: start
    const TileCoord tc = tile_coord<D>(T, tps);
    const bool alone = tps == 1;   // the sequence is this one tile: nothing to exchange, no wait anywhere
    float Am[D * D], start[D];
    load_model_raw<D>(A + (shared_model ? 0 : (size_t)tc.seq * D * D), Am);   // issued ahead of the tile's loads
#pragma unroll
    for (int j = 0; j < D; ++j) start[j] = prior[(shared_model ? 0 : (size_t)tc.seq * D) + j];
    __shared__ unsigned long long header_word;
    if (!alone && threadIdx.x == 0) read_call_header(ws, &header_word);
    load_tile<D>(ll + tc.base * D, tc.nvalid, lds, [&]() {
        model_to_domain<S, D>(Am);
        if constexpr (S::is_max_plus) {
#pragma unroll
            for (int j = 0; j < D; ++j) start[j] = logf(start[j]);
        }
    });
    __syncthreads();
    CallTag ct{0u, false};
    if (!alone) ct = call_tag(&header_word);
    // phase: tile loaded
    float* row = lds + threadIdx.x * C::STRIDE;
    const int n = min(max(tc.nvalid - (int)threadIdx.x * C::L, 0), C::L);
    const bool first = tc.tile == 0 && threadIdx.x == 0;
    Agg<S, D> P, Q, R;
    bool uni_p, uni_q, uni_r;   // per wavefront: the lanes' P / Q / R all have equal row exponents
    chunk_aggregate_auto<S, D, true>(row, n, first, Am, P, uni_p);
    // phase: chunk aggregates
    uni_q = uni_p;
    block_prefix_auto<S, D>(P, Q, wagg, uni_q);
    __syncthreads();
    // phase: wave prefixes
    const bool publish = !alone && !ct.poisoned;
    wave_products<S, D, true>(wagg, wtot, &wprod, nullptr, publish ? ws.agg + blockIdx.x : nullptr,
                        ws.seal + blockIdx.x, ct.tag);
    // phase: published
    // the suffix scan needs nothing from other tiles: it runs while their aggregates arrive
    uni_r = uni_p;
    wave_scan_suffix_auto<S, D>(P, R, uni_r);
    // phase: suffix scan
    float cf[D], cb[D];
    double cfs = 0.0, cbs = 0.0;
    bool ok = true;
    if (alone || ct.poisoned) {
        ok = alone;
#pragma unroll
        for (int j = 0; j < D; ++j) {
            cf[j] = start[j];
            cb[j] = S::one();
        }
        __syncthreads();   // the products of the wave totals
    } else {
        ok = grid_gather<S, D, true>(tc, tps, start, ws, ct.tag, gl, cf, cfs, cb, cbs);
    }
    // phase: tile carries
    float f[D], b[D];
    int bex[D];
    carry_forward_auto<S, D>(Q, uni_q, wagg, &wprod, cf, f);
    carry_backward_auto<S, D>(R, uni_r, wagg, &wprod, cb, b, bex);
    // phase: lane carries
    float* fdst = WRITE_FILT ? flds + threadIdx.x * C::STRIDE : nullptr;
    float acc[COUNTS ? D * D : 1];
#pragma unroll
    for (int e = 0; e < (COUNTS ? D * D : 1); ++e) acc[e] = 0.0f;
    smooth_chunk<S, D, WRITE_FILT, COUNTS>(row, n, first, Am, f, b, bex, fdst, acc);
    // phase: chunk recursions
    __syncthreads();   // all marginals are in LDS (and the first wave's tile total)
    store_tile<D>(marg + tc.base * D, tc.nvalid, lds);
    if constexpr (WRITE_FILT) store_tile<D>(filt + tc.base * D, tc.nvalid, flds);
    if (argmax != nullptr) store_argmax_tile<D>(argmax + tc.base, tc.nvalid, lds);
    if constexpr (COUNTS) store_pair_sums<S, D>(acc, Am, pair_red, pair_partial + (size_t)blockIdx.x * D * D);
    // phase: stored
    // evidence of the sequence, by its last tile: (forward potential entering it) (op) M_last, summed / maximised
    // over the final state -- no backward potential is involved, so no state the two disagree on can be lost
    if (tc.tile == tps - 1 && threadIdx.x == 0) {
        Agg<S, D> Ml;
        float fin1[D];
#pragma unroll
        for (int j = 0; j < D; ++j) fin1[j] = S::one();
        agg_load<S, D>(wtot, Ml);
        const double ev = span_evidence<S, D>(cf, cfs, Ml, fin1, 0.0);
        if (alone) loglik_out[tc.seq] = ev;
        else finish_sequence(ws, ct.tag, ok, ev, loglik_out, tc.seq);
    }
}

template <int D>
__global__ __launch_bounds__(256) void sd_viterbi_fused_kernel(const float* __restrict__ prior,
                                                               const float* __restrict__ A,
                                                               const float* __restrict__ ll, long long T, int tps,
                                                               int shared_model, int32_t* __restrict__ path,
                                                               double* __restrict__ logprob_out, FusedWs ws) {
    using C = SmallCfg<D>;
    using S = MaxPlus;
    constexpr int W = AggImage<D>::WORDS;
    __shared__ float lds[C::LDS_FLOATS];
    __shared__ __align__(8) float wagg[C::NW * W];
    __shared__ __align__(8) float wtot[W];
    __shared__ GridLds<D> gl;
    __shared__ WaveProducts<D> wprod;
    __shared__ uint32_t wmaps[C::NW];
    __shared__ uint32_t wmaps2[C::NW];
    __shared__ uint32_t xend_lds;
    // phase: start
    const TileCoord tc = tile_coord<D>(T, tps);
    const int tile0 = blockIdx.x - tc.tile;
    const bool alone = tps == 1;   // the sequence is this one tile: nothing to exchange, no wait anywhere
    float Am[D * D], start[D];
    load_model_raw<D>(A + (shared_model ? 0 : (size_t)tc.seq * D * D), Am);   // issued ahead of the tile's loads
#pragma unroll
    for (int j = 0; j < D; ++j) start[j] = prior[(shared_model ? 0 : (size_t)tc.seq * D) + j];
    __shared__ unsigned long long header_word;
    if (!alone && threadIdx.x == 0) read_call_header(ws, &header_word);
    load_tile<D>(ll + tc.base * D, tc.nvalid, lds, [&]() {
        model_to_domain<S, D>(Am);
#pragma unroll
        for (int j = 0; j < D; ++j) start[j] = logf(start[j]);
    });
    __syncthreads();
    CallTag ct{0u, false};
    if (!alone) ct = call_tag(&header_word);
    // phase: tile loaded
    float* row = lds + threadIdx.x * C::STRIDE;
    const int n = min(max(tc.nvalid - (int)threadIdx.x * C::L, 0), C::L);
    const bool first = tc.tile == 0 && threadIdx.x == 0;
    const bool last = (tc.tile == tps - 1) && n > 0 && ((int)threadIdx.x * C::L + n == tc.nvalid);
    Agg<S, D> P, Q;
    chunk_aggregate<S, D, false>(row, n, first, Am, P);
    // phase: chunk aggregates
    block_prefix<S, D>(P, Q, wagg);
    __syncthreads();
    // phase: wave prefixes
    const bool exchange = !alone && !ct.poisoned;
    wave_products<S, D, true>(wagg, wtot, &wprod, nullptr, exchange ? ws.agg + blockIdx.x : nullptr,
                        ws.seal + blockIdx.x, ct.tag);
    // phase: published
    float cf[D], cb[D];
    double cfs = 0.0, cbs = 0.0;
    bool ok = !(!alone && ct.poisoned);
#pragma unroll
    for (int j = 0; j < D; ++j) cf[j] = start[j];
    if (exchange) ok = grid_gather<S, D, false>(tc, tps, start, ws, ct.tag, gl, cf, cfs, cb, cbs);
    else __syncthreads();   // the products of the wave totals
    // phase: tile carries
    float v[D];
    carry_forward<S, D>(Q, wagg, &wprod, cf, v);
    // phase: lane carries
    uint32_t bp[C::W], h, xs;
    viterbi_chunk<D>(row, n, first, last, Am, v, bp, h, xs);
    // phase: chunk recursion
    uint32_t excl;
    const uint32_t total = block_map_suffix<D>(h, excl, wmaps);
    if (exchange && ok && (int)threadIdx.x < XCH_COPIES)
        publish_word(ws.tmap + threadIdx.x * XCH_COPY_WORDS + blockIdx.x, total, ct.tag);
    // phase: tile map published
    uint32_t x;
    if (!exchange || !ok) {
        // the maps after a lane's chunk end with the last chunk's, which is constant: any argument will do
        // (a failed exchange decodes every tile on its own: the outputs of such a call are meaningless anyway)
        x = map_apply<D>(excl, 0u);
    } else {
        // the tile maps of the sequence; state at this tile's last step = maps of later tiles composed
        uint32_t tm = map_identity<D>();
        const bool ok2 = await_words<MAPS_HEAD_START>(ws.tmap + (blockIdx.x % XCH_COPIES) * XCH_COPY_WORDS + tile0, tps, ct.tag,
                                                      ws.spin_limit, tm);
        if ((int)threadIdx.x >= tps) tm = map_identity<D>();
        if (!ok2) {
            ok = false;
            tm = map_identity<D>();
            if (threadIdx.x == 0) coherent_store(&ws.hdr->poison, 1u);
        }
        // phase: tile maps gathered
        uint32_t texcl;
        block_map_suffix<D>(tm, texcl, wmaps2);
        if ((int)threadIdx.x == tc.tile) xend_lds = map_apply<D>(texcl, 0u);   // last tile's map is constant
        __syncthreads();
        x = map_apply<D>(excl, xend_lds);
    }
    if (last) x = xs;
    int32_t* stage = reinterpret_cast<int32_t*>(lds);   // the log-likelihood tile is no longer needed
    walk_chunk<D>(bp, n, first, x, stage + threadIdx.x * C::PSTRIDE);
    __syncthreads();
    // phase: walked
    store_path_tile<D>(path + tc.base, tc.nvalid, stage);
    // phase: stored
    // best joint log-weight of the sequence, by its last tile: max_j (forward potential (op) M_last)(j)
    if (tc.tile == tps - 1 && threadIdx.x == 0) {
        Agg<S, D> Ml;
        float zero[D];
#pragma unroll
        for (int j = 0; j < D; ++j) zero[j] = 0.0f;
        agg_load<S, D>(wtot, Ml);
        const double ev = span_evidence<S, D>(cf, cfs, Ml, zero, 0.0);
        if (alone) logprob_out[tc.seq] = ev;
        else finish_sequence(ws, ct.tag, ok, ev, logprob_out, tc.seq);
    }
}

// =============================================================================================
// Short sequences (at most 64 chunks): several per workgroup, nothing exchanged between workgroups
// =============================================================================================

// Smoother / max-product two-filter pass for sequences of at most 64 L steps, 256 >> lcpl of them per
// workgroup (see pack_coord).  The chunk-level scans run inside each sequence's group of lanes; the
// lane-level work is that of the other plans.
template <class S, int D, bool WRITE_FILT>
__global__ __launch_bounds__(256) void sd_smooth_packed_kernel(const float* __restrict__ prior,
                                                               const float* __restrict__ A,
                                                               const float* __restrict__ ll, long long T, int batch,
                                                               int lcpl, int shared_model, float* __restrict__ marg,
                                                               float* __restrict__ filt, int32_t* __restrict__ argmax,
                                                               double* __restrict__ out) {
    using C = SmallCfg<D>;
    __shared__ float lds[C::LDS_FLOATS];
    const PackCoord pc = pack_coord<D>(T, batch, lcpl);
    const int rowlen = (int)T * D;
    const int nfl = pc.nseq * rowlen;
    float Am[D * D];
    load_model_raw<D>(A + (shared_model ? 0 : (size_t)pc.seq * D * D), Am);
    load_packed<D>(ll + (size_t)pc.seq0 * rowlen, nfl, rowlen, lcpl, lds, [&]() { model_to_domain<S, D>(Am); });
    float start[D];
#pragma unroll
    for (int j = 0; j < D; ++j) {
        const float pr = prior[(shared_model ? 0 : (size_t)pc.seq * D) + j];
        start[j] = S::is_max_plus ? logf(pr) : pr;
    }
    __syncthreads();
    float* row = lds + threadIdx.x * C::STRIDE;
    Agg<S, D> P, Q;
    chunk_aggregate<S, D, true>(row, pc.n, pc.first, Am, P);
    float f[D], b[D];
    int bex[D];
    group_exchange<S, D, true>(P, lcpl, pc.c, start, f, b, bex, Q);
    // the group's last lane holds the aggregate of the whole sequence (lanes past its end hold neutral elements)
    if (pc.live && pc.c == (1 << lcpl) - 1) out[pc.seq] = sequence_evidence<S, D>(start, Q);
    float* fdst = WRITE_FILT ? filt + ((size_t)pc.seq * T + (size_t)pc.c * C::L) * D : nullptr;   // lane by lane, as in the apply kernel
    smooth_chunk<S, D, WRITE_FILT>(row, pc.n, pc.first, Am, f, b, bex, fdst);
    __syncthreads();   // all (max-)marginals are in LDS
    store_packed<D>(marg + (size_t)pc.seq0 * rowlen, nfl, rowlen, lcpl, lds);
    if (argmax != nullptr) store_argmax_packed<D>(argmax + (size_t)pc.seq0 * T, pc.nseq * (int)T, (int)T, lcpl, lds);
}

// Viterbi for the same sequences: forward scan with back-pointers, the reversed scan under composition
// inside each group of lanes, walk and coalesced path write.
template <int D>
__global__ __launch_bounds__(256) void sd_viterbi_packed_kernel(const float* __restrict__ prior,
                                                                const float* __restrict__ A,
                                                                const float* __restrict__ ll, long long T, int batch,
                                                                int lcpl, int shared_model, int32_t* __restrict__ path,
                                                                double* __restrict__ logprob_out) {
    using C = SmallCfg<D>;
    using S = MaxPlus;
    __shared__ float lds[C::LDS_FLOATS];
    const PackCoord pc = pack_coord<D>(T, batch, lcpl);
    const int rowlen = (int)T * D;
    const int nfl = pc.nseq * rowlen;
    float Am[D * D];
    load_model_raw<D>(A + (shared_model ? 0 : (size_t)pc.seq * D * D), Am);
    load_packed<D>(ll + (size_t)pc.seq0 * rowlen, nfl, rowlen, lcpl, lds, [&]() { model_to_domain<S, D>(Am); });
    float start[D];
#pragma unroll
    for (int j = 0; j < D; ++j) start[j] = logf(prior[(shared_model ? 0 : (size_t)pc.seq * D) + j]);
    __syncthreads();
    const float* row = lds + threadIdx.x * C::STRIDE;
    Agg<S, D> P, Q;
    chunk_aggregate<S, D, false>(const_cast<float*>(row), pc.n, pc.first, Am, P);
    float v[D], unused[D];
    int unused_ex[D];
    group_exchange<S, D, false>(P, lcpl, pc.c, start, v, unused, unused_ex, Q);
    if (pc.live && pc.c == (1 << lcpl) - 1) logprob_out[pc.seq] = sequence_evidence<S, D>(start, Q);
    uint32_t bp[C::W], h, xs;
    viterbi_chunk<D>(row, pc.n, pc.first, pc.last, Am, v, bp, h, xs);
    // the maps after a lane's chunk end with the last chunk's, which is constant: any argument will do
    uint32_t x = map_apply<D>(group_map_suffix<D>(h, lcpl, pc.c), 0u);
    if (pc.last) x = xs;
    __syncthreads();   // the log-likelihood rows are no longer needed: their space stages the path
    int32_t* stage = reinterpret_cast<int32_t*>(lds);
    walk_chunk<D>(bp, pc.n, pc.first, x, stage + threadIdx.x * C::PSTRIDE);
    __syncthreads();
    store_path_packed<D>(path + (size_t)pc.seq0 * T, pc.nseq * (int)T, (int)T, lcpl, stage);
}

// =============================================================================================
// Block-wise elements (Sec. V-B): the element of the whole block, with its scale
// =============================================================================================

// Aggregate of the lane's chunk as in chunk_aggregate, but keeping what the rescalings remove:
// the true aggregate is P * exp(scale) (SumProd) or P + scale (MaxPlus).
template <class S, int D>
HMM_DEV double chunk_element(const float* row, int n, bool first, const float (&Am)[D * D], float (&P)[D * D]) {
    using C = SmallCfg<D>;
    mat_identity<S, D>(P);
    float bs = 0.0f, rs = 0.0f;   // whole bits taken out of the emission factors / exponents or offsets removed by rescaling
#pragma unroll
    for (int k = 0; k < C::L; ++k) {
        if (k < n) {
            float ev[D];
            lds_read_vec<D>(row + k * D, ev);
            float bits, spread;
            emission<S, D>(ev, bits, spread);
            bs += bits;
            if (k == 0 && first) {   // the block's first step has no transition part
#pragma unroll
                for (int i = 0; i < D; ++i)
#pragma unroll
                    for (int j = 0; j < D; ++j) P[i * D + j] = S::times(P[i * D + j], ev[j]);
            } else {
                absorb<S, D>(P, Am, ev);
            }
            if ((k & 3) == 3 || k == n - 1) rs += renorm<S, D * D>(P);
        }
    }
    return S::is_max_plus ? (double)rs : ((double)bs + (double)rs) * 0.6931471805599453;
}

// Ordered product of one (aggregate, scale) pair per lane over the workgroup; result in thread 0.
// Inside a wave a binary tree over lane distances 1, 2, ..., 32 (lane t ends with the product of
// lanes t .. t + 2^level - 1, of which only lane 0's is used); the four wave results are folded by
// thread 0.  wred: NW * D * D floats, wsc: NW doubles.
template <class S, int D>
HMM_DEV void block_reduce_scaled(float (&P)[D * D], double& sc, float* wred, double* wsc) {
    using C = SmallCfg<D>;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        float Y[D * D], Z[D * D];
#pragma unroll
        for (int e = 0; e < D * D; ++e) Y[e] = __shfl_down(P[e], d, 64);
        const double ysc = __shfl_down(sc, d, 64);
        if (lane + d < 64) {   // lanes without a partner keep their own pair (never used further up)
            mat_mul<S, D>(P, Y, Z);
            const float r = renorm<S, D * D>(Z);
            sc += ysc + (double)r * (S::is_max_plus ? 1.0 : 0.6931471805599453);
#pragma unroll
            for (int e = 0; e < D * D; ++e) P[e] = Z[e];
        }
    }
    if (lane == 0) {
#pragma unroll
        for (int e = 0; e < D * D; ++e) wred[wave * D * D + e] = P[e];
        wsc[wave] = sc;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < C::NW; ++w) {
            float Y[D * D], Z[D * D];
#pragma unroll
            for (int e = 0; e < D * D; ++e) Y[e] = wred[w * D * D + e];
            mat_mul<S, D>(P, Y, Z);
            const float r = renorm<S, D * D>(Z);
            sc += wsc[w] + (double)r * (S::is_max_plus ? 1.0 : 0.6931471805599453);
#pragma unroll
            for (int e = 0; e < D * D; ++e) P[e] = Z[e];
        }
    }
}

// Kernel E1: (aggregate, scale) of every tile of the block.
template <class S, int D>
__global__ __launch_bounds__(256) void sd_element_tile_kernel(const float* __restrict__ A, const float* __restrict__ ll,
                                                              long long T, int tps, int shared_model,
                                                              float* __restrict__ tagg, double* __restrict__ tsc) {
    using C = SmallCfg<D>;
    __shared__ float lds[C::LDS_FLOATS];
    __shared__ float wred[C::NW * D * D];
    __shared__ double wsc[C::NW];
    const TileCoord tc = tile_coord<D>(T, tps);
    load_tile<D>(ll + tc.base * D, tc.nvalid, lds);
    float Am[D * D];
    load_model<S, D>(A + (shared_model ? 0 : (size_t)tc.seq * D * D), Am);
    __syncthreads();
    const int n = min(max(tc.nvalid - (int)threadIdx.x * C::L, 0), C::L);
    float P[D * D];
    double sc = chunk_element<S, D>(lds + threadIdx.x * C::STRIDE, n, tc.tile == 0 && threadIdx.x == 0, Am, P);
    block_reduce_scaled<S, D>(P, sc, wred, wsc);
    if (threadIdx.x == 0) {
#pragma unroll
        for (int e = 0; e < D * D; ++e) tagg[(size_t)blockIdx.x * D * D + e] = P[e];
        tsc[blockIdx.x] = sc;
    }
}

// Kernel E2: the block's element from its tiles.  One workgroup per sequence; lane t folds R
// consecutive tiles, then the workgroup's ordered product.  SumProd: largest entry in [0.5, 1);
// MaxPlus: largest entry 0.
template <class S, int D>
__global__ __launch_bounds__(256) void sd_element_fold_kernel(const float* __restrict__ tagg, const double* __restrict__ tsc,
                                                              int tps, float* __restrict__ element,
                                                              double* __restrict__ log_scale) {
    using C = SmallCfg<D>;
    __shared__ float wred[C::NW * D * D];
    __shared__ double wsc[C::NW];
    const int seq = blockIdx.x;
    const int R = (tps + C::NT - 1) / C::NT;
    const int t0 = threadIdx.x * R;
    float P[D * D];
    mat_identity<S, D>(P);
    double sc = 0.0;
    for (int r = 0; r < R; ++r) {
        const int tile = t0 + r;
        if (tile < tps) {
            float M[D * D], Z[D * D];
#pragma unroll
            for (int e = 0; e < D * D; ++e) M[e] = tagg[((size_t)seq * tps + tile) * D * D + e];
            mat_mul<S, D>(P, M, Z);
            const float rr = renorm<S, D * D>(Z);
            sc += tsc[(size_t)seq * tps + tile] + (double)rr * (S::is_max_plus ? 1.0 : 0.6931471805599453);
#pragma unroll
            for (int e = 0; e < D * D; ++e) P[e] = Z[e];
        }
    }
    block_reduce_scaled<S, D>(P, sc, wred, wsc);
    if (threadIdx.x == 0) {
        const float m = max_of(P);
        const bool none = S::is_max_plus ? (m == -INFINITY) : !(m > 0.0f);   // no sequence of the block has any weight
#pragma unroll
        for (int e = 0; e < D * D; ++e) element[(size_t)seq * D * D + e] = P[e];
        log_scale[seq] = none ? -INFINITY : sc;
    }
}

// =============================================================================================
// Host side
// =============================================================================================
static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

template <int D>
static long long tiles_per_seq(long long T) {
    return (T + SmallCfg<D>::TILE - 1) / SmallCfg<D>::TILE;
}

// Every workspace starts with the exchange region of the single-launch plan, XCH_REGION_BYTES long
// whatever the shape: header, then tagged aggregate slots, then tagged tile-map slots for up to
// XCH_MAX_TILES tiles.  Nothing else is ever written there, so that the words of the region carry either
// zero or the tag of some earlier call, for any sequence of calls on the workspace.
constexpr size_t XCH_AGG_OFFSET = 256;
constexpr size_t XCH_SEAL_OFFSET = XCH_AGG_OFFSET + (size_t)XCH_MAX_TILES * SlotRecord<SMALL_D_MAX>::W * 8;
constexpr size_t XCH_MAP_OFFSET = XCH_SEAL_OFFSET + XCH_COPIES * XCH_COPY_WORDS * 8;
static_assert(XCH_MAP_OFFSET + XCH_COPIES * XCH_COPY_WORDS * 8 <= XCH_REGION_BYTES, "exchange region too small");

struct SmoothWs { size_t agg, fin, bout, total; };
struct ViterbiWs { size_t agg, vin, bp, cmap, tmap, xend, total; };

template <int D>
static SmoothWs smooth_ws(long long T, int batch) {
    const size_t nt = (size_t)tiles_per_seq<D>(T) * batch;
    SmoothWs w;
    size_t o = XCH_REGION_BYTES;
    w.agg = o;   o = align_up(o + nt * AggImage<D>::WORDS * sizeof(float), 256);
    w.fin = o;   o = align_up(o + nt * D * sizeof(float), 256);
    w.bout = o;  o = align_up(o + nt * D * sizeof(float), 256);
    w.total = o;
    return w;
}

template <int D>
static ViterbiWs viterbi_ws(long long T, int batch) {
    using C = SmallCfg<D>;
    const size_t nt = (size_t)tiles_per_seq<D>(T) * batch;
    ViterbiWs w;
    size_t o = XCH_REGION_BYTES;
    w.agg = o;   o = align_up(o + nt * AggImage<D>::WORDS * sizeof(float), 256);
    w.vin = o;   o = align_up(o + nt * D * sizeof(float), 256);
    w.bp = o;    o = align_up(o + nt * C::NT * C::W * sizeof(uint32_t), 256);
    w.cmap = o;  o = align_up(o + nt * C::NT * sizeof(uint32_t), 256);
    w.tmap = o;  o = align_up(o + nt * sizeof(uint32_t), 256);
    w.xend = o;  o = align_up(o + nt * sizeof(uint32_t), 256);
    w.total = o;
    return w;
}

// How many workgroups of `kernel` the current device holds resident at once (cached per kernel and device).
template <int TAG, class K>
static long long resident_capacity(K kernel) {
    constexpr int MAX_DEVICES = 64;
    static long long cached[MAX_DEVICES];
    static bool have[MAX_DEVICES];
    int dev = 0, ncu = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return 0;
    if (have[dev]) return cached[dev];
    if (hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, 256, 0) != hipSuccess) return 0;
    cached[dev] = (long long)ncu * per_cu;
    have[dev] = true;
    return cached[dev];
}

// Polls before an inter-tile wait gives up.  HMMSCAN_SPIN_LIMIT overrides the default; 0 makes every
// wait fail at once, which exercises the failure path (NaN evidence, all kernels still terminate).
static int spin_limit() {
    const char* e = getenv("HMMSCAN_SPIN_LIMIT");
    if (e == nullptr) return SPIN_LIMIT;
    const long v = strtol(e, nullptr, 10);
    return (int)(v < 0 ? 0 : v > (1L << 24) ? (1L << 24) : v);
}

// Short sequences: lanes per sequence as a power of two (log2), or -1 if a sequence needs more than a wave.
template <int D>
static int packed_log2_lanes(long long T) {
    using C = SmallCfg<D>;
    if (T > 64LL * C::L) return -1;
    const int chunks = (int)((T + C::L - 1) / C::L);
    int l = 0;
    while ((1 << l) < chunks) ++l;
    return l;
}

static bool force_multi_launch() {
    const char* e = getenv("HMMSCAN_PLAN");
    return e != nullptr && e[0] == 'm';   // HMMSCAN_PLAN=multi forces the multi-launch plan
}

static FusedWs fused_ws(char* ws, int batch) {
    return FusedWs{reinterpret_cast<XchHeader*>(ws), reinterpret_cast<unsigned long long*>(ws + XCH_AGG_OFFSET),
                   reinterpret_cast<unsigned long long*>(ws + XCH_SEAL_OFFSET),
                   reinterpret_cast<unsigned long long*>(ws + XCH_MAP_OFFSET), batch, spin_limit()};
}

// The two-filter plans for either operator: marginals + optional filtered + log evidence (SumProd),
// or max-marginals + optional per-step maximiser + log of the best joint weight (MaxPlus).
// pair_partial (SumProd without a filtered output only): the kernels also leave, per tile, the sum of the pairwise
// posteriors of the tile's transitions (D*D floats each).  Sequences short enough to share workgroups then take a
// workgroup each (the packed kernels have no such output).
template <class S, int D>
static int two_filter(const SmallArgs& a, float* marg, float* filt, int32_t* argmax, double* out,
                      float* pair_partial = nullptr) {
    using C = SmallCfg<D>;
    constexpr bool MP = S::is_max_plus;
    if (pair_partial != nullptr && (MP || filt != nullptr)) return 2;
    const long long tps = tiles_per_seq<D>(a.T);
    const long long nt = tps * a.batch;
    if (nt > 0x7fffffffLL) return 2;
    const SmoothWs w = smooth_ws<D>(a.T, a.batch);
    if (a.ws_bytes < w.total) return 3;
    char* ws = static_cast<char*>(a.ws);
    float* agg = reinterpret_cast<float*>(ws + w.agg);
    float* fin = reinterpret_cast<float*>(ws + w.fin);
    float* bout = reinterpret_cast<float*>(ws + w.bout);
    hipStream_t st = a.stream;
    const dim3 grid((unsigned)nt), block(C::NT), seqs((unsigned)a.batch);
    const int itps = (int)tps;
    long long cap = 0;
    if constexpr (!MP) {
        if (filt) cap = resident_capacity<0>(sd_smooth_fused_kernel<S, D, true>);
    }
    if (!filt) cap = resident_capacity<(MP ? 5 : 1)>(sd_smooth_fused_kernel<S, D, false>);
    if constexpr (!MP) {
        if (pair_partial) cap = resident_capacity<6>(sd_smooth_fused_kernel<S, D, false, true>);
    }
    if (MP && filt) return 2;   // no filtered output is defined for the max-product plan
    if (cap > XCH_MAX_TILES) cap = XCH_MAX_TILES;
    const int lcpl = packed_log2_lanes<D>(a.T);
    if (!force_multi_launch() && lcpl >= 0 && pair_partial == nullptr) {
        // short sequences, several per workgroup: one launch, no workspace
        const int spw = C::NT >> lcpl;
        const dim3 pgrid((unsigned)((a.batch + spw - 1) / spw));
        const char* name = MP ? "sd_maxprod_packed" : "sd_smooth_packed";
        if constexpr (!MP) {
            if (filt)
                launch(name, sd_smooth_packed_kernel<S, D, true>, pgrid, block, st, a.prior, a.A, a.ll, a.T, a.batch, lcpl,
                       a.shared_model, marg, filt, argmax, out);
        }
        if (!filt)
            launch(name, sd_smooth_packed_kernel<S, D, false>, pgrid, block, st, a.prior, a.A, a.ll, a.T, a.batch, lcpl,
                   a.shared_model, marg, filt, argmax, out);
        return hipGetLastError() == hipSuccess ? 0 : 4;
    }
    // Sequences of one tile each exchange nothing: the single-launch kernel then runs for any number of them
    // (no workgroup waits for another, so they need not be resident together).
    if (!force_multi_launch() && (tps == 1 || (tps <= C::NT && nt <= cap))) {
        const FusedWs fw = fused_ws(ws, a.batch);
        const char* name = MP ? "sd_maxprod_fused" : "sd_smooth_fused";
        if constexpr (!MP) {
            if (filt)
                launch(name, sd_smooth_fused_kernel<S, D, true>, grid, block, st, a.prior, a.A, a.ll, a.T, itps,
                       a.shared_model, marg, filt, argmax, out, fw, (float*)nullptr);
        }
        if constexpr (!MP) {
            if (pair_partial)
                launch(name, sd_smooth_fused_kernel<S, D, false, true>, grid, block, st, a.prior, a.A, a.ll, a.T, itps,
                       a.shared_model, marg, filt, argmax, out, fw, pair_partial);
        }
        if (!filt && !pair_partial)
            launch(name, sd_smooth_fused_kernel<S, D, false>, grid, block, st, a.prior, a.A, a.ll, a.T, itps,
                   a.shared_model, marg, filt, argmax, out, fw, (float*)nullptr);
    } else {
        launch(MP ? "sd_reduce_mp" : "sd_reduce_sp", sd_reduce_kernel<S, D>, grid, block, st, a.A, a.ll, a.T, itps,
               a.shared_model, agg);
        launch(MP ? "sd_carry_mm" : "sd_carry_sp", sd_carry_kernel<S, D, true>, seqs, block, st, a.prior, itps,
               a.shared_model, agg, fin, bout, out);
        const char* name = MP ? "sd_maxprod_apply" : "sd_smooth_apply";
        if constexpr (!MP) {
            if (filt)
                launch(name, sd_smooth_apply_kernel<S, D, true>, grid, block, st, a.A, a.ll, a.T, itps, a.shared_model,
                       fin, bout, marg, filt, argmax, (float*)nullptr);
        }
        if constexpr (!MP) {
            if (pair_partial)
                launch(name, sd_smooth_apply_kernel<S, D, false, true>, grid, block, st, a.A, a.ll, a.T, itps,
                       a.shared_model, fin, bout, marg, filt, argmax, pair_partial);
        }
        if (!filt && !pair_partial)
            launch(name, sd_smooth_apply_kernel<S, D, false>, grid, block, st, a.A, a.ll, a.T, itps, a.shared_model,
                   fin, bout, marg, filt, argmax, (float*)nullptr);
    }
    return hipGetLastError() == hipSuccess ? 0 : 4;
}

template <int D>
int SmallD<D>::smooth(const SmallArgs& a, float* marg, float* filt, double* loglik_out) {
    return two_filter<SumProd, D>(a, marg, filt, nullptr, loglik_out);
}

template <int D>
long long SmallD<D>::tiles(long long T) { return tiles_per_seq<D>(T); }

template <int D>
int SmallD<D>::smooth_pairs(const SmallArgs& a, float* marg, double* loglik_out, float* pair_partial, long long* tiles) {
    *tiles = tiles_per_seq<D>(a.T);
    return two_filter<SumProd, D>(a, marg, nullptr, nullptr, loglik_out, pair_partial);
}

template <int D>
int SmallD<D>::max_product(const SmallArgs& a, float* maxmarg, int32_t* path, double* logprob_out) {
    return two_filter<MaxPlus, D>(a, maxmarg, nullptr, path, logprob_out);
}

template <int D>
int SmallD<D>::viterbi(const SmallArgs& a, int32_t* path, double* logprob_out) {
    using C = SmallCfg<D>;
    const long long tps = tiles_per_seq<D>(a.T);
    const long long nt = tps * a.batch;
    if (nt > 0x7fffffffLL) return 2;
    const ViterbiWs w = viterbi_ws<D>(a.T, a.batch);
    if (a.ws_bytes < w.total) return 3;
    char* ws = static_cast<char*>(a.ws);
    float* agg = reinterpret_cast<float*>(ws + w.agg);
    float* vin = reinterpret_cast<float*>(ws + w.vin);
    uint32_t* bp = reinterpret_cast<uint32_t*>(ws + w.bp);
    uint32_t* cmap = reinterpret_cast<uint32_t*>(ws + w.cmap);
    uint32_t* tmap = reinterpret_cast<uint32_t*>(ws + w.tmap);
    uint32_t* xend = reinterpret_cast<uint32_t*>(ws + w.xend);
    hipStream_t st = a.stream;
    const dim3 grid((unsigned)nt), block(C::NT), seqs((unsigned)a.batch);
    const int itps = (int)tps;
    const int lcpl = packed_log2_lanes<D>(a.T);
    if (!force_multi_launch() && lcpl >= 0) {
        const int spw = C::NT >> lcpl;
        launch("sd_viterbi_packed", sd_viterbi_packed_kernel<D>, dim3((unsigned)((a.batch + spw - 1) / spw)), block, st,
               a.prior, a.A, a.ll, a.T, a.batch, lcpl, a.shared_model, path, logprob_out);
        return hipGetLastError() == hipSuccess ? 0 : 4;
    }
    long long cap = resident_capacity<2>(sd_viterbi_fused_kernel<D>);
    if (cap > XCH_MAX_TILES) cap = XCH_MAX_TILES;
    if (!force_multi_launch() && (tps == 1 || (tps <= C::NT && nt <= cap))) {   // one tile per sequence: see two_filter
        launch("sd_viterbi_fused", sd_viterbi_fused_kernel<D>, grid, block, st, a.prior, a.A, a.ll, a.T, itps,
               a.shared_model, path, logprob_out, fused_ws(ws, a.batch));
    } else {
        launch("sd_reduce_mp", sd_reduce_kernel<MaxPlus, D>, grid, block, st, a.A, a.ll, a.T, itps, a.shared_model, agg);
        launch("sd_carry_mp", sd_carry_kernel<MaxPlus, D, false>, seqs, block, st, a.prior, itps, a.shared_model, agg, vin,
               static_cast<float*>(nullptr), logprob_out);
        launch("sd_viterbi_forward", sd_viterbi_forward_kernel<D>, grid, block, st, a.A, a.ll, a.T, itps, a.shared_model,
               vin, bp, cmap, tmap);
        launch("sd_viterbi_suffix", sd_viterbi_suffix_kernel<D>, seqs, block, st, tmap, itps, xend);
        launch("sd_viterbi_path", sd_viterbi_path_kernel<D>, grid, block, st, a.T, itps, bp, cmap, xend, path);
    }
    return hipGetLastError() == hipSuccess ? 0 : 4;
}

template <int D>
size_t SmallD<D>::element_ws_bytes(long long T, int batch) {
    const size_t nt = (size_t)tiles_per_seq<D>(T) * batch;
    return XCH_REGION_BYTES + align_up(nt * D * D * sizeof(float), 256) + align_up(nt * sizeof(double), 256);
}

template <int D>
int SmallD<D>::block_element(const SmallArgs& a, int max_product, float* element, double* log_scale) {
    using C = SmallCfg<D>;
    const long long tps = tiles_per_seq<D>(a.T);
    const long long nt = tps * a.batch;
    if (nt > 0x7fffffffLL) return 2;
    if (a.ws_bytes < element_ws_bytes(a.T, a.batch)) return 3;
    char* ws = static_cast<char*>(a.ws) + XCH_REGION_BYTES;
    float* tagg = reinterpret_cast<float*>(ws);
    double* tsc = reinterpret_cast<double*>(ws + align_up((size_t)nt * D * D * sizeof(float), 256));
    const dim3 grid((unsigned)nt), block(C::NT), seqs((unsigned)a.batch);
    if (max_product) {
        launch("sd_element_tile_mp", sd_element_tile_kernel<MaxPlus, D>, grid, block, a.stream, a.A, a.ll, a.T, (int)tps,
               a.shared_model, tagg, tsc);
        launch("sd_element_fold_mp", sd_element_fold_kernel<MaxPlus, D>, seqs, block, a.stream, tagg, tsc, (int)tps,
               element, log_scale);
    } else {
        launch("sd_element_tile_sp", sd_element_tile_kernel<SumProd, D>, grid, block, a.stream, a.A, a.ll, a.T, (int)tps,
               a.shared_model, tagg, tsc);
        launch("sd_element_fold_sp", sd_element_fold_kernel<SumProd, D>, seqs, block, a.stream, tagg, tsc, (int)tps,
               element, log_scale);
    }
    return hipGetLastError() == hipSuccess ? 0 : 4;
}

template <int D>
size_t SmallD<D>::smooth_ws_bytes(long long T, int batch) { return smooth_ws<D>(T, batch).total; }

template <int D>
size_t SmallD<D>::viterbi_ws_bytes(long long T, int batch) { return viterbi_ws<D>(T, batch).total; }

template struct SmallD<HMM_SMALL_D>;

#if HMM_SMALL_D == 1 || defined(HMM_ONLY_SMALL_D)
// Zero fill of a workspace's exchange region, enqueued on the stream (one definition for the library).
int small_d_zero_region(void* ws, size_t bytes, hipStream_t stream) {
    const size_t n = bytes / sizeof(uint32_t);
    if (n == 0) return 0;
    launch("sd_zero", sd_zero_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), stream, static_cast<uint32_t*>(ws), n);
    return hipGetLastError() == hipSuccess ? 0 : 4;
}
#endif

}  // namespace hmm
