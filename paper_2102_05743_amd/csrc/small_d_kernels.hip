// Kernels and launch logic of the register-resident path for ONE state-space size
// D = HMM_SMALL_D (this file is compiled once per D in 1..8).
//
// Two launch plans compute the same thing with the same per-lane arithmetic:
//   * single-launch ("fused"): every tile is one co-resident workgroup; tile aggregates (and, for
//     Viterbi, tile back-pointer maps) are exchanged through the workspace, so the
//     log-likelihoods are read from HBM once and nothing but the outputs is written back;
//   * multi-launch: reduce -> carry -> apply (-> suffix -> path) kernels with no inter-workgroup
//     waiting, for shapes with more tiles than the GPU can hold resident at once.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>

#include "ktimer.hpp"
#include "small_d.hpp"
#include "small_d_device.hpp"

#ifndef HMM_SMALL_D
#error "compile with -DHMM_SMALL_D=<1..8>"
#endif

namespace hmm {

// Development aid, compiled out unless HMM_PHASE_STAMPS is defined: wall-clock stamps per workgroup.
#ifdef HMM_PHASE_STAMPS
__device__ unsigned long long g_stamps[1024 * 16];
#define HMM_STAMP(i) do { if ((threadIdx.x & 63) == 0 && blockIdx.x < 256) g_stamps[(blockIdx.x * 4 + (threadIdx.x >> 6)) * 16 + (i)] = wall_clock64(); } while (0)
#else
#define HMM_STAMP(i) do { } while (0)
#endif

// =============================================================================================
// Multi-launch plan
// =============================================================================================

// Kernel 1 (both operators): tile aggregates
template <class S, int D>
__global__ __launch_bounds__(256) void sd_reduce_kernel(const float* __restrict__ A, const float* __restrict__ ll,
                                                        long long T, int tps, int shared_model,
                                                        float* __restrict__ agg) {
    using C = SmallCfg<D>;
    __shared__ float lds[C::LDS_FLOATS];
    __shared__ float wagg[C::NW * D * D];
    const TileCoord tc = tile_coord<D>(T, tps);
    load_tile<D>(ll + tc.base * D, tc.nvalid, lds);
    float Am[D * D];
    load_model<S, D>(A + (shared_model ? 0 : (size_t)tc.seq * D * D), Am);
    __syncthreads();
    const int n = min(max(tc.nvalid - (int)threadIdx.x * C::L, 0), C::L);
    float P[D * D], Q[D * D];
    double msum;
    chunk_aggregate<S, D, false>(lds + threadIdx.x * C::STRIDE, n, tc.tile == 0 && threadIdx.x == 0, Am, P, msum);
    block_prefix<S, D>(P, Q, wagg);
    __syncthreads();
    if (threadIdx.x == 0) {
        float X[D * D];
        block_total<S, D>(wagg, X);
#pragma unroll
        for (int e = 0; e < D * D; ++e) agg[(size_t)blockIdx.x * D * D + e] = X[e];
    }
}

// Kernel 2 (both operators): carries between tiles of one sequence.  One workgroup per sequence;
// lane t folds R consecutive tile aggregates, the workgroup exchanges the folds, then each lane
// walks its tiles again with vectors.  fin[tile] = forward potential before the tile's first
// step (prior for tile 0); bout[tile] = backward potential at the tile's last step (ones at T).
template <class S, int D, bool BWD>
__global__ __launch_bounds__(256) void sd_carry_kernel(const float* __restrict__ prior, int tps, int shared_model,
                                                       const float* __restrict__ agg, float* __restrict__ fin,
                                                       float* __restrict__ bout) {
    using C = SmallCfg<D>;
    __shared__ float wagg[C::NW * D * D];
    const int seq = blockIdx.x;
    const int R = (tps + C::NT - 1) / C::NT;
    const int t0 = threadIdx.x * R;
    const float* sagg = agg + (size_t)seq * tps * D * D;
    float P[D * D];
    mat_identity<S, D>(P);
    for (int r = 0; r < R; ++r) {
        const int tile = t0 + r;
        if (tile < tps) {
            float M[D * D], Z[D * D];
#pragma unroll
            for (int e = 0; e < D * D; ++e) M[e] = sagg[(size_t)tile * D * D + e];
            mat_mul<S, D>(P, M, Z);
            renorm<S, D * D>(Z);
#pragma unroll
            for (int e = 0; e < D * D; ++e) P[e] = Z[e];
        }
    }
    float cf[D], cb[D], f[D], b[D];
    const float* pr = prior + (shared_model ? 0 : (size_t)seq * D);
#pragma unroll
    for (int j = 0; j < D; ++j) {
        cf[j] = S::is_max_plus ? logf(pr[j]) : pr[j];
        cb[j] = S::one();
    }
    block_exchange<S, D, BWD>(P, cf, cb, f, b, wagg);
    float* sfin = fin + (size_t)seq * tps * D;
    for (int r = 0; r < R; ++r) {
        const int tile = t0 + r;
        if (tile < tps) {
#pragma unroll
            for (int j = 0; j < D; ++j) sfin[(size_t)tile * D + j] = f[j];
            float M[D * D], g[D];
#pragma unroll
            for (int e = 0; e < D * D; ++e) M[e] = sagg[(size_t)tile * D * D + e];
            vec_mat<S, D>(f, M, g);
            renorm<S, D>(g);   // the prior itself is handed over unscaled; what follows it is rescaled
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
                float M[D * D], g[D];
#pragma unroll
                for (int e = 0; e < D * D; ++e) M[e] = sagg[(size_t)tile * D * D + e];
                mat_vec<S, D>(M, b, g);
                renorm<S, D>(g);
#pragma unroll
                for (int j = 0; j < D; ++j) b[j] = g[j];
            }
        }
    }
}

// Lane-level two-filter work shared by both plans: forward scan, reversed scan and their per-step
// combination inside the lane's chunk.  SumProd: marginals (Alg. 3), returns the chunk-local log
// evidence.  MaxPlus: max-marginals (Alg. 5 / Theorem 4), returns the chunk-local growth of the log
// of the best joint weight.
template <class S, int D, bool WRITE_FILT>
HMM_DEV double smooth_chunk(float* row, int n, bool first, const float (&Am)[D * D], float (&f)[D], float (&b)[D],
                            double msum, float* __restrict__ filt_dst) {
    using C = SmallCfg<D>;
    float F[C::L][D];
    double delta;
    if constexpr (S::is_max_plus) {
        if (!first) renorm<S, D>(f);   // the log prior is used as given; every other carry starts at max 0
        if (n == C::L) {
            delta = mpv_forward_impl<D, true>(row, n, first, Am, f, F);
            mpv_backward_impl<D, true>(row, n, Am, b, F);
        } else {
            delta = mpv_forward_impl<D, false>(row, n, first, Am, f, F);
            mpv_backward_impl<D, false>(row, n, Am, b, F);
        }
    } else {
        if (!first) {   // the prior is used as given; every other carry is rescaled to sum to one
            const float inv = 1.0f / sum_of(f);
#pragma unroll
            for (int j = 0; j < D; ++j) f[j] *= inv;
        }
        if (n == C::L) {
            delta = sp_forward_impl<D, WRITE_FILT, true>(row, n, first, Am, f, F, msum, filt_dst);
            sp_backward_impl<D, true>(row, n, Am, b, F);
        } else {
            delta = sp_forward_impl<D, WRITE_FILT, false>(row, n, first, Am, f, F, msum, filt_dst);
            sp_backward_impl<D, false>(row, n, Am, b, F);
        }
    }
    return delta;
}

// Kernel 3 (smoother, max-product): forward scan, reversed scan and (max-)marginals inside a tile;
// `argmax`, if given, receives the per-step maximiser (Theorem 4).
template <class S, int D, bool WRITE_FILT>
__global__ __launch_bounds__(256) void sd_smooth_apply_kernel(const float* __restrict__ A,
                                                              const float* __restrict__ ll, long long T, int tps,
                                                              int shared_model, const float* __restrict__ fin_g,
                                                              const float* __restrict__ bout_g,
                                                              float* __restrict__ marg, float* __restrict__ filt,
                                                              int32_t* __restrict__ argmax,
                                                              double* __restrict__ part) {
    using C = SmallCfg<D>;
    __shared__ float lds[C::LDS_FLOATS];
    __shared__ float wagg[C::NW * D * D];
    __shared__ double dsum[C::NW];
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
    float P[D * D];
    double msum;
    chunk_aggregate<S, D, true>(row, n, first, Am, P, msum);
    float f[D], b[D];
    block_exchange<S, D, true>(P, cf, cb, f, b, wagg);
    // (the filtering distributions go to memory lane by lane here: a second staging tile would halve the
    // workgroups per compute unit, which costs more than the scattered stores)
    float* fdst = WRITE_FILT ? filt + (tc.base + (long long)threadIdx.x * C::L) * D : nullptr;
    const double delta = smooth_chunk<S, D, WRITE_FILT>(row, n, first, Am, f, b, msum, fdst);
    const double tile_delta = block_sum(delta, dsum);
    if (threadIdx.x == 0) part[blockIdx.x] = tile_delta;
    __syncthreads();
    store_tile<D>(marg + tc.base * D, tc.nvalid, lds);
    if (argmax != nullptr) store_argmax_tile<D>(argmax + tc.base, tc.nvalid, lds);
}

// Kernel 4: out[seq] = ordered sum of the tile partials of one sequence.
template <int D>
__global__ __launch_bounds__(256) void sd_finalize_kernel(const double* __restrict__ part, int tps,
                                                          double* __restrict__ out) {
    __shared__ double dsum[4];
    const int seq = blockIdx.x;
    double acc = 0.0;
    for (int t = threadIdx.x; t < tps; t += blockDim.x) acc += part[(size_t)seq * tps + t];
    const double s = block_sum(acc, dsum);
    if (threadIdx.x == 0) out[seq] = s;
}

// Lane-level Viterbi forward work shared by both plans.  Returns the offsets removed; h receives
// the chunk map, xs the final state if this lane holds the sequence's last step.
template <int D>
HMM_DEV double viterbi_chunk(const float* row, int n, bool first, bool last, const float (&Am)[D * D], float (&v)[D],
                             uint32_t (&bp)[SmallCfg<D>::W], uint32_t& h, uint32_t& xs) {
    using C = SmallCfg<D>;
    if (!first) renorm<MaxPlus, D>(v);   // the log prior is used as given; other carries start at max 0
    double osum;
    if (n == C::L) osum = mp_forward_impl<D, true>(row, n, first, Am, v, bp);
    else osum = mp_forward_impl<D, false>(row, n, first, Am, v, bp);
    h = chunk_map<D>(bp, n);
    xs = 0u;
    if (last) {   // x*_T = argmax V_T: every later state maps to h(x*_T)
        xs = argmax_state<D>(v);
        h = map_constant<D>(map_apply<D>(h, xs));
    }
    return n > 0 ? osum : 0.0;
}

// Kernel V3: forward max-plus scan inside the tile with back-pointers, each lane's chunk map,
// the tile's map, and the chunk-local log-probability.
template <int D>
__global__ __launch_bounds__(256) void sd_viterbi_forward_kernel(const float* __restrict__ A,
                                                                 const float* __restrict__ ll, long long T,
                                                                 int tps, int shared_model,
                                                                 const float* __restrict__ vin_g,
                                                                 uint32_t* __restrict__ bp_g,
                                                                 uint32_t* __restrict__ cmap_g,
                                                                 uint32_t* __restrict__ tmap_g,
                                                                 double* __restrict__ part) {
    using C = SmallCfg<D>;
    using S = MaxPlus;
    __shared__ float lds[C::LDS_FLOATS];
    __shared__ float wagg[C::NW * D * D];
    __shared__ double dsum[C::NW];
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
    float P[D * D];
    double msum;
    chunk_aggregate<S, D, false>(row, n, first, Am, P, msum);
    float v[D], unused[D];
    block_exchange<S, D, false>(P, cf, cf, v, unused, wagg);
    uint32_t bp[C::W], h, xs;
    const double osum = viterbi_chunk<D>(row, n, first, last, Am, v, bp, h, xs);
    const double tile_delta = block_sum(osum, dsum);
    if (threadIdx.x == 0) part[blockIdx.x] = tile_delta;
    const size_t gl = (size_t)blockIdx.x * C::NT + threadIdx.x;
#pragma unroll
    for (int w = 0; w < C::W; ++w) bp_g[gl * C::W + w] = bp[w];
    cmap_g[gl] = last ? (h | MAP_FINAL_FLAG | (xs << MAP_FINAL_SHIFT)) : h;
    uint32_t excl;
    const uint32_t total = block_map_suffix<D>(h, excl, wmaps);
    if (threadIdx.x == 0) tmap_g[blockIdx.x] = total;
}

// Kernel V4: state at the last step of every tile, by composing tile maps right to left, and the
// sequence's log-probability.  One workgroup per sequence.
template <int D>
__global__ __launch_bounds__(256) void sd_viterbi_suffix_kernel(const uint32_t* __restrict__ tmap_g, int tps,
                                                                uint32_t* __restrict__ xend_g,
                                                                const double* __restrict__ part,
                                                                double* __restrict__ logprob) {
    using C = SmallCfg<D>;
    __shared__ uint32_t wmaps[C::NW];
    __shared__ double dsum[C::NW];
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
    double acc = 0.0;
    for (int t = threadIdx.x; t < tps; t += blockDim.x) acc += part[(size_t)seq * tps + t];
    const double s = block_sum(acc, dsum);
    if (threadIdx.x == 0) logprob[seq] = s;
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

// Fills the exchange slots of a call with the sentinel pattern; launched on the same stream right
// before the fused kernel.
template <int D>
__global__ void sd_clear_kernel(uint32_t* __restrict__ p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = (i == n - 1) ? 0u : SENTINEL32;   // the last word is the error flag
}

struct FusedWs {
    float* agg;        // [tiles][D*D]  tile aggregates
    double* part;      // [tiles]       tile-local log evidence / log-probability
    uint32_t* tmap;    // [tiles]       tile back-pointer maps (Viterbi)
    uint32_t* err;     // [1]           set if a bounded wait ran out
    int spin_limit;    // polls before a wait gives up (every wave terminates whatever the other workgroups do)
};

// LDS scratch of the inter-tile exchange.  Staged aggregates are stored in pairs of tiles, each
// pair padded by four floats so that 64 lanes reading one pair each do not collide on LDS banks.
template <int D>
struct GridLds {
    static constexpr int PAIR = 2 * D * D;
    static constexpr int PSTR = PAIR + 4;
    float red[SmallCfg<D>::NW * D * D];               // per-wave reductions of tile aggregates
    float aggs[(SmallCfg<D>::NT / 2) * PSTR];         // the sequence's tile aggregates, staged
};

// Largest value over the wavefront (every lane must call; all lanes get the result).
HMM_DEV float wave_all_max(float v) {
    v = fmaxf(v, dpp_move<0x111, 0xF>(-INFINITY, v));   // row_shr:1
    v = fmaxf(v, dpp_move<0x112, 0xF>(-INFINITY, v));   // row_shr:2
    v = fmaxf(v, dpp_move<0x114, 0xF>(-INFINITY, v));   // row_shr:4
    v = fmaxf(v, dpp_move<0x118, 0xF>(-INFINITY, v));   // row_shr:8
    v = fmaxf(v, dpp_move<0x142, 0xA>(-INFINITY, v));   // row_bcast:15
    v = fmaxf(v, dpp_move<0x143, 0xC>(-INFINITY, v));   // row_bcast:31
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// The first wave publishes this tile's aggregate, the ordered product of the wave totals in wagg.
// Lane e < D*D owns entry (e / D, e % D) of the running product: its row comes from the other
// lanes by shuffles, the next wave total's column from LDS, so the chain of products costs a few
// instructions per lane instead of whole matrix products in a single lane.
template <class S, int D>
HMM_DEV void grid_publish(const float* wagg, const FusedWs& ws) {
    using C = SmallCfg<D>;
    static_assert(D * D <= 64, "one lane per entry of the aggregate");
    if (threadIdx.x < 64) {
        const int lane = threadIdx.x;
        const int e = lane < D * D ? lane : 0;   // spare lanes shadow entry 0 and never store
        const int i = e / D, j = e % D;
        float x = wagg[e];
#pragma unroll
        for (int w = 1; w < C::NW; ++w) {
            float acc = S::zero();
#pragma unroll
            for (int k = 0; k < D; ++k) acc = S::mul_add(acc, __shfl(x, i * D + k, 64), wagg[(w * D + k) * D + j]);
            const float m = wave_all_max(acc);
            if constexpr (S::is_max_plus) x = acc - ((m == -INFINITY) ? 0.0f : m);
            else x = ldexpf(acc, -__builtin_amdgcn_frexp_expf(m));
        }
        if (lane < D * D)
            coherent_store(reinterpret_cast<uint32_t*>(ws.agg + (size_t)blockIdx.x * D * D) + e, publish_bits(x));
    }
}

// All lanes: poll n consecutive floats at `src` (slots written by other workgroups) until none
// holds the sentinel, staging them into LDS in the padded pair layout.  Coalesced 8-byte loads
// when the base is 8-byte aligned.  Returns false if the bounded wait ran out.
template <int D>
HMM_DEV bool gather_aggregates(const float* src, int n, float* dst_lds, int spin_limit) {
    using G = GridLds<D>;
    const bool wide = (reinterpret_cast<uintptr_t>(src) & 7u) == 0;
    for (int spin = 0; spin < spin_limit; ++spin) {
        bool valid = true;
        if (wide) {
            const unsigned long long* s2 = reinterpret_cast<const unsigned long long*>(src);
            const int n2 = n >> 1;
            constexpr int NB = 8;   // loads in flight per lane: issued together, then checked and staged
            for (int base = 0; base < n2; base += NB * (int)blockDim.x) {
                unsigned long long w[NB];
#pragma unroll
                for (int q = 0; q < NB; ++q) {
                    const int i = base + q * (int)blockDim.x + (int)threadIdx.x;
                    w[q] = coherent_load(s2 + (i < n2 ? i : n2 - 1));
                }
#pragma unroll
                for (int q = 0; q < NB; ++q) {
                    const int i = base + q * (int)blockDim.x + (int)threadIdx.x;
                    if (i < n2) {
                        const uint32_t lo = (uint32_t)w[q], hi = (uint32_t)(w[q] >> 32);
                        valid = valid && lo != SENTINEL32 && hi != SENTINEL32;
                        const int f = 2 * i;
                        const int d0 = (f / G::PAIR) * G::PSTR + f % G::PAIR;
                        const int d1 = ((f + 1) / G::PAIR) * G::PSTR + (f + 1) % G::PAIR;
                        dst_lds[d0] = __uint_as_float(lo);
                        dst_lds[d1] = __uint_as_float(hi);
                    }
                }
            }
            if ((n & 1) && threadIdx.x == 0) {
                const uint32_t w = coherent_load(reinterpret_cast<const uint32_t*>(src) + n - 1);
                valid = valid && w != SENTINEL32;
                dst_lds[((n - 1) / G::PAIR) * G::PSTR + (n - 1) % G::PAIR] = __uint_as_float(w);
            }
        } else {
            for (int i = threadIdx.x; i < n; i += blockDim.x) {
                const uint32_t w = coherent_load(reinterpret_cast<const uint32_t*>(src) + i);
                valid = valid && w != SENTINEL32;
                dst_lds[(i / G::PAIR) * G::PSTR + i % G::PAIR] = __uint_as_float(w);
            }
        }
        if (__syncthreads_and(valid ? 1 : 0)) {
#ifdef HMM_PHASE_STAMPS
            if ((threadIdx.x & 63) == 0 && blockIdx.x < 256) g_stamps[(blockIdx.x * 4 + (threadIdx.x >> 6)) * 16 + 5] = spin;
#endif
            return true;
        }
        __builtin_amdgcn_s_sleep(1);
    }
    return false;
}

// Gather the aggregates of the sequence's tiles and return the vectors entering this tile:
// cf = forward potential before its first step (prior (op) M_0 (op) ... (op) M_{c-1}),
// cb = backward potential at its last step (M_{c+1} (op) ... (op) M_{tps-1} (op) ones).
// The two ordered products are masked reductions over at most 2*128 tile slots: the first two
// waves reduce the tiles before c, the last two the tiles after c (tps <= NT).
template <class S, int D, bool BWD>
HMM_DEV bool grid_gather(const TileCoord& tc, int tps, const float* __restrict__ prior, const FusedWs& ws,
                         GridLds<D>& gl, float (&cf)[D], float (&cb)[D]) {
    using C = SmallCfg<D>;
    using G = GridLds<D>;
    static_assert(C::NW == 4, "the split below assumes four waves");
    const int tile0 = blockIdx.x - tc.tile;   // first tile of this sequence
    const bool ok = gather_aggregates<D>(ws.agg + (size_t)tile0 * D * D, tps * D * D, gl.aggs, ws.spin_limit);
    if (!ok && threadIdx.x == 0) atomicOr(ws.err, 1u);
    HMM_STAMP(14);
    const int wave = threadIdx.x >> 6;
    const int lane = threadIdx.x & 63;
    const bool fwd_half = wave < 2;
    if (fwd_half || BWD) {
        const int u = (int)threadIdx.x & 127;             // pair index 0..127 inside the half
        float Ma[D * D], Mb[D * D], X[D * D];
        const int ta = 2 * u, tb = 2 * u + 1;
        const bool use_a = ok && ta < tps && (fwd_half ? (ta < tc.tile) : (ta > tc.tile));
        const bool use_b = ok && tb < tps && (fwd_half ? (tb < tc.tile) : (tb > tc.tile));
        const float* pa = gl.aggs + u * G::PSTR;
#pragma unroll
        for (int i = 0; i < D; ++i)
#pragma unroll
            for (int j = 0; j < D; ++j) {
                const float id = (i == j) ? S::one() : S::zero();
                Ma[i * D + j] = use_a ? pa[i * D + j] : id;
                Mb[i * D + j] = use_b ? pa[D * D + i * D + j] : id;
            }
        mat_mul<S, D>(Ma, Mb, X);
        wave_scan_prefix<S, D>(X);                        // lane 63 ends with the wave's ordered product
        if (lane == 63) {
#pragma unroll
            for (int e = 0; e < D * D; ++e) gl.red[wave * D * D + e] = X[e];
        }
    }
    __syncthreads();
    HMM_STAMP(15);
    float pr[D], v[D], r[D], Wm[D * D];
#pragma unroll
    for (int j = 0; j < D; ++j) v[j] = pr[j] = S::is_max_plus ? logf(prior[j]) : prior[j];
#pragma unroll
    for (int w = 0; w < 2; ++w) {
#pragma unroll
        for (int e = 0; e < D * D; ++e) Wm[e] = gl.red[w * D * D + e];
        vec_mat<S, D>(v, Wm, r);
        renorm<S, D>(r);
#pragma unroll
        for (int j = 0; j < D; ++j) v[j] = r[j];
    }
    // the first tile starts from the prior exactly as given (its scale is part of the evidence);
    // every later tile's carry is scale-free
#pragma unroll
    for (int j = 0; j < D; ++j) cf[j] = (tc.tile == 0) ? pr[j] : v[j];
#pragma unroll
    for (int j = 0; j < D; ++j) cb[j] = S::one();
    if constexpr (BWD) {
#pragma unroll
        for (int w = 3; w >= 2; --w) {
#pragma unroll
            for (int e = 0; e < D * D; ++e) Wm[e] = gl.red[w * D * D + e];
            mat_vec<S, D>(Wm, cb, r);
            renorm<S, D>(r);
#pragma unroll
            for (int j = 0; j < D; ++j) cb[j] = r[j];
        }
    }
    return ok;   // false: the bounded wait ran out (the tiles were not all resident); the caller poisons its evidence
}

// All lanes: poll the sequence's tile partials until all are published, then out[seq] = their
// ordered sum.  Run by the workgroup of tile 0.
HMM_DEV void grid_sum_parts(int tile0, int tps, const FusedWs& ws, double* dsum, double* __restrict__ out, int seq) {
    double acc = 0.0;
    bool ok = false;
    for (int spin = 0; spin < ws.spin_limit; ++spin) {
        bool valid = true;
        acc = 0.0;
        if ((int)threadIdx.x < tps) {
            const unsigned long long w = coherent_load(reinterpret_cast<const unsigned long long*>(ws.part) + tile0 + threadIdx.x);
            valid = w != SENTINEL64;
            acc = __longlong_as_double((long long)w);
        }
        if (__syncthreads_and(valid ? 1 : 0)) { ok = true; break; }
        __builtin_amdgcn_s_sleep(1);
    }
    if (!ok) {
        if (threadIdx.x == 0) atomicOr(ws.err, 1u);
        acc = __builtin_nan("");
    }
    const double s = block_sum(acc, dsum);
    if (threadIdx.x == 0) out[seq] = s;
}

template <class S, int D, bool WRITE_FILT>
__global__ __launch_bounds__(256) void sd_smooth_fused_kernel(const float* __restrict__ prior,
                                                              const float* __restrict__ A,
                                                              const float* __restrict__ ll, long long T, int tps,
                                                              int shared_model, float* __restrict__ marg,
                                                              float* __restrict__ filt, int32_t* __restrict__ argmax,
                                                              double* __restrict__ loglik_out, FusedWs ws) {
    using C = SmallCfg<D>;
    __shared__ float lds[C::LDS_FLOATS];
    // the filtering distributions of the tile are staged like the marginals, in the space the inter-tile exchange
    // has finished with by then (both do not fit beside the tile at D >= 7)
    __shared__ union FusedShared {
        GridLds<D> gl;
        float flds[WRITE_FILT ? C::LDS_FLOATS : 1];
    } sh;
    GridLds<D>& gl = sh.gl;
    float* flds = sh.flds;
    __shared__ float wagg[C::NW * D * D];
    __shared__ double dsum[C::NW];
    HMM_STAMP(0);
#ifdef HMM_PHASE_STAMPS
    if ((threadIdx.x & 63) == 0 && blockIdx.x < 256) {
        g_stamps[(blockIdx.x * 4 + (threadIdx.x >> 6)) * 16 + 12] = __builtin_amdgcn_s_getreg(63492);   // HW_ID
        g_stamps[(blockIdx.x * 4 + (threadIdx.x >> 6)) * 16 + 13] = __builtin_amdgcn_s_getreg(63508);   // XCC_ID
    }
#endif
    const TileCoord tc = tile_coord<D>(T, tps);
    float Am[D * D];
    load_model_raw<D>(A + (shared_model ? 0 : (size_t)tc.seq * D * D), Am);   // issued ahead of the tile's loads
    load_tile<D>(ll + tc.base * D, tc.nvalid, lds, [&]() { model_to_domain<S, D>(Am); });
    __syncthreads();
    HMM_STAMP(1);
    float* row = lds + threadIdx.x * C::STRIDE;
    const int n = min(max(tc.nvalid - (int)threadIdx.x * C::L, 0), C::L);
    const bool first = tc.tile == 0 && threadIdx.x == 0;
    float P[D * D], Q[D * D], R[D * D];
    double msum;
    chunk_aggregate<S, D, true>(row, n, first, Am, P, msum);
    HMM_STAMP(2);
    block_prefix<S, D>(P, Q, wagg);
    __syncthreads();
    HMM_STAMP(3);
    const bool alone = tps == 1;   // the sequence is this one tile: nothing to exchange, no wait anywhere
    if (!alone) grid_publish<S, D>(wagg, ws);
    HMM_STAMP(4);
    // the suffix scan needs nothing from other tiles: it runs while their aggregates arrive
#pragma unroll
    for (int e = 0; e < D * D; ++e) R[e] = P[e];
    wave_scan_suffix<S, D>(R);
    float cf[D], cb[D];
    bool ok = true;
    if (alone) {
        const float* pr = prior + (shared_model ? 0 : (size_t)tc.seq * D);
#pragma unroll
        for (int j = 0; j < D; ++j) {
            cf[j] = S::is_max_plus ? logf(pr[j]) : pr[j];
            cb[j] = S::one();
        }
    } else {
        ok = grid_gather<S, D, true>(tc, tps, prior + (shared_model ? 0 : (size_t)tc.seq * D), ws, gl, cf, cb);
        if constexpr (WRITE_FILT) __syncthreads();   // every wave is done with the exchange area before it is reused
    }
    HMM_STAMP(6);
    float f[D], b[D];
    carry_forward<S, D>(Q, wagg, cf, f);
    carry_backward<S, D>(R, wagg, cb, b);
    HMM_STAMP(7);
    float* fdst = WRITE_FILT ? flds + threadIdx.x * C::STRIDE : nullptr;
    double delta = smooth_chunk<S, D, WRITE_FILT>(row, n, first, Am, f, b, msum, fdst);
    if (!ok) delta = __builtin_nan("");   // an expired wait makes the call's log evidence NaN
    HMM_STAMP(8);
    const double tile_delta = block_sum(delta, dsum);   // contains a barrier: all marginals are in LDS
    if (threadIdx.x == 0) {
        if (alone) loglik_out[tc.seq] = tile_delta;
        else coherent_store(reinterpret_cast<unsigned long long*>(ws.part) + blockIdx.x, publish_bits(tile_delta));
    }
    HMM_STAMP(9);
    store_tile<D>(marg + tc.base * D, tc.nvalid, lds);
    if constexpr (WRITE_FILT) store_tile<D>(filt + tc.base * D, tc.nvalid, flds);
    if (argmax != nullptr) store_argmax_tile<D>(argmax + tc.base, tc.nvalid, lds);
    HMM_STAMP(10);
    if (!alone && tc.tile == 0) grid_sum_parts(blockIdx.x, tps, ws, dsum, loglik_out, tc.seq);
    HMM_STAMP(11);
}

template <int D>
__global__ __launch_bounds__(256) void sd_viterbi_fused_kernel(const float* __restrict__ prior,
                                                               const float* __restrict__ A,
                                                               const float* __restrict__ ll, long long T, int tps,
                                                               int shared_model, int32_t* __restrict__ path,
                                                               double* __restrict__ logprob_out, FusedWs ws) {
    using C = SmallCfg<D>;
    using S = MaxPlus;
    __shared__ float lds[C::LDS_FLOATS];
    __shared__ float wagg[C::NW * D * D];
    __shared__ GridLds<D> gl;
    __shared__ double dsum[C::NW];
    __shared__ uint32_t wmaps[C::NW];
    __shared__ uint32_t wmaps2[C::NW];
    __shared__ uint32_t xend_lds;
    HMM_STAMP(0);
    const TileCoord tc = tile_coord<D>(T, tps);
    const int tile0 = blockIdx.x - tc.tile;
    float Am[D * D];
    load_model_raw<D>(A + (shared_model ? 0 : (size_t)tc.seq * D * D), Am);   // issued ahead of the tile's loads
    load_tile<D>(ll + tc.base * D, tc.nvalid, lds, [&]() { model_to_domain<S, D>(Am); });
    __syncthreads();
    HMM_STAMP(1);
    float* row = lds + threadIdx.x * C::STRIDE;
    const int n = min(max(tc.nvalid - (int)threadIdx.x * C::L, 0), C::L);
    const bool first = tc.tile == 0 && threadIdx.x == 0;
    const bool last = (tc.tile == tps - 1) && n > 0 && ((int)threadIdx.x * C::L + n == tc.nvalid);
    float P[D * D], Q[D * D];
    double msum;
    chunk_aggregate<S, D, false>(row, n, first, Am, P, msum);
    HMM_STAMP(2);
    block_prefix<S, D>(P, Q, wagg);
    __syncthreads();
    HMM_STAMP(3);
    const bool alone = tps == 1;   // the sequence is this one tile: nothing to exchange, no wait anywhere
    float cf[D], cb[D];
    bool ok = true;
    if (alone) {
        const float* pr = prior + (shared_model ? 0 : (size_t)tc.seq * D);
#pragma unroll
        for (int j = 0; j < D; ++j) cf[j] = logf(pr[j]);
    } else {
        grid_publish<S, D>(wagg, ws);
        HMM_STAMP(4);
        ok = grid_gather<S, D, false>(tc, tps, prior + (shared_model ? 0 : (size_t)tc.seq * D), ws, gl, cf, cb);
    }
    HMM_STAMP(6);
    float v[D];
    carry_forward<S, D>(Q, wagg, cf, v);
    HMM_STAMP(7);
    uint32_t bp[C::W], h, xs;
    double osum = viterbi_chunk<D>(row, n, first, last, Am, v, bp, h, xs);
    if (!ok) osum = __builtin_nan("");   // an expired wait makes the call's log-probability NaN
    HMM_STAMP(8);
    uint32_t excl;
    const uint32_t total = block_map_suffix<D>(h, excl, wmaps);
    if (!alone && threadIdx.x == 0) coherent_store(ws.tmap + blockIdx.x, total);   // a map uses 24 bits: never the sentinel
    HMM_STAMP(9);
    const double tile_delta = block_sum(osum, dsum);   // other tiles wait for the map, not for this
    if (threadIdx.x == 0) {
        if (alone) logprob_out[tc.seq] = tile_delta;
        else coherent_store(reinterpret_cast<unsigned long long*>(ws.part) + blockIdx.x, publish_bits(tile_delta));
    }
    bool ok2 = true;
    uint32_t x;
    if (alone) {
        // the maps after a lane's chunk end with the last chunk's, which is constant: any argument will do
        x = map_apply<D>(excl, 0u);
    } else {
        // the tile maps of the sequence; state at this tile's last step = maps of later tiles composed
        uint32_t tm = map_identity<D>();
        ok2 = false;
        for (int spin = 0; spin < ws.spin_limit; ++spin) {
            bool valid = true;
            if ((int)threadIdx.x < tps) {
                tm = coherent_load(ws.tmap + tile0 + threadIdx.x);
                valid = tm != SENTINEL32;
            }
            if (__syncthreads_and(valid ? 1 : 0)) { ok2 = true; break; }
            __builtin_amdgcn_s_sleep(1);
        }
        if (!ok2) {
            if (threadIdx.x == 0) atomicOr(ws.err, 1u);
            tm = map_identity<D>();
        }
        HMM_STAMP(10);
        uint32_t texcl;
        block_map_suffix<D>(tm, texcl, wmaps2);
        if ((int)threadIdx.x == tc.tile) xend_lds = map_apply<D>(texcl, 0u);   // last tile's map is constant
        __syncthreads();
        x = map_apply<D>(excl, xend_lds);
    }
    if (last) x = xs;
    HMM_STAMP(11);
    int32_t* stage = reinterpret_cast<int32_t*>(lds);   // the log-likelihood tile is no longer needed
    walk_chunk<D>(bp, n, first, x, stage + threadIdx.x * C::PSTRIDE);
    __syncthreads();
    HMM_STAMP(12);
    store_path_tile<D>(path + tc.base, tc.nvalid, stage);
    HMM_STAMP(13);
    if (!alone && tc.tile == 0) {
        if (ok2) grid_sum_parts(blockIdx.x, tps, ws, dsum, logprob_out, tc.seq);
        else if (threadIdx.x == 0) logprob_out[tc.seq] = __builtin_nan("");   // the wait for the tile maps ran out
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
    float P[D * D];
    double msum;
    chunk_aggregate<S, D, true>(row, pc.n, pc.first, Am, P, msum);
    float f[D], b[D];
    group_exchange<S, D, true>(P, lcpl, pc.c, start, f, b);
    float* fdst = WRITE_FILT ? filt + ((size_t)pc.seq * T + (size_t)pc.c * C::L) * D : nullptr;   // lane by lane, as in the apply kernel
    const double delta = smooth_chunk<S, D, WRITE_FILT>(row, pc.n, pc.first, Am, f, b, msum, fdst);
    const double total = group_sum(delta, lcpl);
    if (pc.first) out[pc.seq] = total;
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
    float P[D * D];
    double msum;
    chunk_aggregate<S, D, false>(const_cast<float*>(row), pc.n, pc.first, Am, P, msum);
    float v[D], unused[D];
    group_exchange<S, D, false>(P, lcpl, pc.c, start, v, unused);
    uint32_t bp[C::W], h, xs;
    const double osum = viterbi_chunk<D>(row, pc.n, pc.first, pc.last, Am, v, bp, h, xs);
    const double total = group_sum(osum, lcpl);
    if (pc.first) logprob_out[pc.seq] = total;
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
    float ms = 0.0f, rs = 0.0f;   // sums of at most L emission maxima / L removed exponents or offsets
#pragma unroll
    for (int k = 0; k < C::L; ++k) {
        if (k < n) {
            float ev[D];
            lds_read_vec<D>(row + k * D, ev);
            ms += emission<S, D>(ev);
            if (k == 0 && first) absorb<S, D>(P, Am, ev, true);
            else absorb<S, D>(P, Am, ev, false);
            if ((k & 3) == 3 || k == n - 1) rs += renorm<S, D * D>(P);
        }
    }
    return (double)ms + (double)rs * (S::is_max_plus ? 1.0 : 0.6931471805599453);
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

struct SmoothWs { size_t agg, fin, bout, part, xch, total; };
struct ViterbiWs { size_t agg, vin, bp, cmap, tmap, xend, part, xch, total; };

// Exchange region of the single-launch plan, in 32-bit words: [aggregates][parts][maps][error flag]
struct XchLayout { size_t agg, part, tmap, err, words; };
template <int D>
static XchLayout xch_layout(size_t nt) {
    XchLayout x;
    size_t o = 0;
    x.agg = o;  o += (nt * D * D + 1) / 2 * 2;   // keeps the doubles that follow 8-byte aligned
    x.part = o; o += 2 * nt;
    x.tmap = o; o += nt;
    x.err = o;  o += 1;
    x.words = o;
    return x;
}

template <int D>
static SmoothWs smooth_ws(long long T, int batch) {
    const size_t nt = (size_t)tiles_per_seq<D>(T) * batch;
    SmoothWs w;
    size_t o = 0;
    w.agg = o;   o = align_up(o + nt * D * D * sizeof(float), 256);
    w.fin = o;   o = align_up(o + nt * D * sizeof(float), 256);
    w.bout = o;  o = align_up(o + nt * D * sizeof(float), 256);
    w.part = o;  o = align_up(o + nt * sizeof(double), 256);
    w.xch = o;  o = align_up(o + xch_layout<D>(nt).words * sizeof(uint32_t), 256);
    w.total = o;
    return w;
}

template <int D>
static ViterbiWs viterbi_ws(long long T, int batch) {
    using C = SmallCfg<D>;
    const size_t nt = (size_t)tiles_per_seq<D>(T) * batch;
    ViterbiWs w;
    size_t o = 0;
    w.agg = o;   o = align_up(o + nt * D * D * sizeof(float), 256);
    w.vin = o;   o = align_up(o + nt * D * sizeof(float), 256);
    w.bp = o;    o = align_up(o + nt * C::NT * C::W * sizeof(uint32_t), 256);
    w.cmap = o;  o = align_up(o + nt * C::NT * sizeof(uint32_t), 256);
    w.tmap = o;  o = align_up(o + nt * sizeof(uint32_t), 256);
    w.xend = o;  o = align_up(o + nt * sizeof(uint32_t), 256);
    w.part = o;  o = align_up(o + nt * sizeof(double), 256);
    w.xch = o;  o = align_up(o + xch_layout<D>(nt).words * sizeof(uint32_t), 256);
    w.total = o;
    return w;
}

// How many workgroups of `kernel` the current device holds resident at once (cached per kernel).
template <int TAG, class K>
static long long resident_capacity(K kernel) {
    static long long cached = -1;
    if (cached >= 0) return cached;
    int dev = 0, ncu = 0, per_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, 256, 0) != hipSuccess) return 0;
    cached = (long long)ncu * per_cu;
    return cached;
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

// The two-filter plans for either operator: marginals + optional filtered + log evidence (SumProd),
// or max-marginals + optional per-step maximiser + log of the best joint weight (MaxPlus).
template <class S, int D>
static int two_filter(const SmallArgs& a, float* marg, float* filt, int32_t* argmax, double* out) {
    using C = SmallCfg<D>;
    constexpr bool MP = S::is_max_plus;
    const long long tps = tiles_per_seq<D>(a.T);
    const long long nt = tps * a.batch;
    if (nt > 0x7fffffffLL) return 2;
    const SmoothWs w = smooth_ws<D>(a.T, a.batch);
    if (a.ws_bytes < w.total) return 3;
    char* ws = static_cast<char*>(a.ws);
    float* agg = reinterpret_cast<float*>(ws + w.agg);
    float* fin = reinterpret_cast<float*>(ws + w.fin);
    float* bout = reinterpret_cast<float*>(ws + w.bout);
    double* part = reinterpret_cast<double*>(ws + w.part);
    uint32_t* xch = reinterpret_cast<uint32_t*>(ws + w.xch);
    hipStream_t st = a.stream;
    const dim3 grid((unsigned)nt), block(C::NT), seqs((unsigned)a.batch);
    const int itps = (int)tps;
    long long cap = 0;
    if constexpr (!MP) {
        if (filt) cap = resident_capacity<0>(sd_smooth_fused_kernel<S, D, true>);
    }
    if (!filt) cap = resident_capacity<(MP ? 5 : 1)>(sd_smooth_fused_kernel<S, D, false>);
    if (MP && filt) return 2;   // no filtered output is defined for the max-product plan
    const int lcpl = packed_log2_lanes<D>(a.T);
    if (!force_multi_launch() && lcpl >= 0) {
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
    // (no workgroup waits for another, so they need not be resident together) and no slot is cleared.
    if (!force_multi_launch() && (tps == 1 || (tps <= C::NT && nt <= cap))) {
        const XchLayout xl = xch_layout<D>((size_t)nt);
        FusedWs fw{reinterpret_cast<float*>(xch + xl.agg), reinterpret_cast<double*>(xch + xl.part), xch + xl.tmap,
                   xch + xl.err, spin_limit()};
        const int nwords = (int)xl.words;
        if (tps > 1)
            launch(MP ? "sd_clear_mm" : "sd_clear_sp", sd_clear_kernel<D>, dim3((nwords + 255) / 256), dim3(256), st, xch,
                   nwords);
        const char* name = MP ? "sd_maxprod_fused" : "sd_smooth_fused";
        if constexpr (!MP) {
            if (filt)
                launch(name, sd_smooth_fused_kernel<S, D, true>, grid, block, st, a.prior, a.A, a.ll, a.T, itps,
                       a.shared_model, marg, filt, argmax, out, fw);
        }
        if (!filt)
            launch(name, sd_smooth_fused_kernel<S, D, false>, grid, block, st, a.prior, a.A, a.ll, a.T, itps,
                   a.shared_model, marg, filt, argmax, out, fw);
    } else {
        launch(MP ? "sd_reduce_mp" : "sd_reduce_sp", sd_reduce_kernel<S, D>, grid, block, st, a.A, a.ll, a.T, itps,
               a.shared_model, agg);
        launch(MP ? "sd_carry_mm" : "sd_carry_sp", sd_carry_kernel<S, D, true>, seqs, block, st, a.prior, itps,
               a.shared_model, agg, fin, bout);
        const char* name = MP ? "sd_maxprod_apply" : "sd_smooth_apply";
        if constexpr (!MP) {
            if (filt)
                launch(name, sd_smooth_apply_kernel<S, D, true>, grid, block, st, a.A, a.ll, a.T, itps, a.shared_model,
                       fin, bout, marg, filt, argmax, part);
        }
        if (!filt)
            launch(name, sd_smooth_apply_kernel<S, D, false>, grid, block, st, a.A, a.ll, a.T, itps, a.shared_model,
                   fin, bout, marg, filt, argmax, part);
        launch("sd_finalize", sd_finalize_kernel<D>, seqs, dim3(256), st, part, itps, out);
    }
    return hipGetLastError() == hipSuccess ? 0 : 4;
}

template <int D>
int SmallD<D>::smooth(const SmallArgs& a, float* marg, float* filt, double* loglik_out) {
    return two_filter<SumProd, D>(a, marg, filt, nullptr, loglik_out);
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
    double* part = reinterpret_cast<double*>(ws + w.part);
    uint32_t* xch = reinterpret_cast<uint32_t*>(ws + w.xch);
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
    const long long cap = resident_capacity<2>(sd_viterbi_fused_kernel<D>);
    if (!force_multi_launch() && (tps == 1 || (tps <= C::NT && nt <= cap))) {   // one tile per sequence: see two_filter
        const XchLayout xl = xch_layout<D>((size_t)nt);
        FusedWs fw{reinterpret_cast<float*>(xch + xl.agg), reinterpret_cast<double*>(xch + xl.part), xch + xl.tmap,
                   xch + xl.err, spin_limit()};
        const int nwords = (int)xl.words;
        if (tps > 1) launch("sd_clear_mp", sd_clear_kernel<D>, dim3((nwords + 255) / 256), dim3(256), st, xch, nwords);
        launch("sd_viterbi_fused", sd_viterbi_fused_kernel<D>, grid, block, st, a.prior, a.A, a.ll, a.T, itps,
               a.shared_model, path, logprob_out, fw);
    } else {
        launch("sd_reduce_mp", sd_reduce_kernel<MaxPlus, D>, grid, block, st, a.A, a.ll, a.T, itps, a.shared_model, agg);
        launch("sd_carry_mp", sd_carry_kernel<MaxPlus, D, false>, seqs, block, st, a.prior, itps, a.shared_model, agg, vin,
               static_cast<float*>(nullptr));
        launch("sd_viterbi_forward", sd_viterbi_forward_kernel<D>, grid, block, st, a.A, a.ll, a.T, itps, a.shared_model,
               vin, bp, cmap, tmap, part);
        launch("sd_viterbi_suffix", sd_viterbi_suffix_kernel<D>, seqs, block, st, tmap, itps, xend, part, logprob_out);
        launch("sd_viterbi_path", sd_viterbi_path_kernel<D>, grid, block, st, a.T, itps, bp, cmap, xend, path);
    }
    return hipGetLastError() == hipSuccess ? 0 : 4;
}

template <int D>
size_t SmallD<D>::element_ws_bytes(long long T, int batch) {
    const size_t nt = (size_t)tiles_per_seq<D>(T) * batch;
    return align_up(nt * D * D * sizeof(float), 256) + align_up(nt * sizeof(double), 256);
}

template <int D>
int SmallD<D>::block_element(const SmallArgs& a, int max_product, float* element, double* log_scale) {
    using C = SmallCfg<D>;
    const long long tps = tiles_per_seq<D>(a.T);
    const long long nt = tps * a.batch;
    if (nt > 0x7fffffffLL) return 2;
    if (a.ws_bytes < element_ws_bytes(a.T, a.batch)) return 3;
    char* ws = static_cast<char*>(a.ws);
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

#ifdef HMM_PHASE_STAMPS
extern "C" int hmm_debug_read_stamps(unsigned long long* host_dst) {
    return (int)hipMemcpyFromSymbol(host_dst, HIP_SYMBOL(g_stamps), sizeof(unsigned long long) * 1024 * 16);
}
#endif

}  // namespace hmm
