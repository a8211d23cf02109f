// Small state spaces (D <= 8): every D x D element lives in the registers of one lane.
//
// Chunked all-prefix-sums over time ("block-wise elements", Sec. V-B): a lane owns L consecutive
// time steps, a 256-lane workgroup owns a tile of 256*L steps that it stages through LDS with
// coalesced global accesses.  Elements a_{k-1:k} = psi_k are never written to memory: they are
// rebuilt from the transition matrix and one log-likelihood row whenever they are combined
// (element initialisation of Algorithms 3 and 5 fused into the scan).
//
// Multi-launch pipeline (no inter-workgroup waiting anywhere):
//   smoother : reduce (tile aggregates) -> carry (per-tile forward/backward carries)
//              -> apply (forward + reversed scan inside the tile, marginals) -> finalize (log Z)
//   Viterbi  : reduce -> carry -> forward (back-pointers, chunk maps) -> suffix (state at each
//              tile's end by composing back-pointer maps right to left, log-probability) -> path
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "semiring.hpp"
#include "small_d.hpp"

namespace hmm {

template <int D>
struct SmallCfg {
    static constexpr int NT = 256;                    // lanes per workgroup
    static constexpr int NW = NT / 64;                // wavefronts per workgroup
    static constexpr int L = (D <= 4) ? 16 : 8;       // time steps per lane
    static constexpr int TILE = NT * L;               // time steps per workgroup
    static constexpr int ROW = L * D;                 // floats per lane in LDS
    static constexpr int VEC = (D % 4 == 0) ? 4 : 1;  // floats per global/LDS access
    static constexpr int PAD = (D % 4 == 0) ? 4 : ((D % 2 == 0) ? 2 : 1);
    static constexpr int STRIDE = ROW + PAD;          // odd in units of PAD: conflict-free rows
    static constexpr int LDS_FLOATS = NT * STRIDE;
    // back-pointer packing
    static constexpr int BITS = (D <= 2) ? 1 : (D <= 4) ? 2 : 3;
    static constexpr uint32_t MASK = (1u << BITS) - 1u;
    static constexpr int STEP_BITS = D * BITS;
    static constexpr int SPW = 32 / STEP_BITS;        // steps per 32-bit word
    static constexpr int W = (L + SPW - 1) / SPW;     // words per lane
    static constexpr int PSTRIDE = L + 1;             // path staging row (ints)
};

struct TileCoord {
    int seq;         // sequence index in the batch
    int tile;        // tile index inside the sequence
    int nvalid;      // valid time steps in this tile (1..TILE)
    long long base;  // global step index of the tile's first step: seq*T + tile*TILE
};

template <int D>
HMM_DEV TileCoord tile_coord(long long T, int tps) {
    using C = SmallCfg<D>;
    TileCoord c;
    c.seq = blockIdx.x / tps;
    c.tile = blockIdx.x - c.seq * tps;
    const long long s0 = (long long)c.tile * C::TILE;
    const long long rem = T - s0;
    c.nvalid = rem < C::TILE ? (int)rem : C::TILE;
    c.base = (long long)c.seq * T + s0;
    return c;
}

// ---------------------------------------------------------------------------------------------
// Tile <-> LDS staging (coalesced global side, one padded row per lane on the LDS side)
template <int D>
HMM_DEV void load_tile(const float* __restrict__ g, int nvalid_steps, float* lds) {
    using C = SmallCfg<D>;
    const int nfl = nvalid_steps * D;
    if constexpr (C::VEC == 4) {
        const float4* g4 = reinterpret_cast<const float4*>(g);
#pragma unroll
        for (int it = 0; it < C::ROW / 4; ++it) {
            const int v = it * C::NT + threadIdx.x;
            const int fl = v * 4;
            if (fl < nfl) {
                const float4 x = g4[v];
                const int owner = fl / C::ROW;
                *reinterpret_cast<float4*>(lds + owner * C::STRIDE + (fl - owner * C::ROW)) = x;
            }
        }
    } else {
#pragma unroll 8
        for (int it = 0; it < C::ROW; ++it) {
            const int fl = it * C::NT + threadIdx.x;
            if (fl < nfl) {
                const int owner = fl / C::ROW;
                lds[owner * C::STRIDE + (fl - owner * C::ROW)] = g[fl];
            }
        }
    }
}

template <int D>
HMM_DEV void store_tile(float* __restrict__ g, int nvalid_steps, const float* lds) {
    using C = SmallCfg<D>;
    const int nfl = nvalid_steps * D;
    if constexpr (C::VEC == 4) {
        float4* g4 = reinterpret_cast<float4*>(g);
#pragma unroll
        for (int it = 0; it < C::ROW / 4; ++it) {
            const int v = it * C::NT + threadIdx.x;
            const int fl = v * 4;
            if (fl < nfl) {
                const int owner = fl / C::ROW;
                g4[v] = *reinterpret_cast<const float4*>(lds + owner * C::STRIDE + (fl - owner * C::ROW));
            }
        }
    } else {
#pragma unroll 8
        for (int it = 0; it < C::ROW; ++it) {
            const int fl = it * C::NT + threadIdx.x;
            if (fl < nfl) {
                const int owner = fl / C::ROW;
                g[fl] = lds[owner * C::STRIDE + (fl - owner * C::ROW)];
            }
        }
    }
}

template <int D>
HMM_DEV void lds_read_vec(const float* p, float (&v)[D]) {
    if constexpr (D % 4 == 0) {
#pragma unroll
        for (int q = 0; q < D / 4; ++q) {
            const float4 x = *reinterpret_cast<const float4*>(p + 4 * q);
            v[4 * q] = x.x; v[4 * q + 1] = x.y; v[4 * q + 2] = x.z; v[4 * q + 3] = x.w;
        }
    } else {
#pragma unroll
        for (int j = 0; j < D; ++j) v[j] = p[j];
    }
}

template <int D>
HMM_DEV void lds_write_vec(float* p, const float (&v)[D]) {
    if constexpr (D % 4 == 0) {
#pragma unroll
        for (int q = 0; q < D / 4; ++q)
            *reinterpret_cast<float4*>(p + 4 * q) = make_float4(v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]);
    } else {
#pragma unroll
        for (int j = 0; j < D; ++j) p[j] = v[j];
    }
}

// Transition matrix in the operator's domain: probabilities for SumProd, logarithms for MaxPlus.
template <class S, int D>
HMM_DEV void load_model(const float* __restrict__ A, float (&Am)[D * D]) {
#pragma unroll
    for (int e = 0; e < D * D; ++e) {
        const float a = A[e];
        Am[e] = S::is_max_plus ? logf(a) : a;
    }
}

// Emission factor of one step in the operator's domain.  SumProd: e_k(j) = exp(ll_k(j) - m_k)
// with m_k = max_j ll_k(j) (returned); MaxPlus: ll_k itself (returns 0).
template <class S, int D>
HMM_DEV float emission(float (&ev)[D]) {
    if constexpr (S::is_max_plus) {
        return 0.0f;
    } else {
        float m = max_of(ev);
        const float ms = (m == -INFINITY) ? 0.0f : m;
#pragma unroll
        for (int j = 0; j < D; ++j) ev[j] = __expf(ev[j] - ms);
        return m;
    }
}

// One element absorbed on the right of a chunk aggregate: P <- P (op) psi_k, with
// psi_k(i,j) = Am(i,j) (x) ev(j); the sequence's first element has no transition part.
template <class S, int D>
HMM_DEV void absorb(float (&P)[D * D], const float (&Am)[D * D], const float (&ev)[D], bool no_transition) {
    if (no_transition) {
#pragma unroll
        for (int i = 0; i < D; ++i)
#pragma unroll
            for (int j = 0; j < D; ++j) P[i * D + j] = S::times(P[i * D + j], ev[j]);
    } else {
        float Z[D * D];
        mat_mul<S, D>(P, Am, Z);
#pragma unroll
        for (int i = 0; i < D; ++i)
#pragma unroll
            for (int j = 0; j < D; ++j) P[i * D + j] = S::times(Z[i * D + j], ev[j]);
    }
}

// Aggregate of the lane's chunk: a_{k0-1:k0} (op) ... (op) a_{k1-2:k1-1} over its n valid steps.
// With STORE_E the emission factors replace the log-likelihoods in LDS and the sum of the
// per-step maxima m_k is returned through msum.
template <class S, int D, bool STORE_E>
HMM_DEV void chunk_aggregate(float* row, int n, bool first, const float (&Am)[D * D], float (&P)[D * D],
                             double& msum) {
    using C = SmallCfg<D>;
    mat_identity<S, D>(P);
    double ms = 0.0;
#pragma unroll
    for (int k = 0; k < C::L; ++k) {
        if (k < n) {
            float ev[D];
            lds_read_vec<D>(row + k * D, ev);
            const float m = emission<S, D>(ev);
            if constexpr (STORE_E) {
                lds_write_vec<D>(row + k * D, ev);
                ms += (double)m;
            }
            absorb<S, D>(P, Am, ev, k == 0 && first);
            if ((k & 3) == 3) renorm<S, D * D>(P);
        }
    }
    msum = ms;
}

// ---------------------------------------------------------------------------------------------
// Wave-level scans of chunk aggregates (Kogge-Stone over the 64 lanes of a wavefront)
template <class S, int D>
HMM_DEV void wave_scan_prefix(float (&Q)[D * D]) {   // Q_t <- P_0 (op) ... (op) P_t
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        float Pn[D * D], Z[D * D];
#pragma unroll
        for (int e = 0; e < D * D; ++e) Pn[e] = __shfl_up(Q[e], d, 64);
        mat_mul<S, D>(Pn, Q, Z);
        renorm<S, D * D>(Z);
        const bool take = lane >= d;
#pragma unroll
        for (int e = 0; e < D * D; ++e) Q[e] = take ? Z[e] : Q[e];
    }
}

template <class S, int D>
HMM_DEV void wave_scan_suffix(float (&R)[D * D]) {   // R_t <- P_t (op) ... (op) P_63
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        float Pn[D * D], Z[D * D];
#pragma unroll
        for (int e = 0; e < D * D; ++e) Pn[e] = __shfl_down(R[e], d, 64);
        mat_mul<S, D>(R, Pn, Z);
        renorm<S, D * D>(Z);
        const bool take = lane + d < 64;
#pragma unroll
        for (int e = 0; e < D * D; ++e) R[e] = take ? Z[e] : R[e];
    }
}

// Per-lane carries inside a workgroup.  Given each lane's chunk aggregate P, the vector entering
// the workgroup from the left (cin_f) and, if BWD, the vector entering from the right (cin_b):
//   fin  = cin_f (op) P_0 (op) ... (op) P_{t-1}          (forward potential just before the chunk)
//   bout = P_{t+1} (op) ... (op) P_{NT-1} (op) cin_b      (backward potential at the chunk's last step)
// wagg: NW*D*D floats of LDS.  If tile_agg is non-null, lane 0 also writes the workgroup aggregate.
template <class S, int D, bool FWD, bool BWD>
HMM_DEV void block_exchange(const float (&P)[D * D], const float (&cin_f)[D], const float (&cin_b)[D],
                            float (&fin)[D], float (&bout)[D], float* wagg, float* tile_agg) {
    using C = SmallCfg<D>;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    float Q[D * D];
#pragma unroll
    for (int e = 0; e < D * D; ++e) Q[e] = P[e];
    wave_scan_prefix<S, D>(Q);
    if (lane == 63) {
#pragma unroll
        for (int e = 0; e < D * D; ++e) wagg[wave * D * D + e] = Q[e];
    }
    __syncthreads();
    if constexpr (FWD) {
        float fw[D];
#pragma unroll
        for (int j = 0; j < D; ++j) fw[j] = cin_f[j];
#pragma unroll
        for (int w = 0; w < C::NW - 1; ++w) {
            if (w < wave) {
                float Wm[D * D], r[D];
#pragma unroll
                for (int e = 0; e < D * D; ++e) Wm[e] = wagg[w * D * D + e];
                vec_mat<S, D>(fw, Wm, r);
                renorm<S, D>(r);
#pragma unroll
                for (int j = 0; j < D; ++j) fw[j] = r[j];
            }
        }
        float Qp[D * D], r[D];
#pragma unroll
        for (int e = 0; e < D * D; ++e) Qp[e] = __shfl_up(Q[e], 1, 64);
        vec_mat<S, D>(fw, Qp, r);
#pragma unroll
        for (int j = 0; j < D; ++j) fin[j] = (lane == 0) ? fw[j] : r[j];
    }
    if constexpr (BWD) {
        float R[D * D];
#pragma unroll
        for (int e = 0; e < D * D; ++e) R[e] = P[e];
        wave_scan_suffix<S, D>(R);
        float bw[D];
#pragma unroll
        for (int j = 0; j < D; ++j) bw[j] = cin_b[j];
#pragma unroll
        for (int w = C::NW - 1; w > 0; --w) {
            if (w > wave) {
                float Wm[D * D], r[D];
#pragma unroll
                for (int e = 0; e < D * D; ++e) Wm[e] = wagg[w * D * D + e];
                mat_vec<S, D>(Wm, bw, r);
                renorm<S, D>(r);
#pragma unroll
                for (int j = 0; j < D; ++j) bw[j] = r[j];
            }
        }
        float Rn[D * D], r[D];
#pragma unroll
        for (int e = 0; e < D * D; ++e) Rn[e] = __shfl_down(R[e], 1, 64);
        mat_vec<S, D>(Rn, bw, r);
#pragma unroll
        for (int j = 0; j < D; ++j) bout[j] = (lane == 63) ? bw[j] : r[j];
    }
    if (tile_agg != nullptr && threadIdx.x == 0) {
        float X[D * D], Y[D * D], Z[D * D];
#pragma unroll
        for (int e = 0; e < D * D; ++e) X[e] = wagg[e];
#pragma unroll
        for (int w = 1; w < C::NW; ++w) {
#pragma unroll
            for (int e = 0; e < D * D; ++e) Y[e] = wagg[w * D * D + e];
            mat_mul<S, D>(X, Y, Z);
            renorm<S, D * D>(Z);
#pragma unroll
            for (int e = 0; e < D * D; ++e) X[e] = Z[e];
        }
#pragma unroll
        for (int e = 0; e < D * D; ++e) tile_agg[e] = X[e];
    }
}

// Ordered sum of one double per lane over the workgroup; result valid in thread 0.
HMM_DEV double block_sum(double v, double* scratch /* NW doubles */) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_down(v, d, 64);
    if ((threadIdx.x & 63) == 0) scratch[threadIdx.x >> 6] = v;
    __syncthreads();
    double s = 0.0;
    if (threadIdx.x == 0) {
        for (int w = 0; w < (int)(blockDim.x >> 6); ++w) s += scratch[w];
    }
    return s;
}

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
    float P[D * D];
    double msum;
    chunk_aggregate<S, D, false>(lds + threadIdx.x * C::STRIDE, n, tc.tile == 0 && threadIdx.x == 0, Am, P, msum);
    float dummy_in[D], dummy_out[D];
#pragma unroll
    for (int j = 0; j < D; ++j) dummy_in[j] = 0.0f;
    block_exchange<S, D, false, false>(P, dummy_in, dummy_in, dummy_out, dummy_out, wagg,
                                       agg + (size_t)blockIdx.x * D * D);
}

// =============================================================================================
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
    block_exchange<S, D, true, BWD>(P, cf, cb, f, b, wagg, nullptr);
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
            // the prior itself is handed over unscaled; everything after it is renormalised
            renorm<S, D>(g);
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

// =============================================================================================
// Kernel 3 (smoother): forward scan, reversed scan and marginals inside a tile
template <int D, bool WRITE_FILT>
__global__ __launch_bounds__(256) void sd_smooth_apply_kernel(const float* __restrict__ A,
                                                              const float* __restrict__ ll, long long T, int tps,
                                                              int shared_model, const float* __restrict__ fin_g,
                                                              const float* __restrict__ bout_g,
                                                              float* __restrict__ marg, float* __restrict__ filt,
                                                              double* __restrict__ part) {
    using C = SmallCfg<D>;
    using S = SumProd;
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
    block_exchange<S, D, true, true>(P, cf, cb, f, b, wagg, nullptr);

    // ---- forward: a_{0:k} for the lane's steps, kept in registers (Theorem 1)
    float F[C::L][D];
    if (!first) {   // the prior is used as given; every other carry is rescaled to sum to one
        const float inv = 1.0f / sum_of(f);
#pragma unroll
        for (int j = 0; j < D; ++j) f[j] *= inv;
    }
    int exsum = 0;
    float s_last = 1.0f;
#pragma unroll
    for (int k = 0; k < C::L; ++k) {
        if (k < n) {
            float ev[D], g[D];
            lds_read_vec<D>(row + k * D, ev);
            if (k == 0 && first) {
#pragma unroll
                for (int j = 0; j < D; ++j) g[j] = f[j] * ev[j];
            } else {
                vec_mat<S, D>(f, Am, g);
#pragma unroll
                for (int j = 0; j < D; ++j) g[j] *= ev[j];
            }
            const float s = sum_of(g);
            const int ex = __builtin_amdgcn_frexp_expf(s);
#pragma unroll
            for (int j = 0; j < D; ++j) f[j] = ldexpf(g[j], -ex);
            exsum += ex;
            s_last = ldexpf(s, -ex);
#pragma unroll
            for (int j = 0; j < D; ++j) F[k][j] = f[j];
            if constexpr (WRITE_FILT) {
                const float inv = __builtin_amdgcn_rcpf(s_last);
                float* dst = filt + (tc.base + (long long)threadIdx.x * C::L + k) * D;
#pragma unroll
                for (int j = 0; j < D; ++j) dst[j] = f[j] * inv;
            }
        }
    }
    // chunk-local log evidence: log p(y_chunk | y_before) = sum m_k + ln2 * sum ex_k + log sum_j f_end(j)
    double delta = 0.0;
    if (n > 0) delta = msum + 0.6931471805599453 * (double)exsum + log((double)s_last);
    const double tile_delta = block_sum(delta, dsum);
    if (threadIdx.x == 0) part[blockIdx.x] = tile_delta;

    // ---- backward: a_{k:T+1} (Theorem 2) and the marginal f_k b_k / Z_k
    renorm<S, D>(b);
#pragma unroll
    for (int k = C::L - 1; k >= 0; --k) {
        if (k < n) {
            float ev[D], gam[D];
            lds_read_vec<D>(row + k * D, ev);
#pragma unroll
            for (int j = 0; j < D; ++j) gam[j] = F[k][j] * b[j];
            const float inv = __builtin_amdgcn_rcpf(sum_of(gam));
#pragma unroll
            for (int j = 0; j < D; ++j) gam[j] *= inv;
            lds_write_vec<D>(row + k * D, gam);
            if (k > 0) {
                float t[D], r[D];
#pragma unroll
                for (int j = 0; j < D; ++j) t[j] = ev[j] * b[j];
                mat_vec<S, D>(Am, t, r);
                renorm<S, D>(r);
#pragma unroll
                for (int j = 0; j < D; ++j) b[j] = r[j];
            }
        }
    }
    __syncthreads();
    store_tile<D>(marg + tc.base * D, tc.nvalid, lds);
}

// Kernel 4 (both): out[seq] = ordered sum of the tile partials of one sequence.
__global__ __launch_bounds__(256) void sd_finalize_kernel(const double* __restrict__ part, int tps,
                                                          double* __restrict__ out) {
    __shared__ double dsum[4];
    const int seq = blockIdx.x;
    double acc = 0.0;
    for (int t = threadIdx.x; t < tps; t += blockDim.x) acc += part[(size_t)seq * tps + t];
    const double s = block_sum(acc, dsum);
    if (threadIdx.x == 0) out[seq] = s;
}

// =============================================================================================
// Viterbi back-pointer maps: a map [D] -> [D] packed BITS per entry into one 32-bit word.
template <int D>
HMM_DEV uint32_t map_identity() {
    using C = SmallCfg<D>;
    uint32_t m = 0;
#pragma unroll
    for (int j = 0; j < D; ++j) m |= (uint32_t)j << (j * C::BITS);
    return m;
}

template <int D>
HMM_DEV uint32_t map_apply(uint32_t g, uint32_t x) {
    using C = SmallCfg<D>;
    return (g >> (x * C::BITS)) & C::MASK;
}

// (g o h)(j) = g(h(j)): first h, then g
template <int D>
HMM_DEV uint32_t map_compose(uint32_t g, uint32_t h) {
    using C = SmallCfg<D>;
    uint32_t r = 0;
#pragma unroll
    for (int j = 0; j < D; ++j) {
        const uint32_t hj = (h >> (j * C::BITS)) & C::MASK;
        r |= ((g >> (hj * C::BITS)) & C::MASK) << (j * C::BITS);
    }
    return r;
}

constexpr uint32_t MAP_FINAL_FLAG = 0x80000000u;   // lane holds the sequence's last step
constexpr int MAP_FINAL_SHIFT = 24;                // ... and x*_T is stored here
constexpr uint32_t MAP_BODY = 0x00ffffffu;

// Reversed all-prefix-sums under composition over the workgroup's lanes:
// excl = g_{t+1} o ... o g_{NT-1} for every lane; returns g_0 o ... o g_{NT-1} (valid in every lane).
template <int D>
HMM_DEV uint32_t block_map_suffix(uint32_t g, uint32_t& excl, uint32_t* wmaps /* NW words */) {
    using C = SmallCfg<D>;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    uint32_t G = g;   // inclusive: g_t o ... o g_63 within the wave
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = __shfl_down(G, d, 64);
        const uint32_t c = map_compose<D>(G, o);
        G = (lane + d < 64) ? c : G;
    }
    if (lane == 0) wmaps[wave] = G;
    __syncthreads();
    uint32_t tail = map_identity<D>();   // composition of the waves after mine
#pragma unroll
    for (int w = C::NW - 1; w > 0; --w)
        if (w > wave) tail = map_compose<D>(wmaps[w], tail);
    uint32_t nxt = __shfl_down(G, 1, 64);
    nxt = (lane == 63) ? map_identity<D>() : nxt;
    excl = map_compose<D>(nxt, tail);
    uint32_t total = map_identity<D>();
#pragma unroll
    for (int w = C::NW - 1; w >= 0; --w) total = map_compose<D>(wmaps[w], total);
    return total;
}

// Kernel V3: forward max-plus scan inside the tile with back-pointers u_{k-1}(x_k) (Sec. IV-A),
// each lane's chunk map x_{k1-1} -> x_{k0-1}, the tile's map, and the chunk-local log-probability.
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
    block_exchange<S, D, true, false>(P, cf, cf, v, unused, wagg, nullptr);
    if (!first) renorm<S, D>(v);   // log prior is used as given; other carries start at max 0

    uint32_t bp[C::W];
#pragma unroll
    for (int w = 0; w < C::W; ++w) bp[w] = 0u;
    double osum = 0.0;
#pragma unroll
    for (int k = 0; k < C::L; ++k) {
        if (k < n) {
            float lk[D], g[D];
            lds_read_vec<D>(row + k * D, lk);
            uint32_t word = 0u;
            if (k == 0 && first) {
#pragma unroll
                for (int j = 0; j < D; ++j) {
                    g[j] = v[j] + lk[j];
                    word |= (uint32_t)j << (j * C::BITS);
                }
            } else {
#pragma unroll
                for (int j = 0; j < D; ++j) {
                    float best = v[0] + Am[j];
                    uint32_t arg = 0u;
#pragma unroll
                    for (int i = 1; i < D; ++i) {
                        const float c = v[i] + Am[i * D + j];
                        const bool gt = c > best;      // strict: the lowest index wins ties
                        best = gt ? c : best;
                        arg = gt ? (uint32_t)i : arg;
                    }
                    g[j] = best + lk[j];
                    word |= arg << (j * C::BITS);
                }
            }
            bp[k / C::SPW] |= word << ((k % C::SPW) * C::STEP_BITS);
            osum += (double)renorm<S, D>(g);
#pragma unroll
            for (int j = 0; j < D; ++j) v[j] = g[j];
        }
    }
    const double tile_delta = block_sum(n > 0 ? osum : 0.0, dsum);
    if (threadIdx.x == 0) part[blockIdx.x] = tile_delta;

    // chunk map h: x at the chunk's last step -> x at the step before the chunk
    uint32_t h = map_identity<D>();
#pragma unroll
    for (int k = C::L - 1; k >= 0; --k) {
        if (k < n) {
            const uint32_t u = (bp[k / C::SPW] >> ((k % C::SPW) * C::STEP_BITS)) & ((1u << C::STEP_BITS) - 1u);
            h = map_compose<D>(u, h);
        }
    }
    uint32_t stored = h;
    if (last) {   // x*_T = argmax V_T: every later state maps to h(x*_T)
        uint32_t xs = 0u;
        float best = v[0];
#pragma unroll
        for (int j = 1; j < D; ++j) {
            const bool gt = v[j] > best;
            best = gt ? v[j] : best;
            xs = gt ? (uint32_t)j : xs;
        }
        const uint32_t c = map_apply<D>(h, xs);
        h = 0u;
#pragma unroll
        for (int j = 0; j < D; ++j) h |= c << (j * C::BITS);
        stored = h | MAP_FINAL_FLAG | (xs << MAP_FINAL_SHIFT);
    }
    const size_t gl = (size_t)blockIdx.x * C::NT + threadIdx.x;
#pragma unroll
    for (int w = 0; w < C::W; ++w) bp_g[gl * C::W + w] = bp[w];
    cmap_g[gl] = stored;
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
#pragma unroll
    for (int k = C::L - 1; k >= 0; --k) {
        if (k < n) {
            stage[threadIdx.x * C::PSTRIDE + k] = (int32_t)x;
            if (!(k == 0 && first)) {
                const uint32_t u = bp[k / C::SPW] >> ((k % C::SPW) * C::STEP_BITS);
                x = map_apply<D>(u, x);
            }
        }
    }
    __syncthreads();
    int32_t* dst = path + tc.base;
#pragma unroll
    for (int it = 0; it < C::L; ++it) {
        const int s = it * C::NT + threadIdx.x;
        if (s < tc.nvalid) dst[s] = stage[(s / C::L) * C::PSTRIDE + (s % C::L)];
    }
}

// =============================================================================================
// Host side
static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

template <int D>
static long long tiles_per_seq(long long T) {
    return (T + SmallCfg<D>::TILE - 1) / SmallCfg<D>::TILE;
}

struct SmoothWs { size_t agg, fin, bout, part, total; };
struct ViterbiWs { size_t agg, vin, bp, cmap, tmap, xend, part, total; };

template <int D>
static SmoothWs smooth_ws(long long T, int batch) {
    const size_t nt = (size_t)tiles_per_seq<D>(T) * batch;
    SmoothWs w;
    size_t o = 0;
    w.agg = o;  o = align_up(o + nt * D * D * sizeof(float), 256);
    w.fin = o;  o = align_up(o + nt * D * sizeof(float), 256);
    w.bout = o; o = align_up(o + nt * D * sizeof(float), 256);
    w.part = o; o = align_up(o + nt * sizeof(double), 256);
    w.total = o;
    return w;
}

template <int D>
static ViterbiWs viterbi_ws(long long T, int batch) {
    using C = SmallCfg<D>;
    const size_t nt = (size_t)tiles_per_seq<D>(T) * batch;
    ViterbiWs w;
    size_t o = 0;
    w.agg = o;  o = align_up(o + nt * D * D * sizeof(float), 256);
    w.vin = o;  o = align_up(o + nt * D * sizeof(float), 256);
    w.bp = o;   o = align_up(o + nt * C::NT * C::W * sizeof(uint32_t), 256);
    w.cmap = o; o = align_up(o + nt * C::NT * sizeof(uint32_t), 256);
    w.tmap = o; o = align_up(o + nt * sizeof(uint32_t), 256);
    w.xend = o; o = align_up(o + nt * sizeof(uint32_t), 256);
    w.part = o; o = align_up(o + nt * sizeof(double), 256);
    w.total = o;
    return w;
}

template <int D>
static int smooth_impl(const SmallArgs& a, float* marg, float* filt, double* loglik_out) {
    using C = SmallCfg<D>;
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
    hipStream_t st = a.stream;
    sd_reduce_kernel<SumProd, D><<<dim3((unsigned)nt), dim3(C::NT), 0, st>>>(a.A, a.ll, a.T, (int)tps, a.shared_model, agg);
    sd_carry_kernel<SumProd, D, true><<<dim3(a.batch), dim3(C::NT), 0, st>>>(a.prior, (int)tps, a.shared_model, agg, fin, bout);
    if (filt)
        sd_smooth_apply_kernel<D, true><<<dim3((unsigned)nt), dim3(C::NT), 0, st>>>(a.A, a.ll, a.T, (int)tps, a.shared_model, fin, bout, marg, filt, part);
    else
        sd_smooth_apply_kernel<D, false><<<dim3((unsigned)nt), dim3(C::NT), 0, st>>>(a.A, a.ll, a.T, (int)tps, a.shared_model, fin, bout, marg, nullptr, part);
    sd_finalize_kernel<<<dim3(a.batch), dim3(256), 0, st>>>(part, (int)tps, loglik_out);
    return hipGetLastError() == hipSuccess ? 0 : 4;
}

template <int D>
static int viterbi_impl(const SmallArgs& a, int32_t* path, double* logprob_out) {
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
    hipStream_t st = a.stream;
    sd_reduce_kernel<MaxPlus, D><<<dim3((unsigned)nt), dim3(C::NT), 0, st>>>(a.A, a.ll, a.T, (int)tps, a.shared_model, agg);
    sd_carry_kernel<MaxPlus, D, false><<<dim3(a.batch), dim3(C::NT), 0, st>>>(a.prior, (int)tps, a.shared_model, agg, vin, nullptr);
    sd_viterbi_forward_kernel<D><<<dim3((unsigned)nt), dim3(C::NT), 0, st>>>(a.A, a.ll, a.T, (int)tps, a.shared_model, vin, bp, cmap, tmap, part);
    sd_viterbi_suffix_kernel<D><<<dim3(a.batch), dim3(C::NT), 0, st>>>(tmap, (int)tps, xend, part, logprob_out);
    sd_viterbi_path_kernel<D><<<dim3((unsigned)nt), dim3(C::NT), 0, st>>>(a.T, (int)tps, bp, cmap, xend, path);
    return hipGetLastError() == hipSuccess ? 0 : 4;
}

#define HMM_DISPATCH_SMALL_D(D_, EXPR)          \
    switch (D_) {                               \
        case 1: { constexpr int DD = 1; EXPR; } \
        case 2: { constexpr int DD = 2; EXPR; } \
        case 3: { constexpr int DD = 3; EXPR; } \
        case 4: { constexpr int DD = 4; EXPR; } \
        case 5: { constexpr int DD = 5; EXPR; } \
        case 6: { constexpr int DD = 6; EXPR; } \
        case 7: { constexpr int DD = 7; EXPR; } \
        case 8: { constexpr int DD = 8; EXPR; } \
        default: break;                         \
    }

size_t small_d_smooth_ws_bytes(int D, long long T, int batch) {
    HMM_DISPATCH_SMALL_D(D, return smooth_ws<DD>(T, batch).total)
    return 0;
}

size_t small_d_viterbi_ws_bytes(int D, long long T, int batch) {
    HMM_DISPATCH_SMALL_D(D, return viterbi_ws<DD>(T, batch).total)
    return 0;
}

int small_d_smooth(int D, const SmallArgs& a, float* marg, float* filt, double* loglik_out) {
    HMM_DISPATCH_SMALL_D(D, return smooth_impl<DD>(a, marg, filt, loglik_out))
    return 2;
}

int small_d_viterbi(int D, const SmallArgs& a, int32_t* path, double* logprob_out) {
    HMM_DISPATCH_SMALL_D(D, return viterbi_impl<DD>(a, path, logprob_out))
    return 2;
}

}  // namespace hmm
