// Device-side building blocks of the register-resident path (D <= 8): every D x D element lives
// in the registers of one lane.
//
// Chunked all-prefix-sums over time ("block-wise elements", Sec. V-B): a lane owns L consecutive
// time steps, a 256-lane workgroup owns a tile of 256*L steps that it stages through LDS with
// coalesced global accesses.  Elements a_{k-1:k} = psi_k are never written to memory: they are
// rebuilt from the transition matrix and one log-likelihood row whenever they are combined
// (the element initialisation of Algorithms 3 and 5 fused into the scan).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "semiring.hpp"

namespace hmm {

template <int D>
struct SmallCfg {
    static constexpr int NT = 256;                    // lanes per workgroup
    static constexpr int NW = NT / 64;                // wavefronts per workgroup
    static constexpr int L = (D <= 4) ? 16 : 8;       // time steps per lane
    static constexpr int TILE = NT * L;               // time steps per workgroup
    static constexpr int ROW = L * D;                 // floats per lane in LDS
    static constexpr int VEC = (D % 4 == 0) ? 4 : 1;  // floats per global access
    static constexpr int PAD = (D % 4 == 0) ? 4 : ((D % 2 == 0) ? 2 : 1);
    static constexpr int STRIDE = ROW + PAD;          // odd in units of PAD: conflict-free rows
    static constexpr int LDS_FLOATS = NT * STRIDE;
    // back-pointer packing
    static constexpr int BITS = (D <= 2) ? 1 : (D <= 4) ? 2 : 3;
    static constexpr uint32_t MASK = (1u << BITS) - 1u;
    static constexpr int STEP_BITS = D * BITS;
    static constexpr uint32_t STEP_MASK = (STEP_BITS >= 32) ? 0xffffffffu : ((1u << STEP_BITS) - 1u);
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
// Tile <-> LDS staging: coalesced on the global side, one padded row per lane on the LDS side.
// All global loads of a tile are issued before the first LDS write so they overlap; addresses
// past the valid part are clamped (the rows they fill are never read).
struct NoWork { HMM_DEV void operator()() const {} };

// `between` runs after the tile's loads have been issued and before their data is needed: work
// placed there (such as taking logarithms of the model) is hidden behind the memory latency.
template <int D, class F = NoWork>
HMM_DEV void load_tile(const float* __restrict__ g, int nvalid_steps, float* lds, F between = F()) {
    using C = SmallCfg<D>;
    const int nfl = nvalid_steps * D;
    if constexpr (C::VEC == 4) {
        constexpr int NIT = C::ROW / 4;
        const float4* g4 = reinterpret_cast<const float4*>(g);
        const int last = nfl / 4 - 1;
        float4 x[NIT];
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int v = it * C::NT + threadIdx.x;
            typedef float nt4 __attribute__((ext_vector_type(4)));
            const nt4 y = __builtin_nontemporal_load(reinterpret_cast<const nt4*>(g4 + (v < last ? v : last)));
            x[it] = make_float4(y.x, y.y, y.z, y.w);
        }
        between();
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int fl = (it * C::NT + threadIdx.x) * 4;
            const int owner = fl / C::ROW;
            *reinterpret_cast<float4*>(lds + owner * C::STRIDE + (fl - owner * C::ROW)) = x[it];
        }
    } else {
        constexpr int CH = 8;
        static_assert(C::ROW % CH == 0, "row length must be a multiple of the load batch");
        const int last = nfl - 1;
        for (int it0 = 0; it0 < C::ROW; it0 += CH) {
            float x[CH];
#pragma unroll
            for (int q = 0; q < CH; ++q) {
                const int fl = (it0 + q) * C::NT + threadIdx.x;
                x[q] = g[fl < last ? fl : last];
            }
            if (it0 == 0) between();
#pragma unroll
            for (int q = 0; q < CH; ++q) {
                const int fl = (it0 + q) * C::NT + threadIdx.x;
                const int owner = fl / C::ROW;
                lds[owner * C::STRIDE + (fl - owner * C::ROW)] = x[q];
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
            const int owner = fl / C::ROW;
            typedef float nt4 __attribute__((ext_vector_type(4)));
            const nt4 x = *reinterpret_cast<const nt4*>(lds + owner * C::STRIDE + (fl - owner * C::ROW));
            if (fl < nfl) __builtin_nontemporal_store(x, reinterpret_cast<nt4*>(g4 + v));
        }
    } else {
#pragma unroll 8
        for (int it = 0; it < C::ROW; ++it) {
            const int fl = it * C::NT + threadIdx.x;
            const int owner = fl / C::ROW;
            const float x = lds[owner * C::STRIDE + (fl - owner * C::ROW)];
            if (fl < nfl) g[fl] = x;
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

// The same in two parts, so that other loads can be issued between the model's loads and the
// arithmetic on them.
template <int D>
HMM_DEV void load_model_raw(const float* __restrict__ A, float (&Am)[D * D]) {
#pragma unroll
    for (int e = 0; e < D * D; ++e) Am[e] = A[e];
}

template <class S, int D>
HMM_DEV void model_to_domain(float (&Am)[D * D]) {
    if constexpr (S::is_max_plus) {
#pragma unroll
        for (int e = 0; e < D * D; ++e) Am[e] = logf(Am[e]);
    }
}

// Emission factor of one step in the operator's domain.  SumProd: e_k(j) = exp(ll_k(j) - m_k)
// with m_k = max_j ll_k(j) (returned); MaxPlus: ll_k itself (returns 0).
template <class S, int D>
HMM_DEV float emission(float (&ev)[D]) {
    if constexpr (S::is_max_plus) {
        return 0.0f;
    } else {
        const float m = max_of(ev);
        const float ms = (m == -INFINITY) ? 0.0f : m;
        const float c = -1.4426950408889634f * ms;          // exp(x - m) = exp2(x * log2(e) - m * log2(e))
#pragma unroll
        for (int j = 0; j < D; ++j) ev[j] = __builtin_amdgcn_exp2f(fmaf(ev[j], 1.4426950408889634f, c));
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
// per-step maxima m_k is returned through msum.  FULL: n == L is known (no per-step tests).
template <class S, int D, bool STORE_E, bool FULL>
HMM_DEV void chunk_aggregate_impl(float* row, int n, bool first, const float (&Am)[D * D], float (&P)[D * D],
                                  double& msum) {
    using C = SmallCfg<D>;
    mat_identity<S, D>(P);
    float ms = 0.0f;   // sum of at most L maxima: float is ample, the caller accumulates in double
#pragma unroll
    for (int k = 0; k < C::L; ++k) {
        if (FULL || k < n) {
            float ev[D];
            lds_read_vec<D>(row + k * D, ev);
            const float m = emission<S, D>(ev);
            if constexpr (STORE_E) {
                lds_write_vec<D>(row + k * D, ev);
                ms += m;
            }
            if (k == 0) {
                // P is still the neutral element: P (op) psi = psi, no product needed
#pragma unroll
                for (int i = 0; i < D; ++i)
#pragma unroll
                    for (int j = 0; j < D; ++j) {
                        const float a = first ? ((i == j) ? S::one() : S::zero()) : Am[i * D + j];
                        P[i * D + j] = S::times(a, ev[j]);
                    }
            } else {
                absorb<S, D>(P, Am, ev, false);
            }
            if ((k & 3) == 3) renorm<S, D * D>(P);
        }
    }
    msum = (double)ms;
}

template <class S, int D, bool STORE_E>
HMM_DEV void chunk_aggregate(float* row, int n, bool first, const float (&Am)[D * D], float (&P)[D * D],
                             double& msum) {
    if (n == SmallCfg<D>::L) chunk_aggregate_impl<S, D, STORE_E, true>(row, n, first, Am, P, msum);
    else chunk_aggregate_impl<S, D, STORE_E, false>(row, n, first, Am, P, msum);
}

// ---------------------------------------------------------------------------------------------
// Wave-level scans of chunk aggregates over the 64 lanes of a wavefront, moved with DPP:
// four shifts inside each row of 16 lanes, then the last lane of a row broadcast to the next
// row(s).  A lane that has no source at some level combines with the operator's neutral
// element instead, so no lane needs to be predicated.
template <int CTRL, int ROW_MASK>
HMM_DEV float dpp_move(float neutral, float src) {
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(neutral), __float_as_int(src), CTRL, ROW_MASK,
                                                      0xF, false));
}

template <class S, int D, bool SWAP, int CTRL, int ROW_MASK>
HMM_DEV void wave_scan_level(float (&Q)[D * D]) {
    float Pn[D * D], Z[D * D];
#pragma unroll
    for (int i = 0; i < D; ++i)
#pragma unroll
        for (int j = 0; j < D; ++j)
            Pn[i * D + j] = dpp_move<CTRL, ROW_MASK>((i == j) ? S::one() : S::zero(), Q[i * D + j]);
    if constexpr (SWAP) mat_mul<S, D>(Q, Pn, Z);
    else mat_mul<S, D>(Pn, Q, Z);
    renorm<S, D * D>(Z);
#pragma unroll
    for (int e = 0; e < D * D; ++e) Q[e] = Z[e];
}

// Inclusive scan towards higher lanes.  SWAP = false: Q_t <- P_0 (op) ... (op) P_t;
// SWAP = true: Q_t <- P_t (op) ... (op) P_0 (the operator's arguments exchanged).
template <class S, int D, bool SWAP>
HMM_DEV void wave_scan_up(float (&Q)[D * D]) {
    wave_scan_level<S, D, SWAP, 0x111, 0xF>(Q);   // row_shr:1
    wave_scan_level<S, D, SWAP, 0x112, 0xF>(Q);   // row_shr:2
    wave_scan_level<S, D, SWAP, 0x114, 0xF>(Q);   // row_shr:4
    wave_scan_level<S, D, SWAP, 0x118, 0xF>(Q);   // row_shr:8
    wave_scan_level<S, D, SWAP, 0x142, 0xA>(Q);   // row_bcast:15 into rows 1 and 3
    wave_scan_level<S, D, SWAP, 0x143, 0xC>(Q);   // row_bcast:31 into rows 2 and 3
}

template <class S, int D>
HMM_DEV void wave_scan_prefix(float (&Q)[D * D]) {   // Q_t <- P_0 (op) ... (op) P_t
    wave_scan_up<S, D, false>(Q);
}

// R_t <- P_t (op) ... (op) P_63: the prefix scan with exchanged arguments on mirrored lanes
// (the reversal recipe of Sec. III-B applied across the wavefront).
template <class S, int D>
HMM_DEV void wave_scan_suffix(float (&R)[D * D]) {
    const int mirror = 63 - (int)(threadIdx.x & 63);
#pragma unroll
    for (int e = 0; e < D * D; ++e) R[e] = __shfl(R[e], mirror, 64);
    wave_scan_up<S, D, true>(R);
#pragma unroll
    for (int e = 0; e < D * D; ++e) R[e] = __shfl(R[e], mirror, 64);
}

// Inclusive prefix scan inside each wave; the wave totals go to wagg[NW][D*D] in LDS.
// The caller must __syncthreads() before reading wagg.
template <class S, int D>
HMM_DEV void block_prefix(const float (&P)[D * D], float (&Q)[D * D], float* wagg) {
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
#pragma unroll
    for (int e = 0; e < D * D; ++e) Q[e] = P[e];
    wave_scan_prefix<S, D>(Q);
    if (lane == 63) {
#pragma unroll
        for (int e = 0; e < D * D; ++e) wagg[wave * D * D + e] = Q[e];
    }
}

// Workgroup aggregate W_0 (op) ... (op) W_{NW-1} from the wave totals (any single lane may call).
template <class S, int D>
HMM_DEV void block_total(const float* wagg, float (&X)[D * D]) {
    using C = SmallCfg<D>;
#pragma unroll
    for (int e = 0; e < D * D; ++e) X[e] = wagg[e];
#pragma unroll
    for (int w = 1; w < C::NW; ++w) {
        float Y[D * D], Z[D * D];
#pragma unroll
        for (int e = 0; e < D * D; ++e) Y[e] = wagg[w * D * D + e];
        mat_mul<S, D>(X, Y, Z);
        renorm<S, D * D>(Z);
#pragma unroll
        for (int e = 0; e < D * D; ++e) X[e] = Z[e];
    }
}

// fin = cin_f (op) P_0 (op) ... (op) P_{t-1}: the forward potential just before lane t's chunk,
// from the lane's inclusive wave prefix Q and the wave totals.
template <class S, int D>
HMM_DEV void carry_forward(const float (&Q)[D * D], const float* wagg, const float (&cin_f)[D], float (&fin)[D]) {
    using C = SmallCfg<D>;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
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

// bout = P_{t+1} (op) ... (op) P_{NT-1} (op) cin_b: the backward potential at the last step of
// lane t's chunk, from the lane's inclusive wave suffix R and the wave totals.
template <class S, int D>
HMM_DEV void carry_backward(const float (&R)[D * D], const float* wagg, const float (&cin_b)[D], float (&bout)[D]) {
    using C = SmallCfg<D>;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
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

// Both carries for every lane of the workgroup (contains one __syncthreads()).
template <class S, int D, bool BWD>
HMM_DEV void block_exchange(const float (&P)[D * D], const float (&cin_f)[D], const float (&cin_b)[D],
                            float (&fin)[D], float (&bout)[D], float* wagg) {
    float Q[D * D];
    block_prefix<S, D>(P, Q, wagg);
    __syncthreads();
    carry_forward<S, D>(Q, wagg, cin_f, fin);
    if constexpr (BWD) {
        float R[D * D];
#pragma unroll
        for (int e = 0; e < D * D; ++e) R[e] = P[e];
        wave_scan_suffix<S, D>(R);
        carry_backward<S, D>(R, wagg, cin_b, bout);
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

// ---------------------------------------------------------------------------------------------
// Sum-product work inside a lane's chunk

// Forward: a_{0:k} for the lane's steps, kept in registers as F (Theorem 1).  f enters as the
// carry (sum one, or the prior for the sequence's first chunk) and every step is rescaled by an
// exact power of two; returns the chunk-local log evidence log p(y_chunk | y_before).
template <int D, bool WRITE_FILT, bool FULL>
HMM_DEV double sp_forward_impl(const float* row, int n, bool first, const float (&Am)[D * D], float (&f)[D],
                               float (&F)[SmallCfg<D>::L][D], double msum, float* __restrict__ filt_dst) {
    using C = SmallCfg<D>;
    using S = SumProd;
    int exsum = 0;
    float s_last = 1.0f;
#pragma unroll
    for (int k = 0; k < C::L; ++k) {
        if (FULL || k < n) {
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
#pragma unroll
                for (int j = 0; j < D; ++j) filt_dst[k * D + j] = f[j] * inv;
            }
        }
    }
    if (!FULL && n == 0) return 0.0;
    return msum + 0.6931471805599453 * (double)exsum + log((double)s_last);
}

// Backward: a_{k:T+1} (Theorem 2) and the marginal f_k b_k / Z_k, written over the emission
// factors in LDS.  b enters as the backward potential at the chunk's last step.
template <int D, bool FULL>
HMM_DEV void sp_backward_impl(float* row, int n, const float (&Am)[D * D], float (&b)[D],
                              const float (&F)[SmallCfg<D>::L][D]) {
    using C = SmallCfg<D>;
    using S = SumProd;
    renorm<S, D>(b);
#pragma unroll
    for (int k = C::L - 1; k >= 0; --k) {
        if (FULL || k < n) {
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
}

// ---------------------------------------------------------------------------------------------
// Max-plus work inside a lane's chunk: V_k and the back-pointers u_{k-1}(x_k) of Sec. IV-A.
// v enters as the carry (max 0, or the log prior for the first chunk) and leaves as V at the
// chunk's last step with max 0; returns the sum of the offsets removed on the way.
template <int D, bool FULL>
HMM_DEV double mp_forward_impl(const float* row, int n, bool first, const float (&Am)[D * D], float (&v)[D],
                               uint32_t (&bp)[SmallCfg<D>::W]) {
    using C = SmallCfg<D>;
    using S = MaxPlus;
#pragma unroll
    for (int w = 0; w < C::W; ++w) bp[w] = 0u;
    double osum = 0.0;
#pragma unroll
    for (int k = 0; k < C::L; ++k) {
        if (FULL || k < n) {
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
    return osum;
}

// ---------------------------------------------------------------------------------------------
// Max-product forward/backward work inside a lane's chunk (the lemma of Sec. IV-C on logarithms).

// Forward: psi~^f_k for the lane's steps, kept in registers as F, each step shifted to max 0.
// v enters as the carry (max 0, or the log prior for the sequence's first chunk); returns the sum
// of the shifts, i.e. the chunk-local growth of the log of the best joint weight.
template <int D, bool FULL>
HMM_DEV double mpv_forward_impl(const float* row, int n, bool first, const float (&Am)[D * D], float (&v)[D],
                                float (&F)[SmallCfg<D>::L][D]) {
    using C = SmallCfg<D>;
    using S = MaxPlus;
    double osum = 0.0;
#pragma unroll
    for (int k = 0; k < C::L; ++k) {
        if (FULL || k < n) {
            float lk[D], g[D];
            lds_read_vec<D>(row + k * D, lk);
            if (k == 0 && first) {
#pragma unroll
                for (int j = 0; j < D; ++j) g[j] = v[j] + lk[j];
            } else {
                vec_mat<S, D>(v, Am, g);
#pragma unroll
                for (int j = 0; j < D; ++j) g[j] += lk[j];
            }
            osum += (double)renorm<S, D>(g);
#pragma unroll
            for (int j = 0; j < D; ++j) F[k][j] = v[j] = g[j];
        }
    }
    return (!FULL && n == 0) ? 0.0 : osum;
}

// Backward: psi~^b_k and the max-marginal log psi~^f_k + log psi~^b_k (Theorem 4), shifted so that its
// largest entry is 0 and written over the log-likelihoods in LDS.  b enters as the backward
// potential at the chunk's last step.
template <int D, bool FULL>
HMM_DEV void mpv_backward_impl(float* row, int n, const float (&Am)[D * D], float (&b)[D],
                               const float (&F)[SmallCfg<D>::L][D]) {
    using C = SmallCfg<D>;
    using S = MaxPlus;
    renorm<S, D>(b);
#pragma unroll
    for (int k = C::L - 1; k >= 0; --k) {
        if (FULL || k < n) {
            float lk[D], gam[D];
            lds_read_vec<D>(row + k * D, lk);
#pragma unroll
            for (int j = 0; j < D; ++j) gam[j] = F[k][j] + b[j];
            renorm<S, D>(gam);
            lds_write_vec<D>(row + k * D, gam);
            if (k > 0) {
                float t[D], r[D];
#pragma unroll
                for (int j = 0; j < D; ++j) t[j] = lk[j] + b[j];
                mat_vec<S, D>(Am, t, r);
                renorm<S, D>(r);
#pragma unroll
                for (int j = 0; j < D; ++j) b[j] = r[j];
            }
        }
    }
}

// x_k = argmax_j of the D values of every valid step of the tile in LDS (lowest index on ties),
// written coalesced.
template <int D>
HMM_DEV void store_argmax_tile(int32_t* __restrict__ dst, int nvalid, const float* lds) {
    using C = SmallCfg<D>;
#pragma unroll 4
    for (int it = 0; it < C::L; ++it) {
        const int s = it * C::NT + threadIdx.x;
        if (s < nvalid) {
            const float* p = lds + (s / C::L) * C::STRIDE + (s % C::L) * D;
            float best = p[0];
            int arg = 0;
#pragma unroll
            for (int j = 1; j < D; ++j) {
                const float x = p[j];
                const bool gt = x > best;
                best = gt ? x : best;
                arg = gt ? j : arg;
            }
            __builtin_nontemporal_store((int32_t)arg, dst + s);
        }
    }
}

// ---------------------------------------------------------------------------------------------
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

template <int D>
HMM_DEV uint32_t map_constant(uint32_t c) {
    using C = SmallCfg<D>;
    uint32_t m = 0;
#pragma unroll
    for (int j = 0; j < D; ++j) m |= c << (j * C::BITS);
    return m;
}

constexpr uint32_t MAP_FINAL_FLAG = 0x80000000u;   // lane holds the sequence's last step
constexpr int MAP_FINAL_SHIFT = 24;                // ... and x*_T is stored here
constexpr uint32_t MAP_BODY = 0x00ffffffu;

// For D <= 4 a map also fits one byte per entry, and then composition is a single byte-permute
// instruction (result byte j = byte h(j) of g); chains of compositions convert once on the way
// in and once on the way out.
template <int D>
HMM_DEV uint32_t map_to_bytes(uint32_t g) {
    using C = SmallCfg<D>;
    if constexpr (D == 4) {
        return (g | (g << 6) | (g << 12) | (g << 18)) & 0x03030303u;
    } else {
        uint32_t r = 0;
#pragma unroll
        for (int j = 0; j < D; ++j) r |= ((g >> (j * C::BITS)) & C::MASK) << (8 * j);
        return r;
    }
}

template <int D>
HMM_DEV uint32_t map_from_bytes(uint32_t m) {
    using C = SmallCfg<D>;
    if constexpr (D == 4) {
        return (m | (m >> 6) | (m >> 12) | (m >> 18)) & 0xffu;
    } else {
        uint32_t r = 0;
#pragma unroll
        for (int j = 0; j < D; ++j) r |= ((m >> (8 * j)) & C::MASK) << (j * C::BITS);
        return r;
    }
}

HMM_DEV uint32_t bytes_compose(uint32_t g, uint32_t h) { return __builtin_amdgcn_perm(0u, g, h); }

// Chunk map: x at the chunk's last step -> x at the step before the chunk.
template <int D>
HMM_DEV uint32_t chunk_map(const uint32_t (&bp)[SmallCfg<D>::W], int n) {
    using C = SmallCfg<D>;
    if constexpr (D <= 4) {
        uint32_t h = 0x03020100u;   // identity, one byte per entry
#pragma unroll
        for (int k = C::L - 1; k >= 0; --k) {
            if (k < n) {
                const uint32_t u = (bp[k / C::SPW] >> ((k % C::SPW) * C::STEP_BITS)) & C::STEP_MASK;
                h = bytes_compose(map_to_bytes<D>(u), h);
            }
        }
        return map_from_bytes<D>(h);
    } else {
        uint32_t h = map_identity<D>();
#pragma unroll
        for (int k = C::L - 1; k >= 0; --k) {
            if (k < n) {
                const uint32_t u = (bp[k / C::SPW] >> ((k % C::SPW) * C::STEP_BITS)) & C::STEP_MASK;
                h = map_compose<D>(u, h);
            }
        }
        return h;
    }
}

// x*_T = argmax_j V_T(j), lowest index on ties
template <int D>
HMM_DEV uint32_t argmax_state(const float (&v)[D]) {
    uint32_t xs = 0u;
    float best = v[0];
#pragma unroll
    for (int j = 1; j < D; ++j) {
        const bool gt = v[j] > best;
        best = gt ? v[j] : best;
        xs = gt ? (uint32_t)j : xs;
    }
    return xs;
}

// Reversed all-prefix-sums under composition over the workgroup's lanes:
// excl = g_{t+1} o ... o g_{NT-1} for every lane; returns g_0 o ... o g_{NT-1} (in every lane).
// Contains one __syncthreads(); wmaps: NW words of LDS not in use by anyone else.
template <int D>
HMM_DEV uint32_t block_map_suffix(uint32_t g, uint32_t& excl, uint32_t* wmaps) {
    using C = SmallCfg<D>;
    constexpr bool BYTES = D <= 4;   // compose in the byte form, convert at both ends
    auto comp = [](uint32_t a, uint32_t b) {
        if constexpr (BYTES) return bytes_compose(a, b);
        else return map_compose<D>(a, b);
    };
    const uint32_t ident = BYTES ? 0x03020100u : map_identity<D>();
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    uint32_t G = BYTES ? map_to_bytes<D>(g) : g;   // inclusive: g_t o ... o g_63 within the wave
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t o = __shfl_down(G, d, 64);
        const uint32_t c = comp(G, o);
        G = (lane + d < 64) ? c : G;
    }
    if (lane == 0) wmaps[wave] = G;
    __syncthreads();
    uint32_t tail = ident;   // composition of the waves after mine
#pragma unroll
    for (int w = C::NW - 1; w > 0; --w)
        if (w > wave) tail = comp(wmaps[w], tail);
    uint32_t nxt = __shfl_down(G, 1, 64);
    nxt = (lane == 63) ? ident : nxt;
    excl = comp(nxt, tail);
    uint32_t total = ident;
#pragma unroll
    for (int w = C::NW - 1; w >= 0; --w) total = comp(wmaps[w], total);
    if constexpr (BYTES) {
        excl = map_from_bytes<D>(excl);
        total = map_from_bytes<D>(total);
    }
    return total;
}

// Walk the back-pointers down the lane's chunk from state x at its last step, staging the states
// for a coalesced write.
template <int D>
HMM_DEV void walk_chunk(const uint32_t (&bp)[SmallCfg<D>::W], int n, bool first, uint32_t x, int32_t* stage_row) {
    using C = SmallCfg<D>;
#pragma unroll
    for (int k = C::L - 1; k >= 0; --k) {
        if (k < n) {
            stage_row[k] = (int32_t)x;
            if (!(k == 0 && first)) {
                const uint32_t u = bp[k / C::SPW] >> ((k % C::SPW) * C::STEP_BITS);
                x = map_apply<D>(u, x);
            }
        }
    }
}

template <int D>
HMM_DEV void store_path_tile(int32_t* __restrict__ dst, int nvalid, const int32_t* stage) {
    using C = SmallCfg<D>;
#pragma unroll
    for (int it = 0; it < C::L; ++it) {
        const int s = it * C::NT + threadIdx.x;
        if (s < nvalid) __builtin_nontemporal_store(stage[(s / C::L) * C::PSTRIDE + (s % C::L)], dst + s);
    }
}

// ---------------------------------------------------------------------------------------------
// Several short sequences per workgroup.  A sequence of at most 64 L steps takes cpl = 2^lcpl consecutive
// lanes (one chunk of L steps each, the last ones possibly empty), aligned to a multiple of cpl, so a wave
// holds 64 / cpl whole sequences and the scans over chunk aggregates stop at the groups' boundaries: they
// are the wave scans above cut off after lcpl levels, with the shifts inside a row of 16 lanes masked to
// the group.  The batch is contiguous in memory, so the sequences of a workgroup are one contiguous range
// and are staged through LDS with the same coalesced accesses as a tile, only the owner of an element is
// found by a division by the sequence length.
struct PackCoord {
    int seq0;    // first sequence of the workgroup
    int nseq;    // sequences of the workgroup (the last workgroup may hold fewer)
    int c;       // the lane's chunk inside its sequence
    int seq;     // the lane's sequence (clamped to the batch: lanes past it hold no steps)
    int n;       // valid steps of the lane's chunk
    bool first;  // the chunk starts its sequence
    bool last;   // the chunk holds its sequence's last step
};

template <int D>
HMM_DEV PackCoord pack_coord(long long T, int batch, int lcpl) {
    using C = SmallCfg<D>;
    PackCoord p;
    const int spw = C::NT >> lcpl;
    p.seq0 = (int)blockIdx.x * spw;
    p.nseq = min(spw, batch - p.seq0);
    const int q = (int)threadIdx.x >> lcpl;
    p.c = (int)threadIdx.x & ((1 << lcpl) - 1);
    const bool live = q < p.nseq;
    p.seq = p.seq0 + (live ? q : 0);
    const long long rem = T - (long long)p.c * C::L;
    p.n = live ? (int)(rem < 0 ? 0 : rem > C::L ? C::L : rem) : 0;
    p.first = p.n > 0 && p.c == 0;
    p.last = p.n > 0 && rem <= C::L;
    return p;
}

// x / d and x % d for 0 <= x < 2^23 through the reciprocal, corrected by one either way
HMM_DEV int div_by(int x, int d, float inv_d, int& rem) {
    int q = (int)((float)x * inv_d);
    int r = x - q * d;
    if (r < 0) { --q; r += d; }
    else if (r >= d) { ++q; r -= d; }
    rem = r;
    return q;
}

// LDS position of element `fl` (a float index into the workgroup's range of the batch; rowlen floats per sequence)
template <int D>
HMM_DEV int packed_slot(int fl, int rowlen, float inv_rowlen, int lcpl) {
    using C = SmallCfg<D>;
    int w;
    const int q = div_by(fl, rowlen, inv_rowlen, w);
    const int c = w / C::ROW;
    return ((q << lcpl) + c) * C::STRIDE + (w - c * C::ROW);
}

template <int D, class F = NoWork>
HMM_DEV void load_packed(const float* __restrict__ g, int nfl, int rowlen, int lcpl, float* lds, F between = F()) {
    using C = SmallCfg<D>;
    const float inv = 1.0f / (float)rowlen;
    if constexpr (C::VEC == 4) {
        constexpr int NIT = C::ROW / 4;
        const float4* g4 = reinterpret_cast<const float4*>(g);
        const int last = nfl / 4 - 1;
        float4 x[NIT];
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int v = it * C::NT + threadIdx.x;
            typedef float nt4 __attribute__((ext_vector_type(4)));
            const nt4 y = __builtin_nontemporal_load(reinterpret_cast<const nt4*>(g4 + (v < last ? v : last)));
            x[it] = make_float4(y.x, y.y, y.z, y.w);
        }
        between();
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const int fl = (it * C::NT + threadIdx.x) * 4;
            if (fl < nfl) *reinterpret_cast<float4*>(lds + packed_slot<D>(fl, rowlen, inv, lcpl)) = x[it];
        }
    } else {
        constexpr int CH = 8;
        const int last = nfl - 1;
        for (int it0 = 0; it0 < C::ROW; it0 += CH) {
            float x[CH];
#pragma unroll
            for (int q = 0; q < CH; ++q) {
                const int fl = (it0 + q) * C::NT + threadIdx.x;
                x[q] = g[fl < last ? fl : last];
            }
            if (it0 == 0) between();
#pragma unroll
            for (int q = 0; q < CH; ++q) {
                const int fl = (it0 + q) * C::NT + threadIdx.x;
                if (fl < nfl) lds[packed_slot<D>(fl, rowlen, inv, lcpl)] = x[q];
            }
        }
    }
}

template <int D>
HMM_DEV void store_packed(float* __restrict__ g, int nfl, int rowlen, int lcpl, const float* lds) {
    using C = SmallCfg<D>;
    const float inv = 1.0f / (float)rowlen;
    if constexpr (C::VEC == 4) {
        float4* g4 = reinterpret_cast<float4*>(g);
#pragma unroll
        for (int it = 0; it < C::ROW / 4; ++it) {
            const int v = it * C::NT + threadIdx.x;
            const int fl = v * 4;
            if (fl < nfl) {
                typedef float nt4 __attribute__((ext_vector_type(4)));
                const nt4 x = *reinterpret_cast<const nt4*>(lds + packed_slot<D>(fl, rowlen, inv, lcpl));
                __builtin_nontemporal_store(x, reinterpret_cast<nt4*>(g4 + v));
            }
        }
    } else {
#pragma unroll 8
        for (int it = 0; it < C::ROW; ++it) {
            const int fl = it * C::NT + threadIdx.x;
            if (fl < nfl) g[fl] = lds[packed_slot<D>(fl, rowlen, inv, lcpl)];
        }
    }
}

// Row (lane) and step inside the row of time step s of the workgroup's range (T steps per sequence)
template <int D>
HMM_DEV int packed_step_owner(int s, int T, float inv_T, int lcpl, int& k) {
    using C = SmallCfg<D>;
    int w;
    const int q = div_by(s, T, inv_T, w);
    const int c = w / C::L;
    k = w - c * C::L;
    return (q << lcpl) + c;
}

template <int D>
HMM_DEV void store_argmax_packed(int32_t* __restrict__ dst, int nsteps, int T, int lcpl, const float* lds) {
    using C = SmallCfg<D>;
    const float inv = 1.0f / (float)T;
#pragma unroll 4
    for (int it = 0; it < C::L; ++it) {
        const int s = it * C::NT + threadIdx.x;
        if (s < nsteps) {
            int k;
            const int owner = packed_step_owner<D>(s, T, inv, lcpl, k);
            const float* p = lds + owner * C::STRIDE + k * D;
            float best = p[0];
            int arg = 0;
#pragma unroll
            for (int j = 1; j < D; ++j) {
                const float x = p[j];
                const bool gt = x > best;
                best = gt ? x : best;
                arg = gt ? j : arg;
            }
            __builtin_nontemporal_store((int32_t)arg, dst + s);
        }
    }
}

template <int D>
HMM_DEV void store_path_packed(int32_t* __restrict__ dst, int nsteps, int T, int lcpl, const int32_t* stage) {
    using C = SmallCfg<D>;
    const float inv = 1.0f / (float)T;
#pragma unroll
    for (int it = 0; it < C::L; ++it) {
        const int s = it * C::NT + threadIdx.x;
        if (s < nsteps) {
            int k;
            const int owner = packed_step_owner<D>(s, T, inv, lcpl, k);
            __builtin_nontemporal_store(stage[owner * C::PSTRIDE + k], dst + s);
        }
    }
}

// One level of the scan towards higher lanes in which a lane takes its partner only if `take`.
template <class S, int D, bool SWAP, int CTRL, int ROW_MASK>
HMM_DEV void wave_scan_level_if(float (&Q)[D * D], bool take) {
    float Pn[D * D], Z[D * D];
#pragma unroll
    for (int i = 0; i < D; ++i)
#pragma unroll
        for (int j = 0; j < D; ++j) {
            const float id = (i == j) ? S::one() : S::zero();
            const float m = dpp_move<CTRL, ROW_MASK>(id, Q[i * D + j]);
            Pn[i * D + j] = take ? m : id;
        }
    if constexpr (SWAP) mat_mul<S, D>(Q, Pn, Z);
    else mat_mul<S, D>(Pn, Q, Z);
    renorm<S, D * D>(Z);
#pragma unroll
    for (int e = 0; e < D * D; ++e) Q[e] = Z[e];
}

// Inclusive scan towards higher lanes inside every aligned group of 2^lcpl lanes.
template <class S, int D, bool SWAP>
HMM_DEV void group_scan_up(float (&Q)[D * D], int lcpl) {
    const int pos = (int)(threadIdx.x & 63) & ((1 << lcpl) - 1);
    if (lcpl > 0) wave_scan_level_if<S, D, SWAP, 0x111, 0xF>(Q, pos >= 1);   // row_shr:1
    if (lcpl > 1) wave_scan_level_if<S, D, SWAP, 0x112, 0xF>(Q, pos >= 2);   // row_shr:2
    if (lcpl > 2) wave_scan_level_if<S, D, SWAP, 0x114, 0xF>(Q, pos >= 4);   // row_shr:4
    if (lcpl > 3) wave_scan_level_if<S, D, SWAP, 0x118, 0xF>(Q, pos >= 8);   // row_shr:8
    if (lcpl > 4) wave_scan_level<S, D, SWAP, 0x142, 0xA>(Q);               // row_bcast:15 into rows 1 and 3
    if (lcpl > 5) wave_scan_level<S, D, SWAP, 0x143, 0xC>(Q);               // row_bcast:31 into rows 2 and 3
}

// Forward potential entering every chunk and backward potential at every chunk's last step, for sequences
// that start from `start` (the prior, in the operator's domain) and end inside their group.
template <class S, int D, bool BWD>
HMM_DEV void group_exchange(const float (&P)[D * D], int lcpl, int c, const float (&start)[D], float (&fin)[D],
                            float (&bout)[D]) {
    float Q[D * D], r[D];
#pragma unroll
    for (int e = 0; e < D * D; ++e) Q[e] = P[e];
    group_scan_up<S, D, false>(Q, lcpl);
    float Qp[D * D];
#pragma unroll
    for (int e = 0; e < D * D; ++e) Qp[e] = __shfl_up(Q[e], 1, 64);
    vec_mat<S, D>(start, Qp, r);
#pragma unroll
    for (int j = 0; j < D; ++j) fin[j] = (c == 0) ? start[j] : r[j];
    if constexpr (BWD) {
        const int mirror = 63 - (int)(threadIdx.x & 63);
        float R[D * D], ones[D];
#pragma unroll
        for (int e = 0; e < D * D; ++e) R[e] = __shfl(P[e], mirror, 64);
        group_scan_up<S, D, true>(R, lcpl);
#pragma unroll
        for (int e = 0; e < D * D; ++e) R[e] = __shfl(R[e], mirror, 64);
        float Rn[D * D];
#pragma unroll
        for (int e = 0; e < D * D; ++e) Rn[e] = __shfl_down(R[e], 1, 64);
#pragma unroll
        for (int j = 0; j < D; ++j) ones[j] = S::one();
        mat_vec<S, D>(Rn, ones, r);
#pragma unroll
        for (int j = 0; j < D; ++j) bout[j] = (c == (1 << lcpl) - 1) ? ones[j] : r[j];
    }
}

// Sum of one double per lane over every aligned group of 2^lcpl lanes, in a fixed order; valid in the
// group's first lane.
HMM_DEV double group_sum(double v, int lcpl) {
    for (int d = (1 << lcpl) >> 1; d >= 1; d >>= 1) v += __shfl_down(v, d, 64);
    return v;
}

// excl = g_{c+1} o ... o g_{cpl-1} inside every aligned group of cpl = 2^lcpl lanes
template <int D>
HMM_DEV uint32_t group_map_suffix(uint32_t g, int lcpl, int c) {
    constexpr bool BYTES = D <= 4;
    auto comp = [](uint32_t a, uint32_t b) {
        if constexpr (BYTES) return bytes_compose(a, b);
        else return map_compose<D>(a, b);
    };
    const uint32_t ident = BYTES ? 0x03020100u : map_identity<D>();
    const int cpl = 1 << lcpl;
    uint32_t G = BYTES ? map_to_bytes<D>(g) : g;   // inclusive: g_c o ... o g_{cpl-1}
    for (int d = 1; d < cpl; d <<= 1) {
        const uint32_t o = __shfl_down(G, d, 64);
        const uint32_t cc = comp(G, o);
        G = (c + d < cpl) ? cc : G;
    }
    uint32_t nxt = __shfl_down(G, 1, 64);
    nxt = (c == cpl - 1) ? ident : nxt;
    return BYTES ? map_from_bytes<D>(nxt) : nxt;
}

// ---------------------------------------------------------------------------------------------
// Exchange between co-resident workgroups (single-launch kernels) through self-validating words.
//
// Before the kernel starts, every exchange slot in the workspace holds the all-ones bit pattern
// (a NaN as float or double, an impossible back-pointer map).  A producer overwrites its slots
// with agent-scope (write-through, cache-bypassing) stores of real values, none of which has
// that pattern; consumers poll the slots with agent-scope (cache-bypassing) loads until no
// sentinel is left.  Each 32/64-bit word is written by one store, so a consumer never sees a
// torn word, and no ordering between different words is relied upon: there are no flags, no
// fences (an agent-scope fence writes back / invalidates a whole L2 on this multi-die part) and
// no read-modify-write atomics (a few hundred on one address serialise for microseconds).
// The poll is bounded so that every wave terminates even if the workgroups were, against the
// host's residency check, not all resident.
constexpr int SPIN_LIMIT = 1 << 20;
constexpr uint32_t SENTINEL32 = 0xffffffffu;
constexpr unsigned long long SENTINEL64 = 0xffffffffffffffffull;

template <class T>
HMM_DEV void coherent_store(T* p, T v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <class T>
HMM_DEV T coherent_load(const T* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Bits of a float to publish: any NaN becomes the canonical quiet NaN, which is not the sentinel.
HMM_DEV uint32_t publish_bits(float x) { return (x != x) ? 0x7fc00000u : __float_as_uint(x); }
HMM_DEV unsigned long long publish_bits(double x) {
    return (x != x) ? 0x7ff8000000000000ull : (unsigned long long)__double_as_longlong(x);
}

}  // namespace hmm
