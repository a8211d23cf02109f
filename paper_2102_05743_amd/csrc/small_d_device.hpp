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
#ifdef HMM_TILE_STEPS_PER_LANE
    static constexpr int L = HMM_TILE_STEPS_PER_LANE; // (build-time override for tile-size experiments: a multiple of four)
#else
    static constexpr int L = (D <= 4) ? 16 : 8;       // time steps per lane
#endif
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

// Emission factor of one step in the operator's domain.  MaxPlus: ll_k itself.  SumProd:
// e_k(j) = exp(ll_k(j)) / 2^n with n = the whole number of bits nearest to max_j ll_k(j) / ln 2, so
// that the largest factor lies in [2^-0.5, 2^0.5] and what was taken out is an integer: `bits`
// receives n, `spread` the (non-positive) binary logarithm of the smallest factor relative to 2^n.
template <class S, int D>
HMM_DEV void emission(float (&ev)[D], float& bits, float& spread) {
    if constexpr (S::is_max_plus) {
        bits = 0.0f;
        spread = 0.0f;
    } else {
        constexpr float LOG2E = 1.4426950408889634f;
        const float m = max_of(ev);
        const float n = (m == -INFINITY) ? 0.0f : rintf(m * LOG2E);
        float lo = INFINITY;
#pragma unroll
        for (int j = 0; j < D; ++j) {
            const float x = fmaf(ev[j], LOG2E, -n);
            lo = fminf(lo, x);
            ev[j] = __builtin_amdgcn_exp2f(x);
        }
        bits = n;
        spread = lo;
    }
}

// P <- P (op) psi_k with psi_k(i,j) = Am(i,j) (x) ev(j) on the bare matrix (no rescaling here).
template <class S, int D>
HMM_DEV void absorb(float (&P)[D * D], const float (&Am)[D * D], const float (&ev)[D]) {
    float Z[D * D];
    mat_mul<S, D>(P, Am, Z);
#pragma unroll
    for (int i = 0; i < D; ++i)
#pragma unroll
        for (int j = 0; j < D; ++j) P[i * D + j] = S::times(Z[i * D + j], ev[j]);
}

// Aggregate of the lane's chunk: a_{k0-1:k0} (op) ... (op) a_{k1-2:k1-1} over its n valid steps, with its
// scale.  With STORE_E the emission factors replace the log-likelihoods in LDS.  FULL: n == L is known.
//
// The emission factors of all steps are formed first (one straight run of independent loads and
// exponentials), then the chain of products runs from registers in blocks of four steps.
//
// Range (SumProd).  The rows of P are rescaled after every block, each by its own power of two, to a
// largest entry near 2^WORK_BIAS.  Between two rescalings a row's largest entry cannot shrink faster than
// 2^(spread_k) / D per step (the transition rows sum to one); the spreads of a block's steps are added
// up beforehand, and a block that could cost a row more than 2^-WORK_ROOM rescales before every step
// instead (decided per wavefront): a row's largest entry never falls below 2^(WORK_BIAS-WORK_ROOM-spread of
// one step), and entries 2^-126 below it are still normal numbers.  A state is therefore lost only where a
// step-by-step recursion in single precision loses it as well.
template <class S, int D>
struct ChunkFactors {
    using C = SmallCfg<D>;
    float E[C::L][D];       // emission factors of the lane's steps
    float lost[C::L / 4];   // SumProd: bound on the binary logarithm of what a row can lose during a block of four steps
    float csum;             // whole bits taken out of the factors (at most L steps: exact in float unless the log-likelihoods are astronomically large)
};

template <class S, int D, bool STORE_E, bool FULL>
HMM_DEV void chunk_emissions(float* row, int n, ChunkFactors<S, D>& F) {
    using C = SmallCfg<D>;
    static_assert(C::L % 4 == 0, "blocks of four steps");
    constexpr float PER_STEP = (D <= 2) ? 1.0f : (D <= 4) ? 2.0f : 3.0f;   // log2 D
    F.csum = 0.0f;
#pragma unroll
    for (int b = 0; b < C::L / 4; ++b) F.lost[b] = 0.0f;
#pragma unroll
    for (int k = 0; k < C::L; ++k) {
        if (FULL || k < n) {
            float bits, spread;
            lds_read_vec<D>(row + k * D, F.E[k]);
            emission<S, D>(F.E[k], bits, spread);
            if constexpr (STORE_E) lds_write_vec<D>(row + k * D, F.E[k]);
            F.csum += bits;
            F.lost[k / 4] += spread - PER_STEP;
        }
    }
}

// U: uniform mode (see the *_u operations): `bad` reports that the general operations are needed.
template <class S, int D, bool FULL, bool U>
HMM_DEV void chunk_products(const ChunkFactors<S, D>& F, int n, bool first, const float (&Am)[D * D], Agg<S, D>& P,
                            bool& bad) {
    using C = SmallCfg<D>;
    agg_identity<S, D>(P);
#pragma unroll
    for (int b = 0; b < C::L / 4; ++b) {
        if (FULL || 4 * b < n) {
            bool tight = false;
            if constexpr (!S::is_max_plus) {
                if constexpr (U) bad = bad || (F.lost[b] < -(float)WORK_ROOM);
                else tight = wave_any(F.lost[b] < -(float)WORK_ROOM);
            }
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                const int k = 4 * b + kk;
                if (FULL || k < n) {
                    if (k == 0) {
                        // P is still the neutral element: P (op) psi = psi, no product needed
                        float es[D];
#pragma unroll
                        for (int j = 0; j < D; ++j) es[j] = S::is_max_plus ? F.E[0][j] : ldexpf(F.E[0][j], WORK_BIAS);
#pragma unroll
                        for (int i = 0; i < D; ++i)
#pragma unroll
                            for (int j = 0; j < D; ++j) {
                                const float a = first ? ((i == j) ? S::one() : S::zero()) : Am[i * D + j];
                                P.m[i * D + j] = S::times(a, es[j]);
                            }
                        if constexpr (!S::is_max_plus) {
#pragma unroll
                            for (int i = 0; i < D; ++i) P.ex[i] = -WORK_BIAS;
                        }
                    } else {
                        if constexpr (!U) {
                            if (tight && kk > 0) agg_renorm<S, D, WORK_BIAS>(P);
                        }
                        absorb<S, D>(P.m, Am, F.E[k]);
                    }
                }
            }
            if (4 * b + 4 == C::L) agg_renorm_m<U, S, D, ROW_BIAS>(P, bad);   // (b is a constant once the loop is unrolled)
            else agg_renorm_m<U, S, D, WORK_BIAS>(P, bad);
        }
    }
    if constexpr (!FULL) agg_renorm_m<U, S, D, ROW_BIAS>(P, bad);
    P.c += (double)F.csum;
}

template <class S, int D, bool STORE_E, bool FULL>
HMM_DEV void chunk_aggregate_impl(float* row, int n, bool first, const float (&Am)[D * D], Agg<S, D>& P) {
    ChunkFactors<S, D> F;
    bool unused = false;
    chunk_emissions<S, D, STORE_E, FULL>(row, n, F);
    chunk_products<S, D, FULL, false>(F, n, first, Am, P, unused);
}

template <class S, int D, bool STORE_E>
HMM_DEV void chunk_aggregate(float* row, int n, bool first, const float (&Am)[D * D], Agg<S, D>& P) {
    if (n == SmallCfg<D>::L) chunk_aggregate_impl<S, D, STORE_E, true>(row, n, first, Am, P);
    else chunk_aggregate_impl<S, D, STORE_E, false>(row, n, first, Am, P);
}

// The same, in uniform mode where the data allow it (decided per wavefront).  uni: every lane's P came out
// of the uniform operations (its row exponents are all equal).
template <class S, int D, bool STORE_E, bool FULL>
HMM_DEV bool chunk_aggregate_auto_impl(float* row, int n, bool first, const float (&Am)[D * D], Agg<S, D>& P) {
    ChunkFactors<S, D> F;
    chunk_emissions<S, D, STORE_E, FULL>(row, n, F);
    bool bad = false;
    chunk_products<S, D, FULL, true>(F, n, first, Am, P, bad);
    if constexpr (S::is_max_plus) return false;
    if (!wave_any(bad)) return false;
    chunk_products<S, D, FULL, false>(F, n, first, Am, P, bad);
    return true;
}

template <class S, int D, bool STORE_E>
HMM_DEV void chunk_aggregate_auto(float* row, int n, bool first, const float (&Am)[D * D], Agg<S, D>& P, bool& uni) {
    bool general;
    if (n == SmallCfg<D>::L) general = chunk_aggregate_auto_impl<S, D, STORE_E, true>(row, n, first, Am, P);
    else general = chunk_aggregate_auto_impl<S, D, STORE_E, false>(row, n, first, Am, P);
    uni = !wave_any(general);
}

// ---------------------------------------------------------------------------------------------
// Moving aggregates between lanes and through LDS
template <int CTRL, int ROW_MASK>
HMM_DEV float dpp_move(float neutral, float src) {
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(neutral), __float_as_int(src), CTRL, ROW_MASK,
                                                      0xF, false));
}
// The same with 0.0 for lanes without a source.  Where every row of lanes takes part (ROW_MASK 0xF), the zero is the
// DPP read's own fill value for a missing source lane and the destination needs no initialising move.
template <int CTRL, int ROW_MASK>
HMM_DEV float dpp_move_or_zero(float src) {
    if constexpr (ROW_MASK == 0xF)
        return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(src), CTRL, 0xF, 0xF, true));
    else
        return dpp_move<CTRL, ROW_MASK>(0.0f, src);
}
template <int CTRL, int ROW_MASK>
HMM_DEV int dpp_move_int(int neutral, int src) {
    return __builtin_amdgcn_update_dpp(neutral, src, CTRL, ROW_MASK, 0xF, false);
}
template <int CTRL, int ROW_MASK>
HMM_DEV int dpp_move_int_or_zero(int src) {   // as dpp_move_or_zero
    return __builtin_amdgcn_update_dpp(0, src, CTRL, ROW_MASK, 0xF, ROW_MASK == 0xF);
}
template <int CTRL, int ROW_MASK>
HMM_DEV double dpp_move_double(double src) {   // neutral 0.0
    const long long b = __double_as_longlong(src);
    const int lo = dpp_move_int_or_zero<CTRL, ROW_MASK>((int)b);
    const int hi = dpp_move_int_or_zero<CTRL, ROW_MASK>((int)(b >> 32));
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}

// The aggregate of the lane that the DPP control selects; lanes without a source get the neutral element.
template <class S, int D, int CTRL, int ROW_MASK, bool TRACK_C>
HMM_DEV void agg_dpp(const Agg<S, D>& Q, Agg<S, D>& N) {
#pragma unroll
    for (int i = 0; i < D; ++i)
#pragma unroll
        for (int j = 0; j < D; ++j)
            if constexpr (!S::is_max_plus) {   // neutral element: ones on the diagonal, zeros elsewhere
                N.m[i * D + j] = (i == j) ? dpp_move<CTRL, ROW_MASK>(1.0f, Q.m[i * D + j])
                                          : dpp_move_or_zero<CTRL, ROW_MASK>(Q.m[i * D + j]);
            } else {                           // zeros on the diagonal, minus infinity elsewhere
                N.m[i * D + j] = (i == j) ? dpp_move_or_zero<CTRL, ROW_MASK>(Q.m[i * D + j])
                                          : dpp_move<CTRL, ROW_MASK>(-INFINITY, Q.m[i * D + j]);
            }
    if constexpr (!S::is_max_plus) {
#pragma unroll
        for (int i = 0; i < D; ++i) N.ex[i] = dpp_move_int_or_zero<CTRL, ROW_MASK>(Q.ex[i]);
    }
    if constexpr (TRACK_C) N.c = dpp_move_double<CTRL, ROW_MASK>(Q.c);
    else N.c = 0.0;
}

// The aggregate held by lane `src` of the wavefront (any permutation).
template <class S, int D, bool TRACK_C>
HMM_DEV void agg_shfl(const Agg<S, D>& Q, int src, Agg<S, D>& N) {
#pragma unroll
    for (int e = 0; e < D * D; ++e) N.m[e] = __shfl(Q.m[e], src, 64);
    if constexpr (!S::is_max_plus) {
#pragma unroll
        for (int i = 0; i < D; ++i) N.ex[i] = __shfl(Q.ex[i], src, 64);
    }
    if constexpr (TRACK_C) N.c = __shfl(Q.c, src, 64);
    else N.c = 0.0;
}

// LDS / memory image of an aggregate: D*D floats, D exponents, the common scale as a double.
template <int D>
struct AggImage {
    static constexpr int WORDS = D * D + D + 2;   // D (D + 1) is even: the double is 8-byte aligned
};

template <class S, int D>
HMM_DEV void agg_store(float* p, const Agg<S, D>& Q) {
#pragma unroll
    for (int e = 0; e < D * D; ++e) p[e] = Q.m[e];
#pragma unroll
    for (int i = 0; i < D; ++i) reinterpret_cast<int*>(p)[D * D + i] = S::is_max_plus ? 0 : Q.ex[i];
    *reinterpret_cast<double*>(p + D * D + D) = Q.c;
}

template <class S, int D>
HMM_DEV void agg_load(const float* p, Agg<S, D>& Q) {
#pragma unroll
    for (int e = 0; e < D * D; ++e) Q.m[e] = p[e];
#pragma unroll
    for (int i = 0; i < D; ++i) Q.ex[i] = reinterpret_cast<const int*>(p)[D * D + i];
    Q.c = *reinterpret_cast<const double*>(p + D * D + D);
}

// ---------------------------------------------------------------------------------------------
// Wave-level scans of chunk aggregates over the 64 lanes of a wavefront, moved with DPP:
// four shifts inside each row of 16 lanes, then the last lane of a row broadcast to the next
// row(s).  A lane that has no source at some level combines with the operator's neutral
// element instead, so no lane needs to be predicated.
template <class S, int D, bool SWAP, int CTRL, int ROW_MASK, bool TRACK_C, bool U, int UBIAS = ROW_BIAS>
HMM_DEV void wave_scan_level(Agg<S, D>& Q, bool& bad) {
    Agg<S, D> N, Z;
    agg_dpp<S, D, CTRL, ROW_MASK, TRACK_C>(Q, N);
    if constexpr (U && !S::is_max_plus && UBIAS != ROW_BIAS) {
        if constexpr (SWAP) agg_mul_u<D, TRACK_C, UBIAS>(Q, N, Z, bad);
        else agg_mul_u<D, TRACK_C, UBIAS>(N, Q, Z, bad);
    } else if constexpr (S::is_max_plus && UBIAS != ROW_BIAS) {   // (max,+): a level that does not shift
        if constexpr (SWAP) agg_mul<S, D, TRACK_C, false>(Q, N, Z);
        else agg_mul<S, D, TRACK_C, false>(N, Q, Z);
    } else {
        if constexpr (SWAP) agg_mul_m<U, S, D, TRACK_C>(Q, N, Z, bad);
        else agg_mul_m<U, S, D, TRACK_C>(N, Q, Z, bad);
    }
    Q = Z;
}

template <class S, int D, bool SWAP, int CTRL, int ROW_MASK, bool TRACK_C>
HMM_DEV void wave_scan_level(Agg<S, D>& Q) {
    bool unused = false;
    wave_scan_level<S, D, SWAP, CTRL, ROW_MASK, TRACK_C, false>(Q, unused);
}

// Inclusive scan towards higher lanes.  SWAP = false: Q_t <- P_0 (op) ... (op) P_t;
// SWAP = true: Q_t <- P_t (op) ... (op) P_0 (the operator's arguments exchanged).
// U: uniform mode, `bad` as in the *_u operations.
template <class S, int D, bool SWAP, bool TRACK_C, bool U>
HMM_DEV void wave_scan_up(Agg<S, D>& Q, bool& bad) {
    if constexpr (U && !S::is_max_plus) {
        // Uniform mode renormalises after every other level only.  Rows enter with their largest entry below
        // 2^ROW_BIAS; a renormalising level leaves it in [2^(MID-1), 2^MID), the next level's products are
        // then below D 2^(2 MID) and are left as they are, and the products of those stay below
        // D^3 2^(4 MID) <= 2^121 for D <= 8.  Downwards, a renormalising level has checked that every
        // row's largest entry is at least 2^(MID-21), so after the level without renormalisation it is at least
        // 2^(2 MID - 42) = 2^14: entries 2^-126 below their row's largest are still normal numbers.  The last
        // level restores ROW_BIAS.  Powers of two are exact factors: the results have the mantissas they would
        // have with a renormalisation at every level.
        constexpr int MID = 28, NONE = -1;
        static_assert(D <= 8, "range argument above");
        wave_scan_level<S, D, SWAP, 0x111, 0xF, TRACK_C, U, MID>(Q, bad);    // row_shr:1
        wave_scan_level<S, D, SWAP, 0x112, 0xF, TRACK_C, U, NONE>(Q, bad);   // row_shr:2
        wave_scan_level<S, D, SWAP, 0x114, 0xF, TRACK_C, U, MID>(Q, bad);    // row_shr:4
        wave_scan_level<S, D, SWAP, 0x118, 0xF, TRACK_C, U, NONE>(Q, bad);   // row_shr:8
        wave_scan_level<S, D, SWAP, 0x142, 0xA, TRACK_C, U, MID>(Q, bad);    // row_bcast:15 into rows 1 and 3
        wave_scan_level<S, D, SWAP, 0x143, 0xC, TRACK_C, U>(Q, bad);         // row_bcast:31 into rows 2 and 3
        return;
    }
    if constexpr (S::is_max_plus) {
        // (max,+): the largest entry is moved to zero after every other level only.  Entries are at most zero, so
        // a product's are too; left unshifted for one level they are at most twice as far from zero as they
        // would otherwise be, which costs one bit of absolute precision in that level's sums.
        constexpr int NONE = -1;
        wave_scan_level<S, D, SWAP, 0x111, 0xF, TRACK_C, U, NONE>(Q, bad);   // row_shr:1
        wave_scan_level<S, D, SWAP, 0x112, 0xF, TRACK_C, U>(Q, bad);         // row_shr:2
        wave_scan_level<S, D, SWAP, 0x114, 0xF, TRACK_C, U, NONE>(Q, bad);   // row_shr:4
        wave_scan_level<S, D, SWAP, 0x118, 0xF, TRACK_C, U>(Q, bad);         // row_shr:8
        wave_scan_level<S, D, SWAP, 0x142, 0xA, TRACK_C, U, NONE>(Q, bad);   // row_bcast:15 into rows 1 and 3
        wave_scan_level<S, D, SWAP, 0x143, 0xC, TRACK_C, U>(Q, bad);         // row_bcast:31 into rows 2 and 3
        return;
    }
    wave_scan_level<S, D, SWAP, 0x111, 0xF, TRACK_C, U>(Q, bad);   // row_shr:1
    wave_scan_level<S, D, SWAP, 0x112, 0xF, TRACK_C, U>(Q, bad);   // row_shr:2
    wave_scan_level<S, D, SWAP, 0x114, 0xF, TRACK_C, U>(Q, bad);   // row_shr:4
    wave_scan_level<S, D, SWAP, 0x118, 0xF, TRACK_C, U>(Q, bad);   // row_shr:8
    wave_scan_level<S, D, SWAP, 0x142, 0xA, TRACK_C, U>(Q, bad);   // row_bcast:15 into rows 1 and 3
    wave_scan_level<S, D, SWAP, 0x143, 0xC, TRACK_C, U>(Q, bad);   // row_bcast:31 into rows 2 and 3
}
template <class S, int D, bool SWAP, bool TRACK_C>
HMM_DEV void wave_scan_up(Agg<S, D>& Q) {
    bool unused = false;
    wave_scan_up<S, D, SWAP, TRACK_C, false>(Q, unused);
}

// Q <- inclusive scan of the elements `make()` returns, in uniform mode if every lane's element is uniform (uni,
// a fact about the whole wavefront) and stays so, else with the general operations; uni is updated to describe
// the results.  (make is called again for the second attempt rather than keeping a copy of the elements alive.)
template <class S, int D, bool SWAP, bool TRACK_C, class MAKE>
HMM_DEV void wave_scan_up_auto(Agg<S, D>& Q, bool& uni, MAKE make) {
    make(Q);
    if constexpr (S::is_max_plus) {
        wave_scan_up<S, D, SWAP, TRACK_C>(Q);
    } else {
        if (uni) {
            bool bad = false;
            wave_scan_up<S, D, SWAP, TRACK_C, true>(Q, bad);
            if (!wave_any(bad)) return;
            make(Q);
            uni = false;
        }
        wave_scan_up<S, D, SWAP, TRACK_C>(Q);
    }
}

template <class S, int D>
HMM_DEV void wave_scan_prefix(Agg<S, D>& Q) {   // Q_t <- P_0 (op) ... (op) P_t, scale included
    wave_scan_up<S, D, false, true>(Q);
}

// R_t <- P_t (op) ... (op) P_63: the prefix scan with exchanged arguments on mirrored lanes
// (the reversal recipe of Sec. III-B applied across the wavefront).  The common scale is not
// tracked: only backward potentials come out of it, and those are scale-free.
template <class S, int D>
HMM_DEV void wave_scan_suffix(Agg<S, D>& R) {
    const int mirror = 63 - (int)(threadIdx.x & 63);
    Agg<S, D> T;
    agg_shfl<S, D, false>(R, mirror, T);
    wave_scan_up<S, D, true, false>(T);
    agg_shfl<S, D, false>(T, mirror, R);
}

// R <- P_t (op) ... (op) P_63 from the lanes' P
template <class S, int D>
HMM_DEV void wave_scan_suffix_auto(const Agg<S, D>& P, Agg<S, D>& R, bool& uni) {
    const int mirror = 63 - (int)(threadIdx.x & 63);
    Agg<S, D> T;
    wave_scan_up_auto<S, D, true, false>(T, uni, [&](Agg<S, D>& X) { agg_shfl<S, D, false>(P, mirror, X); });
    agg_shfl<S, D, false>(T, mirror, R);
}

// Sum of one double per lane over the wavefront (every lane gets it).
HMM_DEV double wave_sum(double v) {
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) v += __shfl_xor(v, d, 64);
    return v;
}

// Inclusive prefix scan inside each wave; the wave totals go to wagg[NW][AggImage::WORDS] in LDS.
// The caller must __syncthreads() before reading wagg.  SumProd: the common scale c of an aggregate is a
// plain sum over its elements, so it does not ride along the scan; only the wave total gets it (the scanned
// aggregates Q of the other lanes carry no c).
template <class S, int D>
HMM_DEV void block_prefix(const Agg<S, D>& P, Agg<S, D>& Q, float* wagg) {
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    Q = P;
    if constexpr (S::is_max_plus) {
        wave_scan_up<S, D, false, true>(Q);
    } else {
        wave_scan_up<S, D, false, false>(Q);
        Q.c = wave_sum(P.c);
    }
    if (lane == 63) agg_store<S, D>(wagg + wave * AggImage<D>::WORDS, Q);
}

// The same with the scan in uniform mode where possible; uni: in, the P of every lane of the wavefront are
// uniform; out, so are the Q.
template <class S, int D>
HMM_DEV void block_prefix_auto(const Agg<S, D>& P, Agg<S, D>& Q, float* wagg, bool& uni) {
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    if constexpr (S::is_max_plus) {
        Q = P;
        wave_scan_up<S, D, false, true>(Q);
    } else {
        wave_scan_up_auto<S, D, false, false>(Q, uni, [&](Agg<S, D>& X) { X = P; });
        Q.c = wave_sum(P.c);
    }
    if (lane == 63) agg_store<S, D>(wagg + wave * AggImage<D>::WORDS, Q);
}

// Workgroup aggregate W_0 (op) ... (op) W_{NW-1} from the wave totals (any single lane may call).
template <class S, int D>
HMM_DEV void block_total(const float* wagg, Agg<S, D>& X) {
    using C = SmallCfg<D>;
    agg_load<S, D>(wagg, X);
#pragma unroll
    for (int w = 1; w < C::NW; ++w) {
        Agg<S, D> Y, Z;
        agg_load<S, D>(wagg + w * AggImage<D>::WORDS, Y);
        agg_mul<S, D, true>(X, Y, Z);
        X = Z;
    }
}

// Scale-free vectors: forward potentials are kept with their sum in [0.5, 1) (SumProd) / largest entry 0
// (MaxPlus), backward potentials with their largest entry in [0.5, 1) / at 0.

// Products of the wave totals, formed once per workgroup by wave_products (below) while nothing else is
// pending: wpre[w-1] = W_0 (op) ... (op) W_{w-1} and wsuf[w-1] = W_w (op) ... (op) W_{NW-1} for w = 1 .. NW-1,
// as aggregate images.  With them a lane reaches its carries in two steps instead of up to NW.
template <int D>
struct WaveProducts {
    static constexpr int W = AggImage<D>::WORDS;
    alignas(8) float wpre[(SmallCfg<D>::NW - 1) * W];
    alignas(8) float wsuf[(SmallCfg<D>::NW - 1) * W];
};

// fin = cin_f (op) P_0 (op) ... (op) P_{t-1}: the forward potential just before lane t's chunk,
// from the lane's inclusive wave prefix Q and the wave totals (wp != nullptr: their products).
// U: uniform mode (Q must be uniform; `bad` reports a wave product that is not).
template <class S, int D, bool U>
HMM_DEV void carry_forward(const Agg<S, D>& Q, const float* wagg, const WaveProducts<D>* wp, const float (&cin_f)[D],
                           float (&fin)[D], bool& bad) {
    using C = SmallCfg<D>;
    constexpr int W = AggImage<D>::WORDS;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    float fw[D];
#pragma unroll
    for (int j = 0; j < D; ++j) fw[j] = cin_f[j];
    auto through = [&](const float* src) {
        Agg<S, D> Wm;
        float r[D];
        agg_load<S, D>(src, Wm);
        if constexpr (U && !S::is_max_plus) bad = bad || !agg_is_uniform<D>(Wm);
        vec_agg_m<U, S, D>(fw, Wm, r);
#pragma unroll
        for (int j = 0; j < D; ++j) fw[j] = r[j];
    };
    if (wp != nullptr) {
        if (wave > 0) through(wp->wpre + (wave - 1) * W);
    } else {
#pragma unroll
        for (int w = 0; w < C::NW - 1; ++w) {
            if (w < wave) through(wagg + w * W);
        }
    }
    Agg<S, D> Qp;
    float r[D];
    agg_dpp<S, D, 0x138, 0xF, false>(Q, Qp);   // wave_shr:1, the lane below (lane 0 gets the neutral element and does not use it)
    vec_agg_m<U, S, D>(fw, Qp, r);
#pragma unroll
    for (int j = 0; j < D; ++j) fin[j] = (lane == 0) ? fw[j] : r[j];
}
template <class S, int D>
HMM_DEV void carry_forward(const Agg<S, D>& Q, const float* wagg, const WaveProducts<D>* wp, const float (&cin_f)[D],
                           float (&fin)[D]) {
    bool unused = false;
    carry_forward<S, D, false>(Q, wagg, wp, cin_f, fin, unused);
}
// uni: every lane's Q is uniform
template <class S, int D>
HMM_DEV void carry_forward_auto(const Agg<S, D>& Q, bool uni, const float* wagg, const WaveProducts<D>* wp,
                                const float (&cin_f)[D], float (&fin)[D]) {
    if constexpr (!S::is_max_plus) {
        if (uni) {
            bool bad = false;
            carry_forward<S, D, true>(Q, wagg, wp, cin_f, fin, bad);
            if (!wave_any(bad)) return;
        }
    }
    carry_forward<S, D>(Q, wagg, wp, cin_f, fin);
}

// The backward potential at the last step of lane t's chunk, P_{t+1} (op) ... (op) P_{NT-1} (op) cin_b, from the
// lane's inclusive wave suffix R and the wave totals, as a vector of mantissas with one exponent per entry
// (SumProd; EX_NONE marks a zero) -- the chunk's backward recursion picks the common scale itself, see
// backward_plain -- or shifted to largest entry 0 (MaxPlus; the exponents are not used).
template <class S, int D, bool U>
HMM_DEV void carry_backward(const Agg<S, D>& R, const float* wagg, const WaveProducts<D>* wp, const float (&cin_b)[D],
                            float (&bout)[D], int (&bex)[D], bool& bad) {
    using C = SmallCfg<D>;
    constexpr int W = AggImage<D>::WORDS;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    float bw[D];
#pragma unroll
    for (int j = 0; j < D; ++j) bw[j] = cin_b[j];
    auto through = [&](const float* src) {
        Agg<S, D> Wm;
        float r[D];
        agg_load<S, D>(src, Wm);
        if constexpr (U && !S::is_max_plus) bad = bad || !agg_is_uniform<D>(Wm);
        agg_vec_m<U, S, D>(Wm, bw, r);
#pragma unroll
        for (int j = 0; j < D; ++j) bw[j] = r[j];
    };
    if (wp != nullptr) {
        if (wave < C::NW - 1) through(wp->wsuf + wave * W);   // W_{wave+1} (op) ... (op) W_{NW-1}
    } else {
#pragma unroll
        for (int w = C::NW - 1; w > 0; --w) {
            if (w > wave) through(wagg + w * W);
        }
    }
    Agg<S, D> Rn;
    agg_dpp<S, D, 0x130, 0xF, false>(R, Rn);   // wave_shl:1, the lane above (lane 63 gets the neutral element and does not use it)
    if constexpr (S::is_max_plus) {
        float r[D];
        agg_vec<S, D>(Rn, bw, r);
#pragma unroll
        for (int j = 0; j < D; ++j) {
            bout[j] = (lane == 63) ? bw[j] : r[j];
            bex[j] = 0;
        }
    } else {
        float r[D];
        int er[D];
        agg_vec_raw<D>(Rn, bw, r, er);
#pragma unroll
        for (int j = 0; j < D; ++j) {
            bout[j] = (lane == 63) ? bw[j] : r[j];
            bex[j] = (lane == 63) ? ((bw[j] > 0.0f) ? 0 : EX_NONE) : er[j];
        }
    }
}

template <class S, int D>
HMM_DEV void carry_backward(const Agg<S, D>& R, const float* wagg, const WaveProducts<D>* wp, const float (&cin_b)[D],
                            float (&bout)[D], int (&bex)[D]) {
    bool unused = false;
    carry_backward<S, D, false>(R, wagg, wp, cin_b, bout, bex, unused);
}
// uni: every lane's R is uniform (the last step, R against the wave's vector, is the same in both modes)
template <class S, int D>
HMM_DEV void carry_backward_auto(const Agg<S, D>& R, bool uni, const float* wagg, const WaveProducts<D>* wp,
                                 const float (&cin_b)[D], float (&bout)[D], int (&bex)[D]) {
    if constexpr (!S::is_max_plus) {
        if (uni) {
            bool bad = false;
            carry_backward<S, D, true>(R, wagg, wp, cin_b, bout, bex, bad);
            if (!wave_any(bad)) return;
        }
    }
    carry_backward<S, D>(R, wagg, wp, cin_b, bout, bex);
}

// Both carries for every lane of the workgroup (contains one __syncthreads()); the backward one in the raw
// form of carry_backward.
template <class S, int D, bool BWD>
HMM_DEV void block_exchange(const Agg<S, D>& P, const float (&cin_f)[D], const float (&cin_b)[D],
                            float (&fin)[D], float (&bout)[D], int (&bex)[D], float* wagg) {
    Agg<S, D> Q;
    block_prefix<S, D>(P, Q, wagg);
    __syncthreads();
    carry_forward<S, D>(Q, wagg, nullptr, cin_f, fin);
    if constexpr (BWD) {
        Agg<S, D> R = P;
        wave_scan_suffix<S, D>(R);
        carry_backward<S, D>(R, wagg, nullptr, cin_b, bout, bex);
    }
}

// The evidence of a whole sequence from its start vector and the aggregate of all its elements:
// log of sum_j (start (op) M)(j) for SumProd (log Z of Sec. II), max_j for MaxPlus (Corollary 1).
// `start` is the prior in the operator's domain, taken exactly as given.
template <class S, int D>
HMM_DEV double sequence_evidence(const float (&start)[D], const Agg<S, D>& M) {
    float r[D];
    const double sc = vec_agg<S, D>(start, M, r);
    if constexpr (S::is_max_plus) {
        return M.c + sc;   // r has its largest entry at 0
    } else {
        return 0.6931471805599453 * (M.c + sc) + log((double)sum_of(r));
    }
}

// The same from the forward potential v entering a span (with the scale vs it has been stripped of:
// bits for SumProd, an offset for MaxPlus), the span's aggregate M, and the backward potential b after it
// (scale bs): log of v M b.
template <class S, int D>
HMM_DEV double span_evidence(const float (&v)[D], double vs, const Agg<S, D>& M, const float (&b)[D], double bs) {
    float r[D];
    const double sc = vec_agg<S, D>(v, M, r);
    if constexpr (S::is_max_plus) {
        float best = r[0] + b[0];
#pragma unroll
        for (int j = 1; j < D; ++j) best = fmaxf(best, r[j] + b[j]);
        return vs + M.c + sc + bs + (double)best;
    } else {
        float dot = r[0] * b[0];
#pragma unroll
        for (int j = 1; j < D; ++j) dot = fmaf(r[j], b[j], dot);
        return 0.6931471805599453 * (vs + M.c + sc + bs) + log((double)dot);
    }
}

// ---------------------------------------------------------------------------------------------
// Sum-product work inside a lane's chunk

// Forward: a_{0:k} for the lane's steps, kept in registers as F (Theorem 1).  f enters as the
// carry (or the prior for the sequence's first chunk) and every step is rescaled by an exact power
// of two, to a sum near 2^VEC_BIAS: states down to 2^-(126+VEC_BIAS) of the step's total stay normal
// numbers, and the backward potential, kept at the same height, may weigh them up again.
template <int D, bool WRITE_FILT, bool FULL>
HMM_DEV void sp_forward_impl(const float* row, int n, bool first, const float (&Am)[D * D], float (&f)[D],
                             float (&F)[SmallCfg<D>::L][D], float* __restrict__ filt_dst) {
    using C = SmallCfg<D>;
    using S = SumProd;
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
            const int ex = __builtin_amdgcn_frexp_expf(s) - VEC_BIAS;   // the sum comes to lie in [2^(VEC_BIAS-1), 2^VEC_BIAS)
#pragma unroll
            for (int j = 0; j < D; ++j) F[k][j] = f[j] = ldexpf(g[j], -ex);
            if constexpr (WRITE_FILT) {
                const float inv = __builtin_amdgcn_rcpf(ldexpf(s, -ex));
#pragma unroll
                for (int j = 0; j < D; ++j) filt_dst[k * D + j] = f[j] * inv;
            }
        }
    }
}

// Common scale of a backward potential given as mantissas b with one exponent per entry (bex; EX_NONE marks
// a zero): largest entry into [2^(VEC_BIAS-1), 2^VEC_BIAS).
template <int D>
HMM_DEV void backward_plain(float (&b)[D], const int (&bex)[D]) {
    int e[D], ref = EX_NONE;
#pragma unroll
    for (int i = 0; i < D; ++i) {
        e[i] = (bex[i] != EX_NONE) ? __builtin_amdgcn_frexp_expf(b[i]) + bex[i] : EX_NONE;
        ref = e[i] > ref ? e[i] : ref;
    }
#pragma unroll
    for (int i = 0; i < D; ++i) b[i] = (bex[i] != EX_NONE) ? ldexpf(b[i], max_of_int(bex[i] - ref + VEC_BIAS, -400)) : 0.0f;
}

// Backward: a_{k:T+1} (Theorem 2) and the marginal f_k b_k / Z_k, written over the emission
// factors in LDS.  b enters as the backward potential at the chunk's last step in the raw form of
// carry_backward; every step rescales it to a largest entry near 2^VEC_BIAS.
// COUNTS: also accumulate the pairwise posteriors of the transitions INTO the lane's steps (the expectation
// step's statistic, Sec. V-C), p(x_{k-1}=i, x_k=j | y) = f_{k-1}(i) A(i,j) e_k(j) b_k(j) / s_k, where
// s_k = sum_i f_{k-1}(i) (A (e_k o b_k))(i) is the normaliser of the marginal at k-1: with t = e_k o b_k and
// r = A t already formed for the backward step, that is acc(i,j) += (f_{k-1}(i) / s_k) t(j); the factor A(i,j) is
// applied once at the end by the caller, which also discards the sums of forbidden transitions (A(i,j) = 0: their
// terms are not posteriors and may have overflowed).  fin = forward potential entering the chunk (f_{k-1} for the chunk's
// first step; unused where that step is the sequence's first, which has no transition).  The potentials are
// the scaled ones (largest entries near 2^VEC_BIAS): nothing is lost that the marginals themselves keep.
template <int D, bool FULL, bool COUNTS>
HMM_DEV void sp_backward_impl(float* row, int n, bool first, const float (&Am)[D * D], float (&b)[D],
                              const int (&bex)[D], const float (&F)[SmallCfg<D>::L][D], const float (&fin)[D],
                              float (&acc)[COUNTS ? D * D : 1]) {
    using C = SmallCfg<D>;
    using S = SumProd;
    backward_plain<D>(b, bex);
    // bn = r 2^-ex is the rescaled backward potential of step k-1: the normaliser is taken against it (a plain
    // number near 2^(2 VEC_BIAS) even where r itself is far down), and 2^-ex goes into the left factor
    auto pair_sums = [&](const float (&fprev)[D], const float (&t)[D], const float (&bn)[D], int ex) {
        float s = fprev[0] * bn[0];
#pragma unroll
        for (int i = 1; i < D; ++i) s = fmaf(fprev[i], bn[i], s);
        const float inv = (s > 0.0f) ? __builtin_amdgcn_rcpf(s) : 0.0f;
#pragma unroll
        for (int i = 0; i < D; ++i) {
            const float w = ldexpf(fprev[i] * inv, -ex);
#pragma unroll
            for (int j = 0; j < D; ++j) acc[i * D + j] = fmaf(w, t[j], acc[i * D + j]);
        }
    };
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
            if (k > 0 || (COUNTS && !first)) {
                float t[D], r[D];
#pragma unroll
                for (int j = 0; j < D; ++j) t[j] = ev[j] * b[j];
                mat_vec<S, D>(Am, t, r);
                const int ex = __builtin_amdgcn_frexp_expf(max_of(r)) - VEC_BIAS;
#pragma unroll
                for (int j = 0; j < D; ++j) b[j] = ldexpf(r[j], -ex);
                if constexpr (COUNTS) {
                    if (k > 0) pair_sums(F[k - 1], t, b, ex);
                    else pair_sums(fin, t, b, ex);
                }
            }
        }
    }
}

template <int D, bool FULL>
HMM_DEV void mp_forward_impl(const float* row, int n, bool first, const float (&Am)[D * D], float (&v)[D],
                               uint32_t (&bp)[SmallCfg<D>::W]) {
    using C = SmallCfg<D>;
    using S = MaxPlus;
#pragma unroll
    for (int w = 0; w < C::W; ++w) bp[w] = 0u;
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
            renorm<S, D>(g);
#pragma unroll
            for (int j = 0; j < D; ++j) v[j] = g[j];
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Max-product forward/backward work inside a lane's chunk (the lemma of Sec. IV-C on logarithms).

// Forward: psi~^f_k for the lane's steps, kept in registers as F, each step shifted to max 0.
// v enters as the carry (max 0, or the log prior for the sequence's first chunk).
template <int D, bool FULL>
HMM_DEV void mpv_forward_impl(const float* row, int n, bool first, const float (&Am)[D * D], float (&v)[D],
                                float (&F)[SmallCfg<D>::L][D]) {
    using C = SmallCfg<D>;
    using S = MaxPlus;
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
            renorm<S, D>(g);
#pragma unroll
            for (int j = 0; j < D; ++j) F[k][j] = v[j] = g[j];
        }
    }
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
    bool live;   // the lane belongs to a sequence of the batch
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
    p.live = live;
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
template <class S, int D, bool SWAP, int CTRL, int ROW_MASK, bool TRACK_C>
HMM_DEV void wave_scan_level_if(Agg<S, D>& Q, bool take) {
    Agg<S, D> N, I, Z;
    agg_dpp<S, D, CTRL, ROW_MASK, TRACK_C>(Q, N);
    agg_identity<S, D>(I);
#pragma unroll
    for (int e = 0; e < D * D; ++e) N.m[e] = take ? N.m[e] : I.m[e];
#pragma unroll
    for (int i = 0; i < D; ++i) N.ex[i] = take ? N.ex[i] : 0;
    N.c = take ? N.c : 0.0;
    if constexpr (SWAP) agg_mul<S, D, TRACK_C>(Q, N, Z);
    else agg_mul<S, D, TRACK_C>(N, Q, Z);
    Q = Z;
}

// Inclusive scan towards higher lanes inside every aligned group of 2^lcpl lanes.
template <class S, int D, bool SWAP, bool TRACK_C>
HMM_DEV void group_scan_up(Agg<S, D>& Q, int lcpl) {
    const int pos = (int)(threadIdx.x & 63) & ((1 << lcpl) - 1);
    if (lcpl > 0) wave_scan_level_if<S, D, SWAP, 0x111, 0xF, TRACK_C>(Q, pos >= 1);   // row_shr:1
    if (lcpl > 1) wave_scan_level_if<S, D, SWAP, 0x112, 0xF, TRACK_C>(Q, pos >= 2);   // row_shr:2
    if (lcpl > 2) wave_scan_level_if<S, D, SWAP, 0x114, 0xF, TRACK_C>(Q, pos >= 4);   // row_shr:4
    if (lcpl > 3) wave_scan_level_if<S, D, SWAP, 0x118, 0xF, TRACK_C>(Q, pos >= 8);   // row_shr:8
    if (lcpl > 4) wave_scan_level<S, D, SWAP, 0x142, 0xA, TRACK_C>(Q);               // row_bcast:15 into rows 1 and 3
    if (lcpl > 5) wave_scan_level<S, D, SWAP, 0x143, 0xC, TRACK_C>(Q);               // row_bcast:31 into rows 2 and 3
}

// Forward potential entering every chunk and backward potential at every chunk's last step (in the raw form of
// carry_backward), for sequences that start from `start` (the prior, in the operator's domain) and end inside
// their group; Q receives the lane's inclusive prefix inside its group (the group's last lane then holds the
// whole sequence's aggregate).
template <class S, int D, bool BWD>
HMM_DEV void group_exchange(const Agg<S, D>& P, int lcpl, int c, const float (&start)[D], float (&fin)[D],
                            float (&bout)[D], int (&bex)[D], Agg<S, D>& Q) {
    float r[D];
    Q = P;
    group_scan_up<S, D, false, true>(Q, lcpl);
    Agg<S, D> Qp;
    agg_shfl<S, D, false>(Q, ((int)(threadIdx.x & 63) + 63) & 63, Qp);
    vec_agg<S, D>(start, Qp, r);
#pragma unroll
    for (int j = 0; j < D; ++j) fin[j] = (c == 0) ? start[j] : r[j];
    if constexpr (BWD) {
        const int mirror = 63 - (int)(threadIdx.x & 63);
        Agg<S, D> R, T;
        float ones[D];
        agg_shfl<S, D, false>(P, mirror, T);
        group_scan_up<S, D, true, false>(T, lcpl);
        agg_shfl<S, D, false>(T, mirror, R);
        Agg<S, D> Rn;
        agg_shfl<S, D, false>(R, ((int)(threadIdx.x & 63) + 1) & 63, Rn);
#pragma unroll
        for (int j = 0; j < D; ++j) ones[j] = S::one();
        const bool last = c == (1 << lcpl) - 1;
        if constexpr (S::is_max_plus) {
            agg_vec<S, D>(Rn, ones, r);
#pragma unroll
            for (int j = 0; j < D; ++j) {
                bout[j] = last ? ones[j] : r[j];
                bex[j] = 0;
            }
        } else {
            int er[D];
            agg_vec_raw<D>(Rn, ones, r, er);
#pragma unroll
            for (int j = 0; j < D; ++j) {
                bout[j] = last ? 1.0f : r[j];
                bex[j] = last ? 0 : er[j];
            }
        }
    }
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
// Exchange between co-resident workgroups (single-launch kernels) through tagged words.
//
// A published 32-bit value travels as one 64-bit word {value, tag}; the tag names the call.  The
// exchange region of a workspace starts with a header {generation, poison, sequences finished}: every
// workgroup of a call reads the generation g when it starts and uses the tag g + 1; when the call's
// last sequence has been dealt with, one workgroup stores g + 1 as the new generation, so that
// whatever a later call finds in the slots carries an older tag and is ignored -- nothing has to be
// cleared between calls.  (The region must be zero before its first use: tags start at 1.)
// A producer writes its slots with agent-scope (write-through) stores, consumers poll them with
// agent-scope (cache-bypassing) loads until every word carries the call's tag.  Each word is written by
// one store, so a consumer never sees a torn word, and no ordering between different words is relied
// upon: no flags, no fences (an agent-scope fence writes back / invalidates a whole L2 on this
// multi-die part), and read-modify-write atomics only once per sequence, after its results are out.
// The poll is bounded so that every wave terminates even if the workgroups were, against the host's
// residency check, not all resident; such a call marks the region as poisoned (its workgroups may
// disagree about the generation), and every later call on it gives up at once, with NaN evidence,
// until the region has been zeroed again.
constexpr int SPIN_LIMIT = 1 << 20;

struct XchHeader {
    uint32_t generation;   // tag of the last completed call
    uint32_t poison;       // nonzero: a wait ran out in an earlier call, the region must be re-initialised
    uint32_t seq_done;     // sequences of the running call whose results are out
    uint32_t pad;
};

template <class T>
HMM_DEV void coherent_store(T* p, T v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <class T>
HMM_DEV T coherent_load(const T* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

HMM_DEV unsigned long long tagged(uint32_t value, uint32_t tag) {
    return ((unsigned long long)tag << 32) | (unsigned long long)value;
}
HMM_DEV void publish_word(unsigned long long* slot, uint32_t value, uint32_t tag) { coherent_store(slot, tagged(value, tag)); }
HMM_DEV void publish_word(unsigned long long* slot, float value, uint32_t tag) {
    coherent_store(slot, tagged(__float_as_uint(value), tag));
}

}  // namespace hmm
