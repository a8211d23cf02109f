// Register-resident D x D element algebra for the two associative operators of the paper:
//   SumProd : Definition 3, (a (x) b)(x_i,x_k) = sum_{x_j} a(x_i,x_j) b(x_j,x_k)
//   MaxPlus : Definition 5 on logarithms, (a v b)(x_i,x_k) = max_{x_j} [a(x_i,x_j) + b(x_j,x_k)]
// Matrices are row-major float[D*D] with compile-time indices only, so they live in VGPRs.
//
// The plain float[D*D] helpers below carry no scale (used by the block-element kernels, which
// keep their own); the scans of the inference calls work on Agg<S, D> further down, a matrix
// together with what was removed from it to keep it in range.
#pragma once
#include <hip/hip_runtime.h>

namespace hmm {

#define HMM_DEV __device__ __forceinline__

struct SumProd {
    static constexpr bool is_max_plus = false;
    HMM_DEV static float zero() { return 0.0f; }
    HMM_DEV static float one() { return 1.0f; }
    HMM_DEV static float times(float a, float b) { return a * b; }
    HMM_DEV static float mul_add(float acc, float a, float b) { return fmaf(a, b, acc); }
};

struct MaxPlus {
    static constexpr bool is_max_plus = true;
    HMM_DEV static float zero() { return -INFINITY; }
    HMM_DEV static float one() { return 0.0f; }
    HMM_DEV static float times(float a, float b) { return a + b; }
    HMM_DEV static float mul_add(float acc, float a, float b) { return fmaxf(acc, a + b); }
};

template <int N>
HMM_DEV float max_of(const float (&v)[N]) {
    float m = v[0];
#pragma unroll
    for (int i = 1; i < N; ++i) m = fmaxf(m, v[i]);
    return m;
}

template <int N>
HMM_DEV float sum_of(const float (&v)[N]) {
    float s = v[0];
#pragma unroll
    for (int i = 1; i < N; ++i) s += v[i];
    return s;
}

// Bring an element back into range.  Returns what was removed: for SumProd the binary exponent
// ex (the element was multiplied by 2^-ex), for MaxPlus the subtracted offset.
template <class S, int N>
HMM_DEV float renorm(float (&v)[N]) {
    if constexpr (S::is_max_plus) {
        float m = max_of(v);
        m = (m == -INFINITY) ? 0.0f : m;
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] -= m;
        return m;
    } else {
        const float m = max_of(v);
        const int ex = __builtin_amdgcn_frexp_expf(m);   // 0 for m == 0
#pragma unroll
        for (int i = 0; i < N; ++i) v[i] = ldexpf(v[i], -ex);
        return (float)ex;
    }
}

template <class S, int D>
HMM_DEV void mat_identity(float (&M)[D * D]) {
#pragma unroll
    for (int i = 0; i < D; ++i)
#pragma unroll
        for (int j = 0; j < D; ++j) M[i * D + j] = (i == j) ? S::one() : S::zero();
}

// Z = X (op) Y
template <class S, int D>
HMM_DEV void mat_mul(const float (&X)[D * D], const float (&Y)[D * D], float (&Z)[D * D]) {
#pragma unroll
    for (int i = 0; i < D; ++i)
#pragma unroll
        for (int j = 0; j < D; ++j) {
            float acc = S::times(X[i * D + 0], Y[0 * D + j]);
#pragma unroll
            for (int k = 1; k < D; ++k) acc = S::mul_add(acc, X[i * D + k], Y[k * D + j]);
            Z[i * D + j] = acc;
        }
}

// r = v (op) M   (row vector times matrix: forward direction)
template <class S, int D>
HMM_DEV void vec_mat(const float (&v)[D], const float (&M)[D * D], float (&r)[D]) {
#pragma unroll
    for (int j = 0; j < D; ++j) {
        float acc = S::times(v[0], M[j]);
#pragma unroll
        for (int i = 1; i < D; ++i) acc = S::mul_add(acc, v[i], M[i * D + j]);
        r[j] = acc;
    }
}

// r = M (op) v   (matrix times column vector: backward direction)
template <class S, int D>
HMM_DEV void mat_vec(const float (&M)[D * D], const float (&v)[D], float (&r)[D]) {
#pragma unroll
    for (int i = 0; i < D; ++i) {
        float acc = S::times(M[i * D], v[0]);
#pragma unroll
        for (int j = 1; j < D; ++j) acc = S::mul_add(acc, M[i * D + j], v[j]);
        r[i] = acc;
    }
}

// =============================================================================================
// Scaled aggregates: an element a_{i:k} of the scans together with its scale.
//
//   SumProd: value(i, j) = m[i][j] * 2^ex[i] * 2^c.  EVERY ROW has its own binary exponent: the
//            rows of a product of potentials are the forward recursions started from each state,
//            and with zero transitions (absorbing or one-way states) they drift apart without
//            bound -- one exponent per matrix would flush the small rows although the carry that
//            multiplies the aggregate may sit on exactly those rows.  A row is stored with its
//            largest entry in [2^(ROW_BIAS-1), 2^ROW_BIAS): far above one, so that entries down to
//            2^-(126+ROW_BIAS) of the row's largest stay normal numbers (a backward potential may
//            weigh them up again by as much), yet low enough that the product of two such rows'
//            entries cannot overflow.  Rows that are entirely zero keep a meaningless exponent; every consumer
//            below ignores them.  c collects the whole bits taken out of the emission factors; it is
//            common to the matrix and only the evidence needs it.
//   MaxPlus: value(i, j) = m[i][j] + c, largest entry of m at 0 (logarithms need no exponents).
//
// All scale arithmetic is exact (integers, and doubles holding integers or sums of floats), so
// log Z / the best log-weight follow from an aggregate of the whole sequence with one logarithm.
template <class S, int D>
struct Agg {
    float m[D * D];
    int ex[D];     // SumProd only
    double c;
};

constexpr int EX_NONE = -(1 << 28);   // "this term does not exist" in exponent comparisons
constexpr int FAST_SPREAD = 32;       // row exponents this close together are applied as plain powers of two
constexpr int UNIFORM_SPREAD = 20;    // rows whose largest entries are this close together share one exponent
constexpr int ROW_BIAS = 44;          // stored rows: largest entry below 2^44 (and above 2^(43 - UNIFORM_SPREAD))
constexpr int SLOW_LIFT = 76;         // general product: a row's largest left factor sits at 2^76
constexpr int WORK_BIAS = 100;        // rows inside a chunk's step loop: room to shrink between two rescalings
constexpr int WORK_ROOM = 64;         // ... by at most this many bits
constexpr int VEC_BIAS = 60;          // forward and backward potentials: largest entry in [2^59, 2^60)
// (2 ROW_BIAS + FAST_SPREAD + 3, ROW_BIAS + SLOW_LIFT + 3, ROW_BIAS + VEC_BIAS + 3 and 2 VEC_BIAS + 3 all stay
// below 127: no product of two stored quantities, summed over at most eight terms, overflows.)

HMM_DEV bool wave_any(bool p) { return __builtin_amdgcn_ballot_w64(p) != 0ull; }

HMM_DEV int max_of_int(int a, int b) { return a > b ? a : b; }
HMM_DEV int min_of_int(int a, int b) { return a < b ? a : b; }

template <class S, int D>
HMM_DEV void agg_identity(Agg<S, D>& P) {
    mat_identity<S, D>(P.m);   // (rows of the neutral element are not biased: any power of two is a valid row scale)
#pragma unroll
    for (int i = 0; i < D; ++i) P.ex[i] = 0;
    P.c = 0.0;
}

template <int D>
HMM_DEV float row_max(const float (&m)[D * D], int i) {
    float mx = m[i * D];
#pragma unroll
    for (int j = 1; j < D; ++j) mx = fmaxf(mx, m[i * D + j]);
    return mx;
}

// Rows back to the bias (SumProd) / largest entry back to 0 (MaxPlus); what is removed goes into the scale.
// SumProd: if the rows' largest entries lie within 2^UNIFORM_SPREAD of one another (decided for the whole
// wavefront) they all take the exponent of the largest, so that rows whose exponents were equal keep equal
// exponents -- the usual case, for which products need no alignment at all.  Otherwise every row takes its own.
template <class S, int D, int BIAS = ROW_BIAS>
HMM_DEV void agg_renorm(Agg<S, D>& P) {
    if constexpr (S::is_max_plus) {
        float mx = max_of(P.m);
        mx = (mx == -INFINITY) ? 0.0f : mx;
#pragma unroll
        for (int e = 0; e < D * D; ++e) P.m[e] -= mx;
        P.c += (double)mx;
    } else {
        int e[D];
#pragma unroll
        for (int i = 0; i < D; ++i) e[i] = __builtin_amdgcn_frexp_expf(row_max<D>(P.m, i)) - BIAS;   // (a zero row just drifts: nobody reads its exponent)
        int hi = e[0], lo = e[0];
#pragma unroll
        for (int i = 1; i < D; ++i) {
            hi = e[i] > hi ? e[i] : hi;
            lo = e[i] < lo ? e[i] : lo;
        }
        if (!wave_any(hi - lo > UNIFORM_SPREAD)) {
#pragma unroll
            for (int i = 0; i < D; ++i) e[i] = hi;
        }
#pragma unroll
        for (int i = 0; i < D; ++i) {
#pragma unroll
            for (int j = 0; j < D; ++j) P.m[i * D + j] = ldexpf(P.m[i * D + j], -e[i]);
            P.ex[i] += e[i];
        }
    }
}

// Z = X (op) Y.  TRACK_C = false leaves Z.c alone (scans whose scale nobody reads).
// SumProd: row i of Z is sum_k X(i,k) 2^ey[k] Y(k,.).  When Y's row exponents lie within FAST_SPREAD of
// each other (decided for the whole wavefront, so the branch is uniform) they are applied to X's columns
// as plain powers of two, lifted by 2^FAST_SPREAD so that no entry of X is flushed by it; the bias of the
// stored rows keeps every term that matters to an entry within 2^-126 of its row's largest a normal
// number.  Otherwise every row of Z takes its own reference exponent, the largest exponent among its
// existing terms, so a row that lives only on Y's small rows keeps its full precision.
// MaxPlus: SHIFT = false leaves the largest entry where the product put it (below zero by at most what the factors'
// entries allow) instead of moving it to zero.
template <class S, int D, bool TRACK_C = true, bool SHIFT = true>
HMM_DEV void agg_mul(const Agg<S, D>& X, const Agg<S, D>& Y, Agg<S, D>& Z) {
    if constexpr (S::is_max_plus) {
        mat_mul<S, D>(X.m, Y.m, Z.m);
        if constexpr (SHIFT) {
            float mx = max_of(Z.m);
            mx = (mx == -INFINITY) ? 0.0f : mx;
#pragma unroll
            for (int e = 0; e < D * D; ++e) Z.m[e] -= mx;
            if constexpr (TRACK_C) Z.c = X.c + Y.c + (double)mx;
        } else {
            if constexpr (TRACK_C) Z.c = X.c + Y.c;
        }
    } else {
        int hi = Y.ex[0], lo = Y.ex[0];
#pragma unroll
        for (int k = 1; k < D; ++k) {
            hi = Y.ex[k] > hi ? Y.ex[k] : hi;
            lo = Y.ex[k] < lo ? Y.ex[k] : lo;
        }
        if (!wave_any(hi != lo)) {
            // all of Y's rows share one exponent: the plain product (entries below D 2^(2 ROW_BIAS))
            mat_mul<S, D>(X.m, Y.m, Z.m);
#pragma unroll
            for (int i = 0; i < D; ++i) Z.ex[i] = X.ex[i] + hi;
        } else if (!wave_any(hi - lo > FAST_SPREAD)) {
            float Xs[D * D];
#pragma unroll
            for (int k = 0; k < D; ++k) {
                const int d = Y.ex[k] - hi + FAST_SPREAD;   // 0 .. FAST_SPREAD: nothing of X is scaled down
#pragma unroll
                for (int i = 0; i < D; ++i) Xs[i * D + k] = ldexpf(X.m[i * D + k], d);
            }
            mat_mul<S, D>(Xs, Y.m, Z.m);   // entries below D 2^(2 ROW_BIAS + FAST_SPREAD)
#pragma unroll
            for (int i = 0; i < D; ++i) Z.ex[i] = X.ex[i] + hi - FAST_SPREAD;
        } else {
            int ey[D];
#pragma unroll
            for (int k = 0; k < D; ++k) ey[k] = (row_max<D>(Y.m, k) > 0.0f) ? Y.ex[k] : EX_NONE;
#pragma unroll
            for (int i = 0; i < D; ++i) {
                int ref = EX_NONE;
#pragma unroll
                for (int k = 0; k < D; ++k) {
                    const float x = X.m[i * D + k];
                    const int e = (x > 0.0f && ey[k] != EX_NONE) ? __builtin_amdgcn_frexp_expf(x) + ey[k] : EX_NONE;
                    ref = e > ref ? e : ref;
                }
                float w[D];   // the row's terms' left factors, the largest in [2^(SLOW_LIFT-1), 2^SLOW_LIFT)
#pragma unroll
                for (int k = 0; k < D; ++k)
                    w[k] = (ey[k] != EX_NONE && ref != EX_NONE)
                               ? ldexpf(X.m[i * D + k], max_of_int(ey[k] - ref + SLOW_LIFT, -400)) : 0.0f;
#pragma unroll
                for (int j = 0; j < D; ++j) {
                    float acc = w[0] * Y.m[j];
#pragma unroll
                    for (int k = 1; k < D; ++k) acc = fmaf(w[k], Y.m[k * D + j], acc);
                    Z.m[i * D + j] = acc;
                }
                Z.ex[i] = (ref != EX_NONE) ? X.ex[i] + ref - SLOW_LIFT : X.ex[i];
            }
        }
        if constexpr (TRACK_C) Z.c = X.c + Y.c;
        agg_renorm<S, D>(Z);
    }
}

// r = v (op) M for a non-negative vector v of any scale (SumProd) / a vector of logarithms (MaxPlus), r brought
// back into range: largest entry in [2^(VEC_BIAS-1), 2^VEC_BIAS) / at 0.  Returns what the result was scaled by relative to
// v * value(M) / 2^c: bits (SumProd) or the offset (MaxPlus), for callers that track the scale.
template <class S, int D>
HMM_DEV double vec_agg(const float (&v)[D], const Agg<S, D>& M, float (&r)[D]) {
    if constexpr (S::is_max_plus) {
        vec_mat<S, D>(v, M.m, r);
        float mx = max_of(r);
        mx = (mx == -INFINITY) ? 0.0f : mx;
#pragma unroll
        for (int j = 0; j < D; ++j) r[j] -= mx;
        return (double)mx;
    } else {
        constexpr int LIFT = 60;   // the largest term's left factor sits at 2^60: room below for the others
        {
            int hi = M.ex[0], lo = M.ex[0];
#pragma unroll
            for (int i = 1; i < D; ++i) {
                hi = M.ex[i] > hi ? M.ex[i] : hi;
                lo = M.ex[i] < lo ? M.ex[i] : lo;
            }
            if (!wave_any(hi != lo)) {
                // all rows share one exponent: the plain product, brought to a largest entry near 2^VEC_BIAS
                // (v is a potential of at most 2^VEC_BIAS: entries below D 2^(VEC_BIAS + ROW_BIAS))
                vec_mat<S, D>(v, M.m, r);
                const int ex = __builtin_amdgcn_frexp_expf(max_of(r)) - VEC_BIAS;
#pragma unroll
                for (int j = 0; j < D; ++j) r[j] = ldexpf(r[j], -ex);
                return (double)hi + (double)ex;
            }
        }
        int e[D], ref = EX_NONE;
#pragma unroll
        for (int i = 0; i < D; ++i) {
            e[i] = (v[i] > 0.0f && row_max<D>(M.m, i) > 0.0f) ? __builtin_amdgcn_frexp_expf(v[i]) + M.ex[i] : EX_NONE;
            ref = e[i] > ref ? e[i] : ref;
        }
        float w[D];
#pragma unroll
        for (int i = 0; i < D; ++i)
            w[i] = (e[i] != EX_NONE) ? ldexpf(v[i], max_of_int(M.ex[i] - ref + LIFT, -400)) : 0.0f;
#pragma unroll
        for (int j = 0; j < D; ++j) {
            float acc = w[0] * M.m[j];
#pragma unroll
            for (int i = 1; i < D; ++i) acc = fmaf(w[i], M.m[i * D + j], acc);
            r[j] = acc;   // below D 2^(LIFT + ROW_BIAS)
        }
        const int ex = __builtin_amdgcn_frexp_expf(max_of(r)) - VEC_BIAS;
#pragma unroll
        for (int j = 0; j < D; ++j) r[j] = ldexpf(r[j], -ex);
        return (ref != EX_NONE) ? (double)(ref - LIFT) + (double)ex : 0.0;
    }
}

// The raw form of M (op) v: s[i] = sum_j m[i][j] v[j] with the row exponents left beside it (es[i]; EX_NONE
// where s[i] is zero), for callers that choose the common scale themselves.  SumProd only.
template <int D>
HMM_DEV void agg_vec_raw(const Agg<SumProd, D>& M, const float (&v)[D], float (&s)[D], int (&es)[D]) {
    mat_vec<SumProd, D>(M.m, v, s);
#pragma unroll
    for (int i = 0; i < D; ++i) es[i] = (s[i] > 0.0f) ? M.ex[i] : EX_NONE;
}

// r = M (op) v, largest entry in [2^(VEC_BIAS-1), 2^VEC_BIAS) (SumProd) / at 0 (MaxPlus); returns the scale taken out.
template <class S, int D>
HMM_DEV double agg_vec(const Agg<S, D>& M, const float (&v)[D], float (&r)[D]) {
    if constexpr (S::is_max_plus) {
        mat_vec<S, D>(M.m, v, r);
        float mx = max_of(r);
        mx = (mx == -INFINITY) ? 0.0f : mx;
#pragma unroll
        for (int i = 0; i < D; ++i) r[i] -= mx;
        return (double)mx;
    } else {
        float s[D];
        {
            int hi = M.ex[0], lo = M.ex[0];
#pragma unroll
            for (int i = 1; i < D; ++i) {
                hi = M.ex[i] > hi ? M.ex[i] : hi;
                lo = M.ex[i] < lo ? M.ex[i] : lo;
            }
            if (!wave_any(hi != lo)) {
                mat_vec<S, D>(M.m, v, s);
                const int ex = __builtin_amdgcn_frexp_expf(max_of(s)) - VEC_BIAS;
#pragma unroll
                for (int i = 0; i < D; ++i) r[i] = ldexpf(s[i], -ex);
                return (double)hi + (double)ex;
            }
        }
        int es[D], ref = EX_NONE;
        agg_vec_raw<D>(M, v, s, es);
#pragma unroll
        for (int i = 0; i < D; ++i) {
            es[i] = (es[i] != EX_NONE) ? __builtin_amdgcn_frexp_expf(s[i]) + es[i] : EX_NONE;
            ref = es[i] > ref ? es[i] : ref;
        }
#pragma unroll
        for (int i = 0; i < D; ++i)
            r[i] = (es[i] != EX_NONE) ? ldexpf(s[i], max_of_int(M.ex[i] - ref + VEC_BIAS, -400)) : 0.0f;
        return (ref != EX_NONE) ? (double)(ref - VEC_BIAS) : 0.0;
    }
}

// =============================================================================================
// Uniform mode (SumProd).  In well-conditioned models the rows of every aggregate stay within
// 2^UNIFORM_SPREAD of one another and all share one exponent; the operations above then always take
// their first branch.  The *_u operations below are those first branches on their own: straight-line
// code that assumes its arguments' row exponents are all equal (it reads ex[0]), produces results
// with equal row exponents, and reports in `bad` whenever the general operation would have left its
// first branch (the test is slightly stricter, never laxer).  A caller runs a whole phase in uniform
// mode and, if any lane of the wavefront reported `bad`, runs the phase again with the general
// operations: what comes out is what the general operations alone produce (the same bits for every entry
// within 2^-126 of its row's largest; scalings are exact powers of two), but the usual case has no branch
// per operation.
template <int D>
HMM_DEV bool agg_is_uniform(const Agg<SumProd, D>& P) {
    bool u = true;
#pragma unroll
    for (int i = 1; i < D; ++i) u = u && (P.ex[i] == P.ex[0]);
    return u;
}

template <int D, int BIAS = ROW_BIAS>
HMM_DEV void agg_renorm_u(Agg<SumProd, D>& P, bool& bad) {
    float hi = row_max<D>(P.m, 0), lo = hi;
#pragma unroll
    for (int i = 1; i < D; ++i) {
        const float r = row_max<D>(P.m, i);
        hi = fmaxf(hi, r);
        lo = fminf(lo, r);
    }
    // rows more than 2^UNIFORM_SPREAD apart (a zero row beside a non-zero one included) need their own exponents
    bad = bad || (lo < hi * (1.0f / (float)(1 << UNIFORM_SPREAD)));
    const int e = __builtin_amdgcn_frexp_expf(hi) - BIAS;
#pragma unroll
    for (int k = 0; k < D * D; ++k) P.m[k] = ldexpf(P.m[k], -e);
    const int ne = P.ex[0] + e;
#pragma unroll
    for (int i = 0; i < D; ++i) P.ex[i] = ne;
}

template <int D, bool TRACK_C = true, int BIAS = ROW_BIAS>
HMM_DEV void agg_mul_u(const Agg<SumProd, D>& X, const Agg<SumProd, D>& Y, Agg<SumProd, D>& Z, bool& bad) {
    mat_mul<SumProd, D>(X.m, Y.m, Z.m);
    const int e = X.ex[0] + Y.ex[0];
#pragma unroll
    for (int i = 0; i < D; ++i) Z.ex[i] = e;
    if constexpr (TRACK_C) Z.c = X.c + Y.c;
    if constexpr (BIAS >= 0) agg_renorm_u<D, BIAS>(Z, bad);
}

template <int D>
HMM_DEV double vec_agg_u(const float (&v)[D], const Agg<SumProd, D>& M, float (&r)[D]) {
    vec_mat<SumProd, D>(v, M.m, r);
    const int ex = __builtin_amdgcn_frexp_expf(max_of(r)) - VEC_BIAS;
#pragma unroll
    for (int j = 0; j < D; ++j) r[j] = ldexpf(r[j], -ex);
    return (double)M.ex[0] + (double)ex;
}

template <int D>
HMM_DEV double agg_vec_u(const Agg<SumProd, D>& M, const float (&v)[D], float (&r)[D]) {
    float s[D];
    mat_vec<SumProd, D>(M.m, v, s);
    const int ex = __builtin_amdgcn_frexp_expf(max_of(s)) - VEC_BIAS;
#pragma unroll
    for (int i = 0; i < D; ++i) r[i] = ldexpf(s[i], -ex);
    return (double)M.ex[0] + (double)ex;
}

// One spelling for both modes: U selects the uniform operation (SumProd only; MaxPlus has no branches to
// avoid and always runs the general one).
template <bool U, class S, int D, bool TRACK_C>
HMM_DEV void agg_mul_m(const Agg<S, D>& X, const Agg<S, D>& Y, Agg<S, D>& Z, bool& bad) {
    if constexpr (U && !S::is_max_plus) agg_mul_u<D, TRACK_C>(X, Y, Z, bad);
    else agg_mul<S, D, TRACK_C>(X, Y, Z);
}
template <bool U, class S, int D, int BIAS>
HMM_DEV void agg_renorm_m(Agg<S, D>& P, bool& bad) {
    if constexpr (U && !S::is_max_plus) agg_renorm_u<D, BIAS>(P, bad);
    else agg_renorm<S, D, BIAS>(P);
}
template <bool U, class S, int D>
HMM_DEV double vec_agg_m(const float (&v)[D], const Agg<S, D>& M, float (&r)[D]) {
    if constexpr (U && !S::is_max_plus) return vec_agg_u<D>(v, M, r);
    else return vec_agg<S, D>(v, M, r);
}
template <bool U, class S, int D>
HMM_DEV double agg_vec_m(const Agg<S, D>& M, const float (&v)[D], float (&r)[D]) {
    if constexpr (U && !S::is_max_plus) return agg_vec_u<D>(M, v, r);
    else return agg_vec<S, D>(M, v, r);
}

}  // namespace hmm
