// Register-resident D x D element algebra for the two associative operators of the paper:
//   SumProd : Definition 3, (a (x) b)(x_i,x_k) = sum_{x_j} a(x_i,x_j) b(x_j,x_k)
//   MaxPlus : Definition 5 on logarithms, (a v b)(x_i,x_k) = max_{x_j} [a(x_i,x_j) + b(x_j,x_k)]
// Matrices are row-major float[D*D] with compile-time indices only, so they live in VGPRs.
//
// Neither operator carries a scale: a sum-product element is kept within float range by
// multiplying with an exact power of two, a max-plus element by subtracting its largest entry.
// The scale is never needed downstream -- marginals and arg-maxima are scale-free, and the
// log-likelihood / log-probability are accumulated from chunk-local normalisers instead.
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

}  // namespace hmm
