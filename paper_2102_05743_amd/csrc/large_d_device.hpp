// Device-side building blocks shared by the large-state-space kernels (D in {16, 32, 64, 128}).
//
// The sum-product operator of Definition 3 is a dense D x D matrix product; chunk aggregates
// ("block-wise elements", Sec. V-B) are built on the FP32 matrix cores.  A chunk's running
// product P is advanced one time step at a time,
//     P <- P * (A diag(e_t)),      e_t(j) = exp(ll_t(j) - max_j ll_t(j)),
// which is computed transposed, P^T <- diag(e_t) (A^T P^T): the constant A^T is the MFMA's first
// operand (read from LDS) and P^T, which lives in the accumulators, is the second.  An MFMA
// result register of lane l holds rows {row(mt, r, l / TS)} of a column l % TS, and the second
// operand wants one row per lane group, so result registers can be fed straight back as second
// operands if the reduction index k is enumerated in exactly that row order; the first operand
// is stored in LDS in the matching (permuted) order.  No register ever has to change lanes.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hmm {

#define HMM_DEV __device__ __forceinline__

template <int D>
struct LargeCfg {
    static_assert(D == 16 || D == 32 || D == 64 || D == 128, "supported padded sizes");
    static constexpr int NT = 256;                       // lanes per workgroup (4 waves)
    static constexpr int TS = (D >= 64) ? 32 : 16;       // MFMA tile edge: 32x32x2 or 16x16x4
    static constexpr int NG = 64 / TS;                   // lane groups = reduction depth of one MFMA
    static constexpr int NACC = TS * TS / 64;            // result registers per tile
    static constexpr int MT = D / TS;                    // tiles along a column of P^T
    static constexpr int WPC = D / TS;                   // waves per chunk (one TS-column strip each)
    static constexpr int CPW = 4 / WPC;                  // chunks per workgroup
    static constexpr int NS = MT * NACC;                 // MFMAs per result tile (= D * TS / 64)
    static constexpr int ASTR = NS + 4;                  // padded LDS row of first operands
    static constexpr int AT_FLOATS = MT * 64 * ASTR;     // permuted A^T of one chunk
    static constexpr int EB = 16;                        // time steps per emission batch in LDS
    static constexpr int NORM_EVERY = (D >= 32) ? 4 : 8; // steps between power-of-two rescalings
    // vector apply kernels: lane = (column inside the wave, part of the summation range)
    static constexpr int CPWV = (D < 32) ? D : 32;       // columns per wave
    static constexpr int PARTS = 64 / CPWV;              // lane groups splitting the summation
    static constexpr int RPP = D / PARTS;                // summation terms per lane
    static constexpr int VWPC = D / CPWV;                // waves per chunk in the apply kernels
    static constexpr int VCPW = 4 / VWPC;                // chunks per workgroup in the apply kernels
};

// Row of P^T held by result register r of tile mt in lane group g.
template <int D>
HMM_DEV constexpr int mfma_row(int mt, int r, int g) {
    using C = LargeCfg<D>;
    return C::TS * mt + (4 * C::NG) * (r / 4) + 4 * g + (r % 4);
}

typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));

template <int TS> struct AccT;
template <> struct AccT<32> { typedef v16f type; };
template <> struct AccT<16> { typedef v4f type; };

template <int TS>
HMM_DEV typename AccT<TS>::type mfma_step(float a, float b, typename AccT<TS>::type c) {
    if constexpr (TS == 32) return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
    else return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

// Wave-wide reductions with DPP moves (four shifts inside each row of 16 lanes, then the last lane
// of a row broadcast into the following rows); lane 63 ends with the total, which is then
// broadcast through a scalar register.  Lanes without a source at some level take the neutral value.
template <int CTRL, int ROW_MASK>
HMM_DEV float dpp_take(float neutral, float src) {
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(neutral), __float_as_int(src), CTRL, ROW_MASK,
                                                      0xF, false));
}

HMM_DEV float wave_max(float v) {
    v = fmaxf(v, dpp_take<0x111, 0xF>(-INFINITY, v));   // row_shr:1
    v = fmaxf(v, dpp_take<0x112, 0xF>(-INFINITY, v));   // row_shr:2
    v = fmaxf(v, dpp_take<0x114, 0xF>(-INFINITY, v));   // row_shr:4
    v = fmaxf(v, dpp_take<0x118, 0xF>(-INFINITY, v));   // row_shr:8
    v = fmaxf(v, dpp_take<0x142, 0xA>(-INFINITY, v));   // row_bcast:15
    v = fmaxf(v, dpp_take<0x143, 0xC>(-INFINITY, v));   // row_bcast:31
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// The same for values that are known to be non-negative (and not NaN): their bit patterns order like
// unsigned integers, and the integer maximum needs no canonicalisation of its operands, which halves
// the instructions per level.
template <int CTRL, int ROW_MASK>
HMM_DEV unsigned dpp_take_u(unsigned src) {
    return (unsigned)__builtin_amdgcn_update_dpp(0, (int)src, CTRL, ROW_MASK, 0xF, false);
}

HMM_DEV float wave_max_nonneg(float v) {
    unsigned u = __float_as_uint(v);
    u = max(u, dpp_take_u<0x111, 0xF>(u));
    u = max(u, dpp_take_u<0x112, 0xF>(u));
    u = max(u, dpp_take_u<0x114, 0xF>(u));
    u = max(u, dpp_take_u<0x118, 0xF>(u));
    u = max(u, dpp_take_u<0x142, 0xA>(u));
    u = max(u, dpp_take_u<0x143, 0xC>(u));
    return __uint_as_float((unsigned)__builtin_amdgcn_readlane((int)u, 63));
}

HMM_DEV float wave_sum(float v) {
    v += dpp_take<0x111, 0xF>(0.0f, v);
    v += dpp_take<0x112, 0xF>(0.0f, v);
    v += dpp_take<0x114, 0xF>(0.0f, v);
    v += dpp_take<0x118, 0xF>(0.0f, v);
    v += dpp_take<0x142, 0xA>(0.0f, v);
    v += dpp_take<0x143, 0xC>(0.0f, v);
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// value of the lane whose index differs in bit 0 / bit 1 (inside a quad)
HMM_DEV float quad_xor1(float v) { return dpp_take<0xB1, 0xF>(v, v); }   // quad_perm [1,0,3,2]
HMM_DEV float quad_xor2(float v) { return dpp_take<0x4E, 0xF>(v, v); }   // quad_perm [2,3,0,1]
HMM_DEV int quad_xor1(int v) { return __builtin_amdgcn_update_dpp(v, v, 0xB1, 0xF, 0xF, false); }
HMM_DEV int quad_xor2(int v) { return __builtin_amdgcn_update_dpp(v, v, 0x4E, 0xF, 0xF, false); }

// Rotation inside each DPP row of 16 lanes: lane l receives the value of lane (l - R) mod 16 of its row.
template <int R>
HMM_DEV float row_rot(float v) {
    if constexpr (R == 0) return v;
    else return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x120 + R, 0xF, 0xF, true));
}

// Sum / maximum over the 16 lanes of a DPP row, delivered to every lane of the row.
HMM_DEV float row_allsum(float v) {
    v += row_rot<8>(v);
    v += row_rot<4>(v);
    v += row_rot<2>(v);
    v += row_rot<1>(v);
    return v;
}
HMM_DEV float row_allmax(float v) {
    v = fmaxf(v, row_rot<8>(v));
    v = fmaxf(v, row_rot<4>(v));
    v = fmaxf(v, row_rot<2>(v));
    v = fmaxf(v, row_rot<1>(v));
    return v;
}
HMM_DEV float row_allmin(float v) {
    v = fminf(v, row_rot<8>(v));
    v = fminf(v, row_rot<4>(v));
    v = fminf(v, row_rot<2>(v));
    v = fminf(v, row_rot<1>(v));
    return v;
}

// acc[r & 3] += (x rotated by r lanes inside its DPP row) * a[r] for r = 0..15: sixteen multiply-adds
// whose first operand is read through the DPP rotation itself (v_fmac_f32 with a row_ror modifier),
// so no instruction is spent on moving data.  Written out because the compiler emits a separate DPP
// move per term here.  The leading s_nop covers the wait states a DPP read needs after a vector
// instruction wrote its source register (or EXEC); nothing inside the block rewrites x.
HMM_DEV void row_dot16(float x, const float* a, float (&acc)[4]) {
    asm volatile(
        "s_nop 4\n\t"
        "v_fmac_f32 %0, %4, %5\n\t"
        "v_fmac_f32_dpp %1, %4, %6 row_ror:1 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %2, %4, %7 row_ror:2 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %3, %4, %8 row_ror:3 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %0, %4, %9 row_ror:4 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %1, %4, %10 row_ror:5 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %2, %4, %11 row_ror:6 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %3, %4, %12 row_ror:7 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %0, %4, %13 row_ror:8 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %1, %4, %14 row_ror:9 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %2, %4, %15 row_ror:10 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %3, %4, %16 row_ror:11 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %0, %4, %17 row_ror:12 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %1, %4, %18 row_ror:13 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %2, %4, %19 row_ror:14 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %3, %4, %20 row_ror:15 row_mask:0xf bank_mask:0xf"
        : "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3])
        : "v"(x), "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3]), "v"(a[4]), "v"(a[5]), "v"(a[6]), "v"(a[7]), "v"(a[8]),
          "v"(a[9]), "v"(a[10]), "v"(a[11]), "v"(a[12]), "v"(a[13]), "v"(a[14]), "v"(a[15]));
}

// The same starting the four accumulators (plain products for r = 0..3), so that they need no zeroing.
// Outputs are early-clobber: they are written while inputs are still to be read.
HMM_DEV void row_dot16_first(float x, const float* a, float (&acc)[4]) {
    asm volatile(
        "s_nop 4\n\t"
        "v_mul_f32 %0, %4, %5\n\t"
        "v_mul_f32_dpp %1, %4, %6 row_ror:1 row_mask:0xf bank_mask:0xf\n\t"
        "v_mul_f32_dpp %2, %4, %7 row_ror:2 row_mask:0xf bank_mask:0xf\n\t"
        "v_mul_f32_dpp %3, %4, %8 row_ror:3 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %0, %4, %9 row_ror:4 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %1, %4, %10 row_ror:5 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %2, %4, %11 row_ror:6 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %3, %4, %12 row_ror:7 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %0, %4, %13 row_ror:8 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %1, %4, %14 row_ror:9 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %2, %4, %15 row_ror:10 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %3, %4, %16 row_ror:11 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %0, %4, %17 row_ror:12 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %1, %4, %18 row_ror:13 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %2, %4, %19 row_ror:14 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %3, %4, %20 row_ror:15 row_mask:0xf bank_mask:0xf"
        : "=&v"(acc[0]), "=&v"(acc[1]), "=&v"(acc[2]), "=&v"(acc[3])
        : "v"(x), "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3]), "v"(a[4]), "v"(a[5]), "v"(a[6]), "v"(a[7]), "v"(a[8]),
          "v"(a[9]), "v"(a[10]), "v"(a[11]), "v"(a[12]), "v"(a[13]), "v"(a[14]), "v"(a[15]));
}

// acc[r] += (x rotated by r lanes inside its DPP row) * w for r = 0..15: the sixteen entries of an outer
// product that a lane owns when a DPP row of lanes holds one vector (entry (l - r) mod 16 of x against
// the lane's own w).  Same conventions as row_dot16.
HMM_DEV void row_outer16(float x, float w, float (&acc)[16]) {
    asm volatile(
        "s_nop 4\n\t"
        "v_fmac_f32 %0, %16, %17\n\t"
        "v_fmac_f32_dpp %1, %16, %17 row_ror:1 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %2, %16, %17 row_ror:2 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %3, %16, %17 row_ror:3 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %4, %16, %17 row_ror:4 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %5, %16, %17 row_ror:5 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %6, %16, %17 row_ror:6 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %7, %16, %17 row_ror:7 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %8, %16, %17 row_ror:8 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %9, %16, %17 row_ror:9 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %10, %16, %17 row_ror:10 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %11, %16, %17 row_ror:11 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %12, %16, %17 row_ror:12 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %13, %16, %17 row_ror:13 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %14, %16, %17 row_ror:14 row_mask:0xf bank_mask:0xf\n\t"
        "v_fmac_f32_dpp %15, %16, %17 row_ror:15 row_mask:0xf bank_mask:0xf"
        : "+v"(acc[0]), "+v"(acc[1]), "+v"(acc[2]), "+v"(acc[3]), "+v"(acc[4]), "+v"(acc[5]), "+v"(acc[6]), "+v"(acc[7]),
          "+v"(acc[8]), "+v"(acc[9]), "+v"(acc[10]), "+v"(acc[11]), "+v"(acc[12]), "+v"(acc[13]), "+v"(acc[14]),
          "+v"(acc[15])
        : "v"(x), "v"(w));
}

// acc[qd] = terms of (h times the constant matrix held as a[(qs, qd, r)]): a holds, for source block qs, target
// block qd and rotation r, the matrix entry that pairs component 16 qs + (l - r) mod 16 with component 16 qd + l.
template <int NQ>
HMM_DEV void row_matvec_terms(const float (&h)[NQ], const float (&a)[NQ * NQ * 16], float (&acc)[NQ][4]) {
#pragma unroll
    for (int qd = 0; qd < NQ; ++qd) row_dot16_first(h[0], &a[qd * 16], acc[qd]);
#pragma unroll
    for (int qs = 1; qs < NQ; ++qs)
#pragma unroll
        for (int qd = 0; qd < NQ; ++qd) row_dot16(h[qs], &a[(qs * NQ + qd) * 16], acc[qd]);
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every outstanding
// global load and store of the wave (its fence covers global memory), which puts a full memory
// round trip on the critical path of loops that store a result or prefetch an input per step.
HMM_DEV void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Ordering point for LDS traffic inside ONE wave: a wave's LDS instructions execute in order, so a
// write followed by a read of another lane's slot needs no wait, only that the compiler keeps the
// order and re-reads LDS afterwards.  (A wavefront-scope fence would do that too, but it also waits
// for every outstanding global load and store, which serialises loops that prefetch.)
HMM_DEV void wave_lds_sync() { __builtin_amdgcn_wave_barrier(); }

// Wait for the wave's outstanding global loads and mark `v` as produced here, so that later waits
// on loop-carried uses of it do not drain loads issued in between.
HMM_DEV void settle_loaded(float& v) { asm volatile("s_waitcnt vmcnt(0)\n\tv_mov_b32 %0, %0" : "+v"(v)::"memory"); }

struct ChunkCoord {
    int seq;        // sequence
    int cidx;       // chunk index inside the sequence
    long long t0;   // first time step of the chunk inside the sequence
    int nsteps;     // valid steps (0 if the chunk id is out of range)
};

HMM_DEV ChunkCoord chunk_coord(long long chunk, long long nchunks, int cps, long long T, int Lc) {
    ChunkCoord c;
    if (chunk >= nchunks) { c.seq = 0; c.cidx = 0; c.t0 = 0; c.nsteps = 0; return c; }
    c.seq = (int)(chunk / cps);
    c.cidx = (int)(chunk - (long long)c.seq * cps);
    c.t0 = (long long)c.cidx * Lc;
    const long long rem = T - c.t0;
    c.nsteps = rem < Lc ? (int)rem : Lc;
    return c;
}

}  // namespace hmm
