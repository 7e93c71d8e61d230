// Device-side building blocks shared by the SemantiCache kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sc {

// Storage tag for bf16 elements (the kernels only ever look at the bits).
struct bf16_t { uint16_t bits; };

constexpr int kWave = 64;

// ------------------------------------------------------------------ bf16 <-> fp32
__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

// round-to-nearest-even; NaN stays NaN
__device__ __forceinline__ uint32_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

// ------------------------------------------------------------------ 8-element row pieces
// Every kernel gives a lane 8 consecutive elements of a row (16 B of bf16, 32 B of fp32), so a row
// of d elements is covered by d/8 neighbouring lanes with fully coalesced 16-byte accesses.
__device__ __forceinline__ void load8(const bf16_t *p, float (&x)[8]) {
    const uint4 v = *reinterpret_cast<const uint4 *>(p);
    x[0] = bf16_lo(v.x); x[1] = bf16_hi(v.x); x[2] = bf16_lo(v.y); x[3] = bf16_hi(v.y);
    x[4] = bf16_lo(v.z); x[5] = bf16_hi(v.z); x[6] = bf16_lo(v.w); x[7] = bf16_hi(v.w);
}
__device__ __forceinline__ void load8(const float *p, float (&x)[8]) {
    const float4 a = *reinterpret_cast<const float4 *>(p);
    const float4 b = *reinterpret_cast<const float4 *>(p + 4);
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
}
// two fp32 -> packed bf16 pair, round-to-nearest-even (v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    typedef __bf16 bf16x2_v __attribute__((ext_vector_type(2)));
    typedef float f32x2_v __attribute__((ext_vector_type(2)));
    const f32x2_v f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_v));
}
__device__ __forceinline__ void store8(bf16_t *p, const float (&x)[8]) {
    uint4 v;
    v.x = pack_bf16x2(x[0], x[1]);
    v.y = pack_bf16x2(x[2], x[3]);
    v.z = pack_bf16x2(x[4], x[5]);
    v.w = pack_bf16x2(x[6], x[7]);
    *reinterpret_cast<uint4 *>(p) = v;
}
__device__ __forceinline__ void store8(float *p, const float (&x)[8]) {
    *reinterpret_cast<float4 *>(p) = make_float4(x[0], x[1], x[2], x[3]);
    *reinterpret_cast<float4 *>(p + 4) = make_float4(x[4], x[5], x[6], x[7]);
}
__device__ __forceinline__ double load1_f64(const bf16_t *p) { return (double)__uint_as_float((uint32_t)p->bits << 16); }
__device__ __forceinline__ double load1_f64(const float *p) { return (double)*p; }

// ------------------------------------------------------------------ bf16 pairs of two rows -> MFMA operand words
// A lane that holds the same two columns of two rows (a, b: one dword each) gets the words
// (column 0 of a, column 0 of b) and (column 1 of a, column 1 of b): v_perm_b32, one instruction each.
__device__ __forceinline__ uint32_t pack_lo(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x05040100u); }
__device__ __forceinline__ uint32_t pack_hi(uint32_t a, uint32_t b) { return __builtin_amdgcn_perm(b, a, 0x07060302u); }
__device__ __forceinline__ uint32_t dword_of(const uint4 &v, int j) {   // j compile-time after unrolling
    return j == 0 ? v.x : (j == 1 ? v.y : (j == 2 ? v.z : v.w));
}

// ------------------------------------------------------------------ cross-lane moves (DPP)
// Symmetric lane pairings inside a row of 16 lanes; all lanes of the wave must be active.
constexpr int kDppQuadXor1 = 0xB1;      // quad_perm [1,0,3,2]
constexpr int kDppQuadXor2 = 0x4E;      // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141;   // lane i <-> 7 - i inside each 8 lanes
constexpr int kDppMirror = 0x140;       // lane i <-> 15 - i inside each 16 lanes
constexpr int kDppRor4 = 0x124;         // rotate by 4 inside each 16 lanes
constexpr int kDppRor8 = 0x128;         // rotate by 8 inside each 16 lanes

template <int CTRL>
__device__ __forceinline__ float dpp(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true));
}
template <int CTRL>
__device__ __forceinline__ int dpp(int x) {
    return __builtin_amdgcn_update_dpp(0, x, CTRL, 0xf, 0xf, true);
}

// Sum over the LPR (8 or 16) neighbouring lanes that share a row; every lane gets the total.
template <int LPR>
__device__ __forceinline__ float row_allreduce_sum(float x) {
    x += dpp<kDppQuadXor1>(x);
    x += dpp<kDppQuadXor2>(x);
    x += dpp<kDppHalfMirror>(x);
    if (LPR == 16) x += dpp<kDppMirror>(x);
    return x;
}
template <int LPR>
__device__ __forceinline__ float row_allreduce_max(float x) {
    x = fmaxf(x, dpp<kDppQuadXor1>(x));
    x = fmaxf(x, dpp<kDppQuadXor2>(x));
    x = fmaxf(x, dpp<kDppHalfMirror>(x));
    if (LPR == 16) x = fmaxf(x, dpp<kDppMirror>(x));
    return x;
}

// "Transposed" reduction: every lane holds LPR partial sums p[0..LPR); lane c of each LPR-lane
// group ends up with the group-wide total of p[c].  Costs ~2*LPR adds instead of LPR*log2(LPR).
template <int LPR>
__device__ __forceinline__ float row_transpose_reduce(const float (&p)[LPR], int c) {
    float q8[8];
    if constexpr (LPR == 16) {
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const float lo = p[t] + dpp<kDppMirror>(p[t]);
            const float hi = p[(t + 8) % LPR] + dpp<kDppMirror>(p[(t + 8) % LPR]);
            q8[t] = (c & 8) ? hi : lo;
        }
    } else {
#pragma unroll
        for (int t = 0; t < 8; ++t) q8[t] = p[t];
    }
    float q4[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const float lo = q8[t] + dpp<kDppHalfMirror>(q8[t]);
        const float hi = q8[t + 4] + dpp<kDppHalfMirror>(q8[t + 4]);
        q4[t] = (c & 4) ? hi : lo;
    }
    float q2[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const float lo = q4[t] + dpp<kDppQuadXor2>(q4[t]);
        const float hi = q4[t + 2] + dpp<kDppQuadXor2>(q4[t + 2]);
        q2[t] = (c & 2) ? hi : lo;
    }
    const float lo = q2[0] + dpp<kDppQuadXor1>(q2[0]);
    const float hi = q2[1] + dpp<kDppQuadXor1>(q2[1]);
    return (c & 1) ? hi : lo;
}

// Reductions over the four 16-lane rows of a wave (same position inside the row), every lane gets the
// result.  v_permlane16_swap / v_permlane32_swap exchange odd and even rows (halves) of two registers
// in one VALU operation: swapping x with itself yields {even|even, odd|odd}, whose sum is the pair sum.
__device__ __forceinline__ float rows_allreduce_sum(float x) {
    auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = __uint_as_float(r[0]) + __uint_as_float(r[1]);
    r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float rows_allreduce_max(float x) {
    auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
    r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// Arbitrary lane gather through the LDS crossbar (no LDS memory is touched).
__device__ __forceinline__ float lane_gather(float x, int src_lane) {
    return __int_as_float(__builtin_amdgcn_ds_bpermute(src_lane << 2, __float_as_int(x)));
}
__device__ __forceinline__ int lane_gather(int x, int src_lane) {
    return __builtin_amdgcn_ds_bpermute(src_lane << 2, x);
}

__device__ __forceinline__ uint64_t ballot64(bool pred) { return __ballot(pred); }
// 16 bytes that are read (written) once by this launch and not again soon: the non-temporal hint keeps
// them from displacing lines that are (provisional rows, partials, offsets)
typedef unsigned int stream_u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load16_stream(const void *p) {
    const stream_u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const stream_u32x4_t *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store16_stream(void *p, const uint4 &v) {
    const stream_u32x4_t t = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(t, reinterpret_cast<stream_u32x4_t *>(p));
}
__device__ __forceinline__ int first_bit(uint64_t m) { return __ffsll((unsigned long long)m) - 1; }

// fp64 sum over the wave, every lane gets the total: DPP moves inside the rows of 16 lanes and row
// swaps across them, on the two halves of the value (a __shfl_xor butterfly on doubles is twelve trips
// through the LDS crossbar)
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double x) {
    const unsigned long long u = __builtin_bit_cast(unsigned long long, x);
    const unsigned lo = (unsigned)__builtin_amdgcn_update_dpp(0, (int)(unsigned)u, CTRL, 0xf, 0xf, true);
    const unsigned hi = (unsigned)__builtin_amdgcn_update_dpp(0, (int)(unsigned)(u >> 32), CTRL, 0xf, 0xf, true);
    return __builtin_bit_cast(double, ((unsigned long long)hi << 32) | lo);
}
__device__ __forceinline__ double wave_allreduce_sum(double x) {
    x += dpp_f64<kDppQuadXor1>(x);
    x += dpp_f64<kDppQuadXor2>(x);
    x += dpp_f64<kDppHalfMirror>(x);
    x += dpp_f64<kDppMirror>(x);
    {
        const unsigned long long u = __builtin_bit_cast(unsigned long long, x);
        const auto l = __builtin_amdgcn_permlane16_swap((unsigned)u, (unsigned)u, false, false);
        const auto h = __builtin_amdgcn_permlane16_swap((unsigned)(u >> 32), (unsigned)(u >> 32), false, false);
        x = __builtin_bit_cast(double, ((unsigned long long)h[0] << 32) | l[0]) +
            __builtin_bit_cast(double, ((unsigned long long)h[1] << 32) | l[1]);
    }
    {
        const unsigned long long u = __builtin_bit_cast(unsigned long long, x);
        const auto l = __builtin_amdgcn_permlane32_swap((unsigned)u, (unsigned)u, false, false);
        const auto h = __builtin_amdgcn_permlane32_swap((unsigned)(u >> 32), (unsigned)(u >> 32), false, false);
        x = __builtin_bit_cast(double, ((unsigned long long)h[0] << 32) | l[0]) +
            __builtin_bit_cast(double, ((unsigned long long)h[1] << 32) | l[1]);
    }
    return x;
}

}  // namespace sc
