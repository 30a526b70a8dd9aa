// Device-side helpers shared by the gfx950 kernels of this library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ds3 {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float as_f32(unsigned int u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ unsigned int as_u32(float f) { return __builtin_bit_cast(unsigned int, f); }

// BF16 -> FP32 widening is a 16-bit shift; a 32-bit word holds two elements,
// the lower-addressed one in the low half.
__device__ __forceinline__ float bf16_lo(unsigned int w) { return as_f32(w << 16); }
__device__ __forceinline__ float bf16_hi(unsigned int w) { return as_f32(w & 0xffff0000u); }

// FP32 -> BF16, round to nearest even (finite inputs).
__device__ __forceinline__ unsigned int f32_to_bf16_rne(float f) {
    unsigned int u = as_u32(f);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ unsigned int pack_bf16x2(float lo, float hi) {
    return f32_to_bf16_rne(lo) | (f32_to_bf16_rne(hi) << 16);
}

// Max over the 16 lanes of a DPP row; every lane of the row gets the result.
// Operates on the bit patterns of non-negative finite floats, for which the
// unsigned integer order equals the floating-point order (no NaN handling,
// no canonicalisation instructions).
template <int CTRL>
__device__ __forceinline__ unsigned int dpp_u32(unsigned int v) {
    return (unsigned int)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, 0xF, 0xF, true);
}
__device__ __forceinline__ unsigned int umax(unsigned int a, unsigned int b) { return a > b ? a : b; }
__device__ __forceinline__ unsigned int row16_max_bits(unsigned int v) {
    v = umax(v, dpp_u32<0xB1>(v));   // quad_perm [1,0,3,2]
    v = umax(v, dpp_u32<0x4E>(v));   // quad_perm [2,3,0,1]
    v = umax(v, dpp_u32<0x141>(v));  // row_half_mirror: quads 0<->1, 2<->3
    v = umax(v, dpp_u32<0x140>(v));  // row_mirror: halves
    return v;
}

// The two per-group factors of the quantisation contract: the stored scale
// s = amax / 448 and the multiplier r = 448 / amax, both correctly rounded
// FP32 divisions; an all-zero group gives s = 1, r = 0.
//
// With `pow2` set the scale is instead the smallest power of two not below
// amax / 448 (the "round scaled" factors of Section 3.3.3) and r its exact
// reciprocal.  448 = 1.75 * 2^8, so for amax = m * 2^E, 1 <= m < 2, the
// exponent is E - 8 when m <= 1.75 and E - 7 otherwise; both factors are built
// from exponent fields directly.
struct GroupScale { float s, r; };
__device__ __forceinline__ GroupScale group_scale(float amax, int pow2) {
    GroupScale g;
    if (amax == 0.0f) { g.s = 1.0f; g.r = 0.0f; }
    else if (pow2) {
        const unsigned int bits = as_u32(amax);
        const unsigned int e = (bits >> 23) - 8u + ((bits & 0x7fffffu) > 0x600000u ? 1u : 0u);
        g.s = as_f32(e << 23);
        g.r = as_f32((254u - e) << 23);
    } else { g.s = amax / 448.0f; g.r = 448.0f / amax; }
    return g;
}

// E5M6 (12-bit cache format: sign, 5 exponent bits with bias 15, 6 mantissa bits; the
// upper 12 bits of IEEE binary16, exponent field 31 never produced): round to nearest
// even from FP32, saturating at 65024.  Normal results round the FP32 significand in
// place; results below 2^-14 are rounded by an FP32 addition whose ulp is the subnormal
// quantum 2^-20.
__device__ __forceinline__ unsigned int e5m6_rne(float y) {
    unsigned int u = as_u32(y);
    const unsigned int sign = (u >> 20) & 0x800u;
    u &= 0x7fffffffu;
    unsigned int code;
    if (u >= 0x38800000u) {                       // |y| >= 2^-14
        u += 0xffffu + ((u >> 17) & 1u);
        code = (u >> 17) - (112u << 6);
        code = code < 0x7bfu ? code : 0x7bfu;
    } else {
        code = as_u32(as_f32(u) + 8.0f) - as_u32(8.0f);
    }
    return sign | code;
}
__device__ __forceinline__ float e5m6_decode(unsigned int c) {
    const unsigned int mag = c & 0x7ffu;
    // exponent field 0: mantissa * 2^-20 (exact in FP32); otherwise re-bias into FP32
    const float v = mag < 64u ? (float)mag * 9.5367431640625e-07f : as_f32((mag << 17) + (112u << 23));
    return (c & 0x800u) ? -v : v;
}
// The smallest power of two >= amax / 65024 and its reciprocal (65024 = (2 - 2^-6) * 2^15).
__device__ __forceinline__ GroupScale group_scale_e5m6(float amax) {
    GroupScale g;
    if (amax == 0.0f) { g.s = 1.0f; g.r = 0.0f; return g; }
    const unsigned int bits = as_u32(amax);
    const unsigned int e = (bits >> 23) - 15u + ((bits & 0x7fffffu) > 0x7e0000u ? 1u : 0u);
    g.s = as_f32(e << 23);
    g.r = as_f32((254u - e) << 23);
    return g;
}

// silu(g) * u in FP32 with the hardware reciprocal (1 ulp) instead of an IEEE
// division: the result is rounded to BF16 (8 significant bits) by every caller,
// and all callers share this one expression so that they agree bit for bit.
__device__ __forceinline__ float silu_mul(float g, float u) {
    return g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)) * u;
}

// Four FP32 values -> four E4M3 codes in one 32-bit word (lowest address in
// the low byte); the hardware conversion rounds to nearest even.
__device__ __forceinline__ unsigned int cvt4_e4m3(float a, float b, float c, float d) {
    int w = __builtin_amdgcn_cvt_pk_fp8_f32(a, b, 0, false);
    w = __builtin_amdgcn_cvt_pk_fp8_f32(c, d, w, true);
    return (unsigned int)w;
}

}  // namespace ds3
