// Device-side NVFP4 helpers for gfx950: E4M3 block-scale encode/decode, E2M1 element
// encode, one-block quantization.  Formats per Appendix A / Table "formats" of the paper:
// E2M1 bias 1 max 6, E4M3 bias 7 max 448 (finite flavour), 16 elements per block.
//
// Every function spells out its fp32 operations one by one; this translation unit is
// compiled with -ffp-contract=off and correctly rounded division so that the sequence
//   u = amax * ginv;  sbyte = E4M3(u);  s = E4M3value * s_T;  inv = 1 / s;  w = |v| * inv
// rounds exactly once per step (Section 3.1 eq. (1) evaluated in fp32).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace arcq {

// E4M3 byte (0x00..0x7E) for u, saturating at 448.  up == false: the nearest value, ties to even
// mantissa; up == true: the smallest value not below u (the scale is never rounded down, which is
// what the error analysis of Section 3.4 assumes: alpha >= 1).  `up` is uniform over the launch.
// Precondition: u >= 0 and not NaN.
__device__ __forceinline__ uint32_t e4m3_encode_sat(float u, bool up = false) {
    if (!(u < 448.0f)) return 0x7Eu;
    if (u >= 0.015625f) {                       // normal range, >= 2^-6
        uint32_t bits = __float_as_uint(u);
        // keep 3 mantissa bits: add half an ulp minus one plus the kept lsb (nearest even), or a whole
        // ulp minus one (up), then truncate
        bits += up ? 0xFFFFFu : 0x7FFFFu + ((bits >> 20) & 1u);
        return (bits >> 20) - (120u << 3);      // rebias exponent 127 -> 7
    }
    // subnormal range: multiples of 2^-9; the product is exact, rint is nearest-even;
    // a result of 8 is the byte of the smallest normal, 2^-6
    const float t = u * 512.0f;
    return (uint32_t)(up ? __builtin_ceilf(t) : __builtin_rintf(t));
}

// Value of an E4M3 byte in 0x00..0x7E as fp32 (exact).
__device__ __forceinline__ float e4m3_decode(uint32_t b) {
    float sub = (float)b * 0x1p-9f;                               // exponent field 0
    float nor = __uint_as_float((b << 20) + (120u << 23));        // exponent field e -> e + 120
    return b < 8u ? sub : nor;
}

// Quantize one block of 16 fp32 values.  Outputs the scale byte, the effective scale
// s = E4M3value * s_T, and the 16 codes packed low-nibble-first into lo (elements 0..7)
// and hi (elements 8..15).
//
// The element rounding uses v_cvt_scalef32_pk_fp4_f32 with scale 1.0: two fp32 -> two E2M1
// codes in one byte (first operand in the low nibble), round-to-nearest-even on the E2M1
// grid, saturating at +-6, sign bit kept for zeros.  The signed quotient v * inv is fed
// directly: rounding is symmetric, so this equals sign | round(|v| * inv).
__device__ __forceinline__ void quantize_block16(const float (&v)[16], float s_T, float ginv,
                                                 uint32_t& sbyte, float& s,
                                                 uint32_t& lo, uint32_t& hi, bool scale_up = false) {
    float amax = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) amax = fmaxf(amax, fabsf(v[i]));
    float u = amax * ginv;
    sbyte = e4m3_encode_sat(u, scale_up);
    s = e4m3_decode(sbyte) * s_T;
    float inv = (s != 0.0f) ? 1.0f / s : 0.0f;
    lo = 0u;
    hi = 0u;
    lo = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(lo, v[0] * inv, v[1] * inv, 1.0f, 0);
    lo = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(lo, v[2] * inv, v[3] * inv, 1.0f, 1);
    lo = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(lo, v[4] * inv, v[5] * inv, 1.0f, 2);
    lo = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(lo, v[6] * inv, v[7] * inv, 1.0f, 3);
    hi = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(hi, v[8] * inv, v[9] * inv, 1.0f, 0);
    hi = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(hi, v[10] * inv, v[11] * inv, 1.0f, 1);
    hi = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(hi, v[12] * inv, v[13] * inv, 1.0f, 2);
    hi = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(hi, v[14] * inv, v[15] * inv, 1.0f, 3);
}

typedef float float2v __attribute__((ext_vector_type(2)));

// Residual of one block: r_i = fma(-G[code_i] * sign_i, s, v_i), one rounding
// (Section 3.2 step (2): R_o = X_o - s * Q_{X_o}).  v_cvt_scalef32_pk_f32_fp4 with scale 1.0
// returns the two signed grid values of one byte (low nibble first).
__device__ __forceinline__ void residual_block16(const float (&v)[16], float s,
                                                 uint32_t lo, uint32_t hi, float (&r)[16]) {
    float2v g[8];
    g[0] = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(lo, 1.0f, 0);
    g[1] = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(lo, 1.0f, 1);
    g[2] = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(lo, 1.0f, 2);
    g[3] = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(lo, 1.0f, 3);
    g[4] = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(hi, 1.0f, 0);
    g[5] = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(hi, 1.0f, 1);
    g[6] = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(hi, 1.0f, 2);
    g[7] = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(hi, 1.0f, 3);
#pragma unroll
    for (int i = 0; i < 16; ++i) r[i] = __builtin_fmaf(-g[i >> 1][i & 1], s, v[i]);
}

}  // namespace arcq
