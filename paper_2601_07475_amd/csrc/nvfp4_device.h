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

// E4M3 byte (0x00..0x7E) nearest to u, ties to even mantissa, saturating at 448.
// Precondition: u >= 0 and not NaN.
__device__ __forceinline__ uint32_t e4m3_encode_sat(float u) {
    if (!(u < 448.0f)) return 0x7Eu;
    if (u >= 0.015625f) {                       // normal range, >= 2^-6
        uint32_t bits = __float_as_uint(u);
        // keep 3 mantissa bits: add half an ulp minus one plus the kept lsb, then truncate
        bits += 0x7FFFFu + ((bits >> 20) & 1u);
        return (bits >> 20) - (120u << 3);      // rebias exponent 127 -> 7
    }
    // subnormal range: multiples of 2^-9; the product is exact, rint is nearest-even;
    // a result of 8 is the byte of the smallest normal, 2^-6
    return (uint32_t)__builtin_rintf(u * 512.0f);
}

// Value of an E4M3 byte in 0x00..0x7E as fp32 (exact).
__device__ __forceinline__ float e4m3_decode(uint32_t b) {
    float sub = (float)b * 0x1p-9f;                               // exponent field 0
    float nor = __uint_as_float((b << 20) + (120u << 23));        // exponent field e -> e + 120
    return b < 8u ? sub : nor;
}

// Index 0..7 of the E2M1 magnitude nearest to w >= 0; ties to the even index; w > 6 -> 6.
// Midpoints 0.25 .75 1.25 1.75 2.5 3.5 5: the tie goes down when the lower neighbour is even.
__device__ __forceinline__ uint32_t e2m1_encode_mag(float w) {
    return (uint32_t)(w > 0.25f) + (uint32_t)(w >= 0.75f) + (uint32_t)(w > 1.25f) +
           (uint32_t)(w >= 1.75f) + (uint32_t)(w > 2.5f) + (uint32_t)(w >= 3.5f) +
           (uint32_t)(w > 5.0f);
}

// E2M1 magnitude of index 0..7 as fp32.
__device__ __forceinline__ float e2m1_mag(uint32_t idx) {
    float sub = 0.5f * (float)idx;                                // 0, 0.5
    float nor = __uint_as_float((idx << 22) + 0x3F000000u);       // (1 + m/2) * 2^(e-1)
    return idx < 2u ? sub : nor;
}

// Quantize one block of 16 fp32 values.  Outputs the scale byte, the effective scale
// s = E4M3value * s_T, and the 16 codes packed low-nibble-first into lo (elements 0..7)
// and hi (elements 8..15).
__device__ __forceinline__ void quantize_block16(const float (&v)[16], float s_T, float ginv,
                                                 uint32_t& sbyte, float& s,
                                                 uint32_t& lo, uint32_t& hi) {
    float amax = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) amax = fmaxf(amax, fabsf(v[i]));
    float u = amax * ginv;
    sbyte = e4m3_encode_sat(u);
    s = e4m3_decode(sbyte) * s_T;
    float inv = (s != 0.0f) ? 1.0f / s : 0.0f;
    lo = 0u;
    hi = 0u;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        float w = fabsf(v[i]) * inv;
        uint32_t code = e2m1_encode_mag(w) | ((__float_as_uint(v[i]) >> 28) & 8u);
        if (i < 8) lo |= code << (4 * i);
        else       hi |= code << (4 * (i - 8));
    }
}

// Residual of one block: r_i = fma(-G[code_i] * sign_i, s, v_i), one rounding
// (Section 3.2 step (2): R_o = X_o - s * Q_{X_o}).
__device__ __forceinline__ void residual_block16(const float (&v)[16], float s,
                                                 uint32_t lo, uint32_t hi, float (&r)[16]) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        uint32_t code = ((i < 8 ? lo : hi) >> (4 * (i & 7))) & 0xFu;
        float g = e2m1_mag(code & 7u);
        float gs = __uint_as_float(__float_as_uint(g) | ((code & 8u) << 28));
        r[i] = __builtin_fmaf(-gs, s, v[i]);
    }
}

}  // namespace arcq
