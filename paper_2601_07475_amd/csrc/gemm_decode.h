// Exact decode of packed NVFP4 operands to fp16 in registers, shared by the GEMM kernels.
// A code * scale product needs up to 6 significant bits and lies in [2^-10, 2688]: exactly representable in fp16.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace arcq {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
// Both halves of a packed fp16 pair set to (E4M3 value of byte b) * 2^-8: (b << 7) read as fp16
// has the E4M3 exponent and mantissa fields in place with an exponent bias of 15 instead of 7,
// and the subnormal ranges of the two formats line up.  b <= 0x7E.
__device__ __forceinline__ half2v scale_pair(uint32_t b) {
    return __builtin_bit_cast(half2v, b * 0x00800080u);
}

// Eight E2M1 codes (element i in bits 4i..4i+3) times one block scale -> 8 fp16, exact.
// v_cvt_scalef32_pk_f16_fp4 turns one byte into two fp16 (low nibble first) times a power of
// two; 2^8 undoes the 2^-8 of scale_pair.  code * 256 <= 1536 and the product <= 2688 fit fp16.
__device__ __forceinline__ half8 decode8(uint32_t c, half2v sc) {
    half2v p0 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(c, 256.0f, 0) * sc;
    half2v p1 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(c, 256.0f, 1) * sc;
    half2v p2 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(c, 256.0f, 2) * sc;
    half2v p3 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(c, 256.0f, 3) * sc;
    half8 out = {p0[0], p0[1], p1[0], p1[1], p2[0], p2[1], p3[0], p3[1]};
    return out;
}

// The same with the scale taken from one half of a register that holds the fp16 scales of two blocks:
// a byte permute spreads two scale bytes (bits 0-7 and 8-15 of s) to bits 0-7 and 16-23, one shift puts
// both in place, and the packed multiplies broadcast the half they need through their operand-select
// modifiers.  Two vector instructions per two blocks (four k-steps) instead of two per k-step.
// `sel` picks the two bytes: 0x0C010C00 takes bytes 0 and 1 of s, 0x0C030C02 bytes 2 and 3.
__device__ __forceinline__ uint32_t scale_halves(uint32_t s, uint32_t sel) {
    return __builtin_amdgcn_perm(0u, s, sel) << 7;
}
__device__ __forceinline__ half8 decode8_half(uint32_t c, uint32_t halves, int hi) {
    const _Float16 s = __builtin_bit_cast(_Float16, (uint16_t)(hi ? halves >> 16 : halves));
    const half2v sc = {s, s};
    half2v p0 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(c, 256.0f, 0) * sc;
    half2v p1 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(c, 256.0f, 1) * sc;
    half2v p2 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(c, 256.0f, 2) * sc;
    half2v p3 = __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(c, 256.0f, 3) * sc;
    half8 out = {p0[0], p0[1], p1[0], p1[1], p2[0], p2[1], p3[0], p3[1]};
    return out;
}

// Loads with the alignment the interface guarantees rather than that of their size (codes: 8 bytes; scale bytes: 1).
// Global memory serves them in one request whatever the address; declaring the alignment keeps the access defined.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef u32x4 u32x4_a8 __attribute__((aligned(8)));
typedef u32x2 u32x2_a1 __attribute__((aligned(1)));
typedef uint32_t u32_a1 __attribute__((aligned(1)));
typedef uint16_t u16_a1 __attribute__((aligned(1)));
__device__ __forceinline__ uint4 load16_a8(const uint8_t* p) {
    const u32x4 v = *reinterpret_cast<const u32x4_a8*>(p);
    return uint4{v[0], v[1], v[2], v[3]};
}
typedef u32x4 u32x4_a4 __attribute__((aligned(4)));
__device__ __forceinline__ uint4 load16_a4(const uint8_t* p) {
    const u32x4 v = *reinterpret_cast<const u32x4_a4*>(p);
    return uint4{v[0], v[1], v[2], v[3]};
}
__device__ __forceinline__ uint2 load8_a8(const uint8_t* p) {
    const u32x2 v = *reinterpret_cast<const u32x2*>(p);
    return uint2{v[0], v[1]};
}
__device__ __forceinline__ uint2 load8_a1(const uint8_t* p) {
    const u32x2 v = *reinterpret_cast<const u32x2_a1*>(p);
    return uint2{v[0], v[1]};
}
__device__ __forceinline__ uint32_t load4_a1(const uint8_t* p) { return *reinterpret_cast<const u32_a1*>(p); }
__device__ __forceinline__ uint32_t load2_a1(const uint8_t* p) { return *reinterpret_cast<const u16_a1*>(p); }

}  // namespace arcq
