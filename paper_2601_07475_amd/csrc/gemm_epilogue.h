// Output side shared by the GEMM kernels: conversion and stores of a wave's accumulator tiles.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace arcq {

typedef float float16v __attribute__((ext_vector_type(16)));

__device__ __forceinline__ void store_out(float* p, float v) { *p = v; }
__device__ __forceinline__ void store_out(_Float16* p, float v) { *p = (_Float16)v; }

// The same tile computed with the operands swapped (weights as the row operand): lane holds
// output ROW m (lane % 32) and register e holds column 8 * (e / 4) + 4 * (lane / 32) + e % 4, so
// every group of four registers is four consecutive n of one row of y: one 8-byte (fp16) or
// 16-byte (fp32) store instead of four scalar ones.  `vec_ok`: y and ldy allow such stores.
__device__ __forceinline__ void store4(float* p, float a, float b, float c, float d) {
    *reinterpret_cast<float4*>(p) = make_float4(a, b, c, d);
}
__device__ __forceinline__ void store4(_Float16* p, float a, float b, float c, float d) {
    typedef _Float16 half4v __attribute__((ext_vector_type(4)));
    *reinterpret_cast<half4v*>(p) = half4v{(_Float16)a, (_Float16)b, (_Float16)c, (_Float16)d};
}
// fragment row I of the tile
template <int WM, int WN, int I, typename OutT>
__device__ __forceinline__ void store_fragment_row_swapped(const float16v (&acc)[WM][WN], int m0, int n0, int r, int h, int M,
                                                           int N, float alpha, OutT* __restrict__ y, int64_t ldy, bool vec_ok) {
    const int m = m0 + 32 * I + r;
    if (m >= M) return;
    OutT* yrow = y + (int64_t)m * ldy;
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int n = n0 + 32 * j + 8 * g + 4 * h;
            const float v0 = acc[I][j][4 * g] * alpha, v1 = acc[I][j][4 * g + 1] * alpha,
                        v2 = acc[I][j][4 * g + 2] * alpha, v3 = acc[I][j][4 * g + 3] * alpha;
            if (vec_ok && n + 3 < N) {
                store4(yrow + n, v0, v1, v2, v3);
            } else {
                if (n < N) store_out(yrow + n, v0);
                if (n + 1 < N) store_out(yrow + n + 1, v1);
                if (n + 2 < N) store_out(yrow + n + 2, v2);
                if (n + 3 < N) store_out(yrow + n + 3, v3);
            }
        }
}
template <int WM, int WN, typename OutT>
__device__ __forceinline__ void store_tile_swapped(const float16v (&acc)[WM][WN], int m0, int n0, int r, int h, int M,
                                                   int N, float alpha, OutT* __restrict__ y, int64_t ldy, bool vec_ok) {
    store_fragment_row_swapped<WM, WN, 0>(acc, m0, n0, r, h, M, N, alpha, y, ldy, vec_ok);
    if constexpr (WM > 1) store_fragment_row_swapped<WM, WN, 1>(acc, m0, n0, r, h, M, N, alpha, y, ldy, vec_ok);
    if constexpr (WM > 2) store_fragment_row_swapped<WM, WN, 2>(acc, m0, n0, r, h, M, N, alpha, y, ldy, vec_ok);
    if constexpr (WM > 3) store_fragment_row_swapped<WM, WN, 3>(acc, m0, n0, r, h, M, N, alpha, y, ldy, vec_ok);
    static_assert(WM <= 4, "up to four fragment rows");
}

// fp16 output through the LDS, so that the global stores are whole lines: in the accumulator layout a
// store instruction of a wave touches 32 different rows with 16 bytes each, and the address unit of a
// CU spends about as long on such an instruction as on four that write eight full 128-byte lines; on
// tiles with a short reduction dimension the direct epilogue took several microseconds per tile.
// A wave writes two fragment rows (64 rows x 32 WN columns of fp16) into its own LDS region, row pitch
// 64 WN + 16 bytes (the padding spreads the 32 rows of one write over the banks and keeps every row
// 16-byte aligned), and reads them back row-contiguous, 16 bytes per lane: one store instruction then
// covers 16 / WN whole rows.
// lds_wave: this wave's region of epilogue_lds_bytes(WN) bytes, 16-byte aligned, not in use by anyone
// else (the caller synchronises the workgroup after the last read of the operand buffers).  Everything
// else as above.
constexpr int epilogue_lds_bytes(int WN) { return 64 * (64 * WN + 16); }

// Fragment rows I0 .. I0 + NI - 1 of a wave's tile (NI = 1 or 2) in one pass through the region.
template <int WM, int WN, int I0, int NI>
__device__ __forceinline__ void store_fragment_rows_f16_via_lds(const float16v (&acc)[WM][WN], uint8_t* lds_wave, int m0,
                                                                int n0, int lane, int M, int N, float alpha,
                                                                _Float16* __restrict__ y, int64_t ldy, bool vec_ok) {
    typedef _Float16 half4v __attribute__((ext_vector_type(4)));
    typedef _Float16 half8v __attribute__((ext_vector_type(8)));
    constexpr int ROWB = 64 * WN + 16;
    constexpr int LPR = 4 * WN;             // lanes per row when reading back (16 bytes each)
    constexpr int RPI = 64 / LPR;           // rows per store instruction
    const int r = lane & 31, h = lane >> 5;
#pragma unroll
    for (int ii = 0; ii < NI; ++ii)
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const half4v v = {(_Float16)(acc[I0 + ii][j][4 * g] * alpha), (_Float16)(acc[I0 + ii][j][4 * g + 1] * alpha),
                                  (_Float16)(acc[I0 + ii][j][4 * g + 2] * alpha), (_Float16)(acc[I0 + ii][j][4 * g + 3] * alpha)};
                *reinterpret_cast<half4v*>(lds_wave + (32 * ii + r) * ROWB + 2 * (32 * j + 8 * g + 4 * h)) = v;
            }
    // the reads below take what other lanes of this wave wrote: LDS operations of a wave complete in order
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int k = 0; k < 32 * NI / RPI; ++k) {
        const int row = k * RPI + lane / LPR, chunk = lane % LPR;
        const half8v v = *reinterpret_cast<const half8v*>(lds_wave + row * ROWB + 16 * chunk);
        const int m = m0 + 32 * I0 + row, n = n0 + 8 * chunk;
        if (m >= M) continue;
        _Float16* dst = y + (int64_t)m * ldy + n;
        if (vec_ok && n + 7 < N) {
            *reinterpret_cast<half8v*>(dst) = v;
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (n + e < N) dst[e] = v[e];
        }
    }
    // a following pass reuses the region
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int WM, int WN>
__device__ __forceinline__ void store_tile_f16_via_lds(const float16v (&acc)[WM][WN], uint8_t* lds_wave, int m0, int n0,
                                                       int lane, int M, int N, float alpha, _Float16* __restrict__ y,
                                                       int64_t ldy, bool vec_ok) {
    static_assert(WM >= 2 && WM <= 4, "two fragment rows at a time, then the rest");
    store_fragment_rows_f16_via_lds<WM, WN, 0, 2>(acc, lds_wave, m0, n0, lane, M, N, alpha, y, ldy, vec_ok);
    if constexpr (WM == 3)
        store_fragment_rows_f16_via_lds<WM, WN, 2, 1>(acc, lds_wave, m0, n0, lane, M, N, alpha, y, ldy, vec_ok);
    if constexpr (WM == 4)
        store_fragment_rows_f16_via_lds<WM, WN, 2, 2>(acc, lds_wave, m0, n0, lane, M, N, alpha, y, ldy, vec_ok);
}

}  // namespace arcq
