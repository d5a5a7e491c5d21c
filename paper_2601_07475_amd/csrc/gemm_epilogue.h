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
template <int WM, int WN, typename OutT>
__device__ __forceinline__ void store_tile_swapped(const float16v (&acc)[WM][WN], int m0, int n0, int r, int h, int M,
                                                   int N, float alpha, OutT* __restrict__ y, int64_t ldy, bool vec_ok) {
#pragma unroll
    for (int i = 0; i < WM; ++i) {
        const int m = m0 + 32 * i + r;
        if (m >= M) continue;
        OutT* yrow = y + (int64_t)m * ldy;
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int n = n0 + 32 * j + 8 * g + 4 * h;
                const float v0 = acc[i][j][4 * g] * alpha, v1 = acc[i][j][4 * g + 1] * alpha,
                            v2 = acc[i][j][4 * g + 2] * alpha, v3 = acc[i][j][4 * g + 3] * alpha;
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
}

}  // namespace arcq
