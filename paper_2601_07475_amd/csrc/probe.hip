// Diagnostic: the rate at which this machine issues the matrix instructions the GEMMs are built on
// (v_mfma_f32_32x32x16_f16 for NVFP4, v_mfma_scale_f32_32x32x64_f8f6f4 on FP4 operands for MXFP4), with
// both operands held in registers and no memory traffic in the loop.  The figures are the practical
// ceilings the GEMMs' roofline fractions should be read against: under a sustained matrix load the chip
// clocks below the frequency the published peaks assume.
#include "internal.h"
#include "gemm_epilogue.h"

namespace arcq {

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));

constexpr int PROBE_WGS = 1024;      // 4 workgroups of 4 waves per CU on 256 CUs: four waves per SIMD
constexpr int PROBE_THREADS = 256;

__global__ __launch_bounds__(PROBE_THREADS) void mfma_rate_kernel(int iters, float* __restrict__ sink) {
    const int gid = blockIdx.x * PROBE_THREADS + threadIdx.x;
    // operands that differ from lane to lane and from element to element (the data decides how many
    // wires toggle, and with them the power and the clock), small enough for the sums to stay finite
    half8 a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        a[e] = (_Float16)(0.001f * (float)(((gid * 8 + e) * 37) % 61 - 30));
        b[e] = (_Float16)(0.001f * (float)(((gid * 8 + e) * 53) % 59 - 29));
    }
    float16v acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[j][e] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc[j], 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[j][e];
    sink[gid] = s;
}

typedef int int8v __attribute__((ext_vector_type(8)));

__global__ __launch_bounds__(PROBE_THREADS) void mfma_fp4_rate_kernel(int iters, float* __restrict__ sink) {
    const int gid = blockIdx.x * PROBE_THREADS + threadIdx.x;
    // 32 E2M1 codes per operand and lane, different from lane to lane; unit block scales (E8M0 127)
    int8v a = {0, 0, 0, 0, 0, 0, 0, 0}, b = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        a[e] = (int)(0x9E3779B9u * (uint32_t)(gid * 4 + e + 1));
        b[e] = (int)(0x85EBCA6Bu * (uint32_t)(gid * 4 + e + 1));
    }
    const int one = 127;
    float16v acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[j][e] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc[j], 4, 4, 0, one, 0, one);
    }
    float s = 0.0f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[j][e];
    sink[gid] = s;
}

}  // namespace

arcq_status launch_probe_mfma_fp4(int iters, float* sink, double* flop_host, hipStream_t stream) {
    hipLaunchKernelGGL(mfma_fp4_rate_kernel, dim3(PROBE_WGS), dim3(PROBE_THREADS), 0, stream, iters, sink);
    if (arcq_status st = check_launch("mfma_fp4_rate_kernel")) return st;
    // waves * iterations * 4 instructions * 2 * 32 * 32 * 64 flop
    *flop_host = (double)PROBE_WGS * (PROBE_THREADS / 64) * (double)iters * 4.0 * 2.0 * 32.0 * 32.0 * 64.0;
    return ARCQ_OK;
}

arcq_status launch_probe_mfma_f16(int iters, float* sink, double* flop_host, hipStream_t stream) {
    hipLaunchKernelGGL(mfma_rate_kernel, dim3(PROBE_WGS), dim3(PROBE_THREADS), 0, stream, iters, sink);
    if (arcq_status st = check_launch("mfma_rate_kernel")) return st;
    // waves * iterations * 4 instructions * 2 * 32 * 32 * 16 flop
    *flop_host = (double)PROBE_WGS * (PROBE_THREADS / 64) * (double)iters * 4.0 * 2.0 * 32.0 * 32.0 * 16.0;
    return ARCQ_OK;
}

}  // namespace arcq
