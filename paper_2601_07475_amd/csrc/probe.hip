// Diagnostic: the rate at which this machine issues the fp16 matrix instruction the NVFP4 GEMM is built on
// (v_mfma_f32_32x32x16_f16), with both operands held in registers and no memory traffic in the loop.  The
// figure is the practical ceiling the GEMM's roofline fraction should be read against: under a sustained
// matrix load the chip clocks below the frequency the published peak assumes.
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

}  // namespace

arcq_status launch_probe_mfma_f16(int iters, float* sink, double* flop_host, hipStream_t stream) {
    hipLaunchKernelGGL(mfma_rate_kernel, dim3(PROBE_WGS), dim3(PROBE_THREADS), 0, stream, iters, sink);
    if (arcq_status st = check_launch("mfma_rate_kernel")) return st;
    // waves * iterations * 4 instructions * 2 * 32 * 32 * 16 flop
    *flop_host = (double)PROBE_WGS * (PROBE_THREADS / 64) * (double)iters * 4.0 * 2.0 * 32.0 * 32.0 * 16.0;
    return ARCQ_OK;
}

}  // namespace arcq
