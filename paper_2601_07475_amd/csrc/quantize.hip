// Fused NVFP4 quantizer with augmented residual channels (activations) or duplicated
// outlier blocks (weights).  Section 3.2 "Online Activation Quantization" steps (1)-(3)
// and "Offline Weight Quantization"; Section 3.3 (single fused kernel, coalesced reads
// during the reorder, both quantizations held in registers).
//
// Shape of the kernel (HBM-bandwidth bound: 2K bytes in, 9K'/16 bytes out per row):
//   * a workgroup owns whole rows (grid-stride over rows); one row of fp16 is streamed
//     into LDS with 16-byte coalesced loads, because the channel permutation is arbitrary
//     and a direct gather from HBM would touch one cache line per element;
//   * each lane owns whole 16-channel blocks: it gathers its 16 values from LDS through
//     the permutation (kept in registers as LDS byte offsets for all rows), so block amax,
//     scale, codes, residual and the second quantization need no cross-lane traffic;
//   * a lane writes 8 bytes of codes and 1 scale byte per block; consecutive lanes write
//     consecutive addresses.
#include "internal.h"
#include "nvfp4_device.h"

#include <hip/hip_fp16.h>

namespace arcq {

namespace {

template <int BPT, int MODE>
__global__ void quantize_rows_kernel(const uint16_t* __restrict__ x, int64_t ldx, int rows, int K,
                                     int S, const int32_t* __restrict__ perm, float s_T, float ginv,
                                     uint8_t* __restrict__ codes, uint8_t* __restrict__ scales) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds_row[];   // K fp16 values
    const int tid = threadIdx.x;
    const int T = blockDim.x;
    const int nb = K >> 4;                  // primary blocks per row
    const int nbo = S >> 4;                 // outlier blocks per row
    const int first_o = nb - nbo;
    const int64_t code_pitch = (int64_t)(K + S) >> 1;
    const int64_t scale_pitch = (int64_t)(K + S) >> 4;

    // LDS byte offsets of this lane's channels, fixed for every row
    uint32_t off[BPT][16];
#pragma unroll
    for (int j = 0; j < BPT; ++j) {
        const int b = tid + j * T;
#pragma unroll
        for (int i = 0; i < 16; ++i) off[j][i] = (b < nb) ? 2u * (uint32_t)perm[16 * b + i] : 0u;
    }

    const int n16 = K >> 3;                 // 16-byte pieces per row
    for (int row = blockIdx.x; row < rows; row += gridDim.x) {
        const uint4* src = reinterpret_cast<const uint4*>(x + (int64_t)row * ldx);
        __syncthreads();                    // every lane is done gathering the previous row
        for (int i = tid; i < n16; i += T) reinterpret_cast<uint4*>(lds_row)[i] = src[i];
        __syncthreads();

#pragma unroll
        for (int j = 0; j < BPT; ++j) {
            const int b = tid + j * T;
            if (b >= nb) break;
            float v[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const __half h = *reinterpret_cast<const __half*>(lds_row + off[j][i]);
                v[i] = __half2float(h);
            }
            uint32_t sbyte, lo, hi;
            float s;
            quantize_block16(v, s_T, ginv, sbyte, s, lo, hi);
            uint8_t* crow = codes + (int64_t)row * code_pitch;
            uint8_t* srow = scales + (int64_t)row * scale_pitch;
            *reinterpret_cast<uint2*>(crow + 8 * (int64_t)b) = make_uint2(lo, hi);
            srow[b] = (uint8_t)sbyte;
            if (b >= first_o) {
                const int ba = nb + (b - first_o);      // augmented block index
                if (MODE == 0) {
                    float r[16];
                    residual_block16(v, s, lo, hi, r);
                    quantize_block16(r, s_T, ginv, sbyte, s, lo, hi);
                }
                *reinterpret_cast<uint2*>(crow + 8 * (int64_t)ba) = make_uint2(lo, hi);
                srow[ba] = (uint8_t)sbyte;
            }
        }
    }
}

int g_num_cu = 0;

int num_cu() {
    if (g_num_cu == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            n = 256;
        g_num_cu = n;
    }
    return g_num_cu;
}

template <int BPT, int MODE>
arcq_status launch_t(int threads, int grid, size_t lds, const void* x, int64_t rows, int64_t K,
                     int64_t ldx, const int32_t* perm, int64_t S, float s_T, float ginv,
                     uint8_t* codes, uint8_t* scales, hipStream_t stream) {
    auto kern = quantize_rows_kernel<BPT, MODE>;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return fail(ARCQ_HIP_ERROR, "hipFuncSetAttribute(LDS=%zu): %s", lds, hipGetErrorString(e));
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(threads), lds, stream,
                       static_cast<const uint16_t*>(x), ldx, (int)rows, (int)K, (int)S, perm, s_T,
                       ginv, codes, scales);
    return check_launch("quantize_rows_kernel");
}

}  // namespace

arcq_status launch_quantize(int mode, const void* x, int64_t rows, int64_t K, int64_t ldx,
                            const int32_t* perm, int64_t S, float s_T,
                            uint8_t* codes, uint8_t* scales, hipStream_t stream) {
    const int nb = (int)(K >> 4);
    const int bpt = (nb + 1023) / 1024;                       // blocks per lane: 1..4 for K <= 65536
    const int threads = ((nb + bpt - 1) / bpt + 63) / 64 * 64;
    const size_t lds = (size_t)K * 2;
    // enough workgroups to fill every CU several times over, never more than rows
    const int waves = threads / 64;
    int per_cu = 32 / waves;
    const int by_lds = (int)((160 * 1024) / (lds + 256));
    if (per_cu > by_lds) per_cu = by_lds;
    if (per_cu < 1) per_cu = 1;
    int64_t grid = (int64_t)num_cu() * per_cu;
    if (grid > rows) grid = rows;
    // fp32 reciprocal of 6 * s_T, one rounding each (the host computes in IEEE binary32)
    volatile float six_sT = 6.0f * s_T;
    volatile float ginv = 1.0f / six_sT;

#define ARCQ_Q_CASE(B)                                                                             \
    return mode == 0 ? launch_t<B, 0>(threads, (int)grid, lds, x, rows, K, ldx, perm, S, s_T, ginv, \
                                      codes, scales, stream)                                       \
                     : launch_t<B, 1>(threads, (int)grid, lds, x, rows, K, ldx, perm, S, s_T, ginv, \
                                      codes, scales, stream)
    switch (bpt) {
        case 1: ARCQ_Q_CASE(1);
        case 2: ARCQ_Q_CASE(2);
        case 3: ARCQ_Q_CASE(3);
        default: ARCQ_Q_CASE(4);
    }
#undef ARCQ_Q_CASE
}

}  // namespace arcq
