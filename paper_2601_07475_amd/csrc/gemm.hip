// W4A4 GEMM over the extended reduction dimension K' = K + S (Section 3.2 "Unified GEMM
// Execution", eq. (2)): y[m,n] = alpha * sum_b sa[m,b] sw[n,b] sum_i qa[m,16b+i] qw[n,16b+i].
//
// gfx950's scaled FP4 MFMA takes one power-of-two (E8M0) scale per 32 elements; NVFP4 has one
// E4M3 scale per 16.  A code*scale product needs up to 6 significant bits (2 from E2M1, 4 from
// E4M3) and lies in [2^-10, 2688], so it is exactly representable in fp16 (and in no 8/6/4-bit
// float).  Operands are therefore decoded exactly to fp16 in registers and multiplied with
// v_mfma_f32_32x32x16_f16; products (12 significant bits) are exact in the fp32 accumulator, so
// the only rounding is fp32 accumulation, plus the output cast.  The tensor scales form the
// epilogue factor alpha.
#include "internal.h"

#include <hip/hip_fp16.h>

namespace arcq {

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float float16v __attribute__((ext_vector_type(16)));

// E4M3 byte (finite, non-negative) -> fp16, exact.  (b << 7) read as fp16 is the value times
// 2^-8 (the subnormal ranges of the two formats line up), and 2^8 * 448 fits fp16.
__device__ __forceinline__ _Float16 scale_to_half(uint32_t b) {
    uint16_t bits = (uint16_t)(b << 7);
    _Float16 h = __builtin_bit_cast(_Float16, bits);
    return h * (_Float16)256.0f;
}

// Eight E2M1 codes (one uint32, element i in bits 4i..4i+3) times one block scale -> 8 fp16.
// magnitude bits eem placed at fp16 bits 11..9 read as the E2M1 value times 2^-14 (again the
// subnormals line up); multiply by 2^14, then by the scale: both products are exact.
__device__ __forceinline__ half8 decode8(uint32_t c, _Float16 scale) {
    half8 out;
    const half2v k14 = {(_Float16)16384.0f, (_Float16)16384.0f};
    const half2v sc = {scale, scale};
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        uint32_t byte = (c >> (8 * p)) & 0xFFu;
        uint32_t lo = ((byte & 0x7u) << 9) | ((byte & 0x8u) << 12);
        uint32_t hi = ((byte & 0x70u) << 5) | ((byte & 0x80u) << 8);
        uint32_t packed = lo | (hi << 16);
        half2v v = __builtin_bit_cast(half2v, packed);
        v = (v * k14) * sc;
        out[2 * p] = v[0];
        out[2 * p + 1] = v[1];
    }
    return out;
}

__device__ __forceinline__ void store_out(float* p, float v) { *p = v; }
__device__ __forceinline__ void store_out(_Float16* p, float v) { *p = (_Float16)v; }

// Workgroup = 4 waves in a 2 x 2 arrangement, tile 128 x 128, each wave 64 x 64 as 2 x 2 MFMA
// tiles of 32 x 32.  In the MFMA a lane supplies 8 consecutive k of row (lane % 32); lanes 0-31
// and 32-63 supply different k.  One loop iteration covers 64 k (4 blocks): lanes of half h read
// blocks 4q + 2h and 4q + 2h + 1 (16 bytes of codes, 2 scale bytes) of their rows and feed them
// to 4 MFMAs; A and W use the same lane -> k mapping, so the sum over k is complete.
template <typename OutT>
__global__ __launch_bounds__(256) void gemm_direct_kernel(
    const uint8_t* __restrict__ a_codes, const uint8_t* __restrict__ a_scales,
    const uint8_t* __restrict__ w_codes, const uint8_t* __restrict__ w_scales, int M, int N,
    int nbk, float alpha, OutT* __restrict__ y, int64_t ldy) {
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int r = lane & 31, h = lane >> 5;
    const int m0 = blockIdx.y * 128 + (wave >> 1) * 64;
    const int n0 = blockIdx.x * 128 + (wave & 1) * 64;
    const int64_t cpitch = (int64_t)nbk * 8, spitch = nbk;

    const uint8_t *ac[2], *as[2], *wc[2], *ws[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        int m = m0 + 32 * i + r;
        m = m < M ? m : M - 1;              // rows past the edge re-read the last row; never stored
        int n = n0 + 32 * i + r;
        n = n < N ? n : N - 1;
        ac[i] = a_codes + m * cpitch;
        as[i] = a_scales + m * spitch;
        wc[i] = w_codes + n * cpitch;
        ws[i] = w_scales + n * spitch;
    }

    float16v acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    for (int q = 0; q * 4 < nbk; ++q) {
        const int b0 = 4 * q + 2 * h;
        uint2 ca[2][2], cw[2][2];
        _Float16 sa[2][2], sw[2][2];
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int b = b0 + t;
                const bool ok = b < nbk;        // blocks past K' contribute zero
                ca[i][t] = ok ? *reinterpret_cast<const uint2*>(ac[i] + 8 * (int64_t)b) : make_uint2(0, 0);
                cw[i][t] = ok ? *reinterpret_cast<const uint2*>(wc[i] + 8 * (int64_t)b) : make_uint2(0, 0);
                sa[i][t] = scale_to_half(ok ? as[i][b] : 0);
                sw[i][t] = scale_to_half(ok ? ws[i][b] : 0);
            }
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            half8 fa[2], fw[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                fa[i] = decode8((t & 1) ? ca[i][t >> 1].y : ca[i][t >> 1].x, sa[i][t >> 1]);
                fw[i] = decode8((t & 1) ? cw[i][t >> 1].y : cw[i][t >> 1].x, sw[i][t >> 1]);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[i], fw[j], acc[i][j], 0, 0, 0);
        }
    }

    // D layout of the 32x32 MFMA: lane holds column (lane % 32); register e holds row
    // 8 * (e / 4) + 4 * (lane / 32) + e % 4.
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int n = n0 + 32 * j + r;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int m = m0 + 32 * i + 8 * (e >> 2) + 4 * h + (e & 3);
                if (m < M && n < N) store_out(y + (int64_t)m * ldy + n, acc[i][j][e] * alpha);
            }
        }
}

}  // namespace

size_t gemm_workspace_bytes(int64_t, int64_t, int64_t) { return 0; }

arcq_status launch_gemm(const uint8_t* a_codes, const uint8_t* a_scales,
                        const uint8_t* w_codes, const uint8_t* w_scales,
                        int64_t M, int64_t N, int64_t Kp, float alpha,
                        void* y, int y_dtype, int64_t ldy,
                        void*, size_t, hipStream_t stream) {
    dim3 grid((unsigned)((N + 127) / 128), (unsigned)((M + 127) / 128));
    const int nbk = (int)(Kp >> 4);
    if (y_dtype == ARCQ_DTYPE_F16)
        hipLaunchKernelGGL(gemm_direct_kernel<_Float16>, grid, dim3(256), 0, stream, a_codes, a_scales,
                           w_codes, w_scales, (int)M, (int)N, nbk, alpha, static_cast<_Float16*>(y), ldy);
    else
        hipLaunchKernelGGL(gemm_direct_kernel<float>, grid, dim3(256), 0, stream, a_codes, a_scales,
                           w_codes, w_scales, (int)M, (int)N, nbk, alpha, static_cast<float*>(y), ldy);
    return check_launch("gemm_direct_kernel");
}

}  // namespace arcq
