// MXFP4 variant of the fused activation quantizer and the offline weight packer: blocks of 32 E2M1
// elements with one E8M0 (power-of-two) scale, no tensor scale (Section 3.1 "Block-scaled
// Quantization", Appendix A); the residual channels, their placement behind the K primary channels
// and the duplicated weight blocks are those of Section 3.2 unchanged.  The scale follows the OCP
// Microscaling rule: shared exponent = floor(log2(block maximum)) - 2.  Everything but the element
// rounding is exact (power-of-two scaling; the residual v - X Q needs at most 13 significant bits).
//
// Same row pipeline as the NVFP4 quantizer: a workgroup owns whole rows, a row travels HBM -> LDS with
// global_load_lds_dwordx4 into one of two buffers while the previous row is being processed, every
// lane owns whole 32-channel blocks and gathers its channels from LDS by the permutation.
#include "internal.h"
#include "lds_dma.h"

#include <hip/hip_fp16.h>

namespace arcq {

namespace {

typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(1))) const void global_void_t;
typedef float float2v __attribute__((ext_vector_type(2)));

#define ARCQ_MX_WAIT_VMCNT(N) __builtin_amdgcn_s_waitcnt(((N) & 0xF) | (((N) >> 4) << 14) | 0x0F70)

// One block of 32 fp32 values -> E8M0 byte, the scale X = 2^(byte - 127) and 32 codes (element i in
// nibble i % 8 of c[i / 8]).  v_cvt_scalef32_pk_fp4_f32 with scale 1.0 rounds to nearest even on the
// E2M1 grid, saturates at +-6 and keeps the sign of zero (checked on the GPU over every fp16 input).
// scale_up (uniform over the launch): X is the smallest power of two with amax <= 6 X, one step above the
// rule above exactly when the significand of amax exceeds 1.5, so that no element saturates.
__device__ __forceinline__ void mx_quantize_block32(const float (&v)[32], uint32_t& sbyte, float& X, uint32_t (&c)[4],
                                                    bool scale_up = false) {
    float amax = 0.0f;
#pragma unroll
    for (int i = 0; i < 32; ++i) amax = fmaxf(amax, fabsf(v[i]));
    // amax is zero or a normal fp32 number: its exponent field is floor(log2) + 127
    const uint32_t ef = __float_as_uint(amax) >> 23;
    const uint32_t bump = scale_up && (__float_as_uint(amax) & 0x7FFFFFu) > 0x400000u ? 1u : 0u;
    sbyte = amax > 0.0f ? ef - 2u + bump : 127u;
    X = __uint_as_float(sbyte << 23);
    const float inv = __uint_as_float((254u - sbyte) << 23);            // 1 / X, exact
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        uint32_t p = 0u;
        p = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p, v[8 * w + 0] * inv, v[8 * w + 1] * inv, 1.0f, 0);
        p = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p, v[8 * w + 2] * inv, v[8 * w + 3] * inv, 1.0f, 1);
        p = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p, v[8 * w + 4] * inv, v[8 * w + 5] * inv, 1.0f, 2);
        p = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p, v[8 * w + 6] * inv, v[8 * w + 7] * inv, 1.0f, 3);
        c[w] = p;
    }
}

// r_i = v_i - X * Q_i (Section 3.2 step (2)), exact.
__device__ __forceinline__ void mx_residual_block32(const float (&v)[32], float X, const uint32_t (&c)[4], float (&r)[32]) {
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const float2v g[4] = {__builtin_amdgcn_cvt_scalef32_pk_f32_fp4(c[w], 1.0f, 0),
                              __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(c[w], 1.0f, 1),
                              __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(c[w], 1.0f, 2),
                              __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(c[w], 1.0f, 3)};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            r[8 * w + 2 * q] = __builtin_fmaf(-g[q][0], X, v[8 * w + 2 * q]);
            r[8 * w + 2 * q + 1] = __builtin_fmaf(-g[q][1], X, v[8 * w + 2 * q + 1]);
        }
    }
}

// BPT  32-channel blocks per lane (1 or 2);  MODE 0: activations (residual blocks), 1: weights (copies)
// DB   two LDS row buffers (rows up to 36864 channels), else one.
// STREAM  inputs far larger than the caches: rows are loaded with the non-temporal, system-scope policy.
// flags   ARCQ_LAYOUT_INTERLEAVED: the partner of outlier block i sits right behind it (Appendix D);
//         ARCQ_SCALE_ROUND_UP: see mx_quantize_block32.
template <int BPT, int MODE, bool DB, bool STREAM>
__global__ __launch_bounds__(1024) void mx_quantize_rows_kernel(
    const uint16_t* __restrict__ x, int64_t ldx, int rows, int K, int S, const int32_t* __restrict__ perm,
    uint8_t* __restrict__ codes, uint8_t* __restrict__ scales, uint32_t flags) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds_row[];
    const bool interleaved = (flags & ARCQ_LAYOUT_INTERLEAVED) != 0;
    const bool scale_up = (flags & ARCQ_SCALE_ROUND_UP) != 0;
    constexpr int NPRE = 4 * BPT;           // 16-byte pieces of a row per lane
    const int tid = threadIdx.x, T = blockDim.x;
    const int nb = K >> 5, nbo = S >> 5, first_o = nb - nbo;
    const int n16 = K >> 3;
    const uint32_t lds_stride = 64u * BPT * (uint32_t)T;     // >= 2K bytes
    const int64_t code_pitch = (int64_t)(K + S) >> 1, scale_pitch = (int64_t)(K + S) >> 5;

    int row = blockIdx.x;
    if (row >= rows) return;

    int piece[NPRE];
#pragma unroll
    for (int p = 0; p < NPRE; ++p) piece[p] = min(tid + p * T, n16 - 1);
    const uint32_t wave_first = (uint32_t)(tid & ~63);
    auto issue = [&](int r, uint32_t base) {
        const uint4* src = reinterpret_cast<const uint4*>(x + (int64_t)r * ldx);
#pragma unroll
        for (int p = 0; p < NPRE; ++p) {
            const uint32_t dst = base + 16u * (wave_first + (uint32_t)(p * T));
            __builtin_amdgcn_global_load_lds((global_void_t*)(src + piece[p]), (lds_void_t*)(lds_row + dst), 16, 0, STREAM ? 18 : 0);   // 2 = nt, 16 = sc1
        }
    };

    // lanes past the last block repeat it (same values to the same addresses)
    int blk[BPT];
    uint32_t chan[BPT][16];                 // source channels of the lane's blocks, two 16-bit indices per register
#pragma unroll
    for (int j = 0; j < BPT; ++j) {
        blk[j] = min(tid + j * T, nb - 1);
        const int4* pp = reinterpret_cast<const int4*>(perm + 32 * blk[j]);
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int4 v4 = pp[q];
            chan[j][2 * q] = (uint32_t)v4.x | ((uint32_t)v4.y << 16);
            chan[j][2 * q + 1] = (uint32_t)v4.z | ((uint32_t)v4.w << 16);
        }
    }

    uint32_t base = 0;
    if (DB) {
        issue(row, 0);
        ARCQ_MX_WAIT_VMCNT(0);
    }
    for (; row < rows; row += gridDim.x) {
        if (DB) {
            __syncthreads();                // row landed for every wave; previous compute finished
            const int next = row + gridDim.x;
            issue(next < rows ? next : row, base ^ lds_stride);
        } else {
            issue(row, 0);
            ARCQ_MX_WAIT_VMCNT(0);
            __syncthreads();
        }
        uint8_t* crow = codes + (int64_t)row * code_pitch;
        uint8_t* srow = scales + (int64_t)row * scale_pitch;
#pragma unroll
        for (int j = 0; j < BPT; ++j) {
            const int b = blk[j];
            float v[32];
#pragma unroll
            for (int i = 0; i < 32; ++i) {
                const uint32_t ch = (chan[j][i >> 1] >> (16 * (i & 1))) & 0xFFFFu;
                v[i] = __half2float(*reinterpret_cast<const __half*>(lds_row + base + 2u * ch));
            }
            uint32_t sbyte, c[4];
            float X;
            mx_quantize_block32(v, sbyte, X, c, scale_up);
            const int io = b - first_o;                 // >= 0: outlier block number
            const int bp = interleaved && io > 0 ? b + io : b;
            *reinterpret_cast<uint4*>(crow + 16 * (int64_t)bp) = make_uint4(c[0], c[1], c[2], c[3]);
            srow[bp] = (uint8_t)sbyte;
            if (io >= 0) {
                const int ba = interleaved ? bp + 1 : nb + io;
                if (MODE == 0) {
                    float r[32];
                    mx_residual_block32(v, X, c, r);
                    mx_quantize_block32(r, sbyte, X, c, scale_up);
                }
                *reinterpret_cast<uint4*>(crow + 16 * (int64_t)ba) = make_uint4(c[0], c[1], c[2], c[3]);
                srow[ba] = (uint8_t)sbyte;
            }
        }
        if (DB) {
            ARCQ_MX_WAIT_VMCNT(2 * BPT);    // the next row's loads are older than these stores
            base ^= lds_stride;
        } else {
            __syncthreads();
        }
    }
}

// Rows of up to 16384 channels: TWO lanes per block, 16 channels each, so that a row keeps twice as many lanes
// busy and a lane's dependent chain is half as long (the 22 MB input of a 2048 x 4096 layer went from 9.4 to
// about 7 us; with 32 channels per lane such a row occupies two waves).  The two lanes of a block are
// neighbours: they exchange their partial block maxima with one data-parallel-primitive move, compute the same
// scale, and each encodes and stores its own 8 bytes of codes.  Both store the scale byte (same value, same
// address), which keeps the number of stores per wave behind the row copies uniform for the counted wait.
// Everything else as in mx_quantize_rows_kernel with one block per lane and two row buffers.
__device__ __forceinline__ float pair_max(float a) {
    const int o = __builtin_amdgcn_update_dpp(0, __float_as_int(a), 0xB1, 0xF, 0xF, true);   // quad_perm [1,0,3,2]
    return fmaxf(a, __int_as_float(o));
}
__device__ __forceinline__ void mx_quantize_half16(const float (&v)[16], uint32_t& sbyte, float& X, uint32_t (&c)[2], bool scale_up) {
    float amax = 0.0f;
#pragma unroll
    for (int i = 0; i < 16; ++i) amax = fmaxf(amax, fabsf(v[i]));
    amax = pair_max(amax);
    const uint32_t ef = __float_as_uint(amax) >> 23;
    const uint32_t bump = scale_up && (__float_as_uint(amax) & 0x7FFFFFu) > 0x400000u ? 1u : 0u;
    sbyte = amax > 0.0f ? ef - 2u + bump : 127u;
    X = __uint_as_float(sbyte << 23);
    const float inv = __uint_as_float((254u - sbyte) << 23);            // 1 / X, exact
#pragma unroll
    for (int w = 0; w < 2; ++w) {
        uint32_t p = 0u;
        p = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p, v[8 * w + 0] * inv, v[8 * w + 1] * inv, 1.0f, 0);
        p = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p, v[8 * w + 2] * inv, v[8 * w + 3] * inv, 1.0f, 1);
        p = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p, v[8 * w + 4] * inv, v[8 * w + 5] * inv, 1.0f, 2);
        p = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(p, v[8 * w + 6] * inv, v[8 * w + 7] * inv, 1.0f, 3);
        c[w] = p;
    }
}

template <int MODE, bool STREAM>
__global__ __launch_bounds__(1024) void mx_quantize_pairs_kernel(
    const uint16_t* __restrict__ x, int64_t ldx, int rows, int K, int S, const int32_t* __restrict__ perm,
    uint8_t* __restrict__ codes, uint8_t* __restrict__ scales, uint32_t flags) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds_row[];
    const bool interleaved = (flags & ARCQ_LAYOUT_INTERLEAVED) != 0;
    const bool scale_up = (flags & ARCQ_SCALE_ROUND_UP) != 0;
    constexpr int NPRE = 2;                 // 16-byte pieces of a row per lane
    const int tid = threadIdx.x, T = blockDim.x;
    const int nb = K >> 5, nbo = S >> 5, first_o = nb - nbo;
    const int n16 = K >> 3;
    const uint32_t lds_stride = 32u * (uint32_t)T;           // >= 2K bytes
    const int64_t code_pitch = (int64_t)(K + S) >> 1, scale_pitch = (int64_t)(K + S) >> 5;

    int row = blockIdx.x;
    if (row >= rows) return;

    int piece[NPRE];
#pragma unroll
    for (int p = 0; p < NPRE; ++p) piece[p] = min(tid + p * T, n16 - 1);
    const uint32_t wave_first = (uint32_t)(tid & ~63);
    auto issue = [&](int r, uint32_t base) {
        const uint4* src = reinterpret_cast<const uint4*>(x + (int64_t)r * ldx);
#pragma unroll
        for (int p = 0; p < NPRE; ++p) {
            const uint32_t dst = base + 16u * (wave_first + (uint32_t)(p * T));
            __builtin_amdgcn_global_load_lds((global_void_t*)(src + piece[p]), (lds_void_t*)(lds_row + dst), 16, 0, STREAM ? 18 : 0);
        }
    };

    // lane pairs past the last block repeat it (same values to the same addresses)
    const int b = min(tid >> 1, nb - 1), half = tid & 1;
    uint32_t chan[8];                       // source channels of the lane's half block, two 16-bit indices per register
    {
        const int4* pp = reinterpret_cast<const int4*>(perm + 32 * b + 16 * half);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int4 v4 = pp[q];
            chan[2 * q] = (uint32_t)v4.x | ((uint32_t)v4.y << 16);
            chan[2 * q + 1] = (uint32_t)v4.z | ((uint32_t)v4.w << 16);
        }
    }
    const int io = b - first_o;                 // >= 0: outlier block number
    const int bp = interleaved && io > 0 ? b + io : b;
    const int ba = interleaved ? bp + 1 : nb + io;

    uint32_t base = 0;
    issue(row, 0);
    ARCQ_MX_WAIT_VMCNT(0);
    for (; row < rows; row += gridDim.x) {
        __syncthreads();                    // row landed for every wave; previous compute finished
        const int next = row + gridDim.x;
        issue(next < rows ? next : row, base ^ lds_stride);
        uint8_t* crow = codes + (int64_t)row * code_pitch;
        uint8_t* srow = scales + (int64_t)row * scale_pitch;
        float v[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const uint32_t ch = (chan[i >> 1] >> (16 * (i & 1))) & 0xFFFFu;
            v[i] = __half2float(*reinterpret_cast<const __half*>(lds_row + base + 2u * ch));
        }
        uint32_t sbyte, c[2];
        float X;
        mx_quantize_half16(v, sbyte, X, c, scale_up);
        *reinterpret_cast<uint2*>(crow + 16 * (int64_t)bp + 8 * half) = make_uint2(c[0], c[1]);
        srow[bp] = (uint8_t)sbyte;
        if (io >= 0) {                      // the same for both lanes of a pair
            if (MODE == 0) {
                // r_i = v_i - X * Q_i (Section 3.2 step (2)), exact
                float r[16];
#pragma unroll
                for (int w = 0; w < 2; ++w) {
                    const float2v g[4] = {__builtin_amdgcn_cvt_scalef32_pk_f32_fp4(c[w], 1.0f, 0),
                                          __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(c[w], 1.0f, 1),
                                          __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(c[w], 1.0f, 2),
                                          __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(c[w], 1.0f, 3)};
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        r[8 * w + 2 * q] = __builtin_fmaf(-g[q][0], X, v[8 * w + 2 * q]);
                        r[8 * w + 2 * q + 1] = __builtin_fmaf(-g[q][1], X, v[8 * w + 2 * q + 1]);
                    }
                }
                mx_quantize_half16(r, sbyte, X, c, scale_up);
            }
            *reinterpret_cast<uint2*>(crow + 16 * (int64_t)ba + 8 * half) = make_uint2(c[0], c[1]);
            srow[ba] = (uint8_t)sbyte;
        }
        ARCQ_MX_WAIT_VMCNT(2);              // the next row's loads are older than these stores
        base ^= lds_stride;
    }
}

template <int BPT, int MODE, bool DB, bool STREAM, bool PAIRS = false>
arcq_status launch_mx_t(int threads, size_t lds, const void* x, int64_t rows, int64_t K, int64_t ldx,
                        const int32_t* perm, int64_t S, uint8_t* codes, uint8_t* scales, uint32_t flags, hipStream_t stream) {
    auto kern = PAIRS ? mx_quantize_pairs_kernel<MODE, STREAM> : mx_quantize_rows_kernel<BPT, MODE, DB, STREAM>;
    static std::atomic<uint64_t> lds_raised{0};
    if (arcq_status st = raise_lds_limit(reinterpret_cast<const void*>(kern), lds_raised)) return st;
    // as many workgroups as the chip holds at once, never more than rows
    static thread_local int cached_threads = 0, cached_per_cu = 0;
    static thread_local size_t cached_lds = 0;
    if (cached_threads != threads || cached_lds != lds) {
        int n = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kern, threads, lds) != hipSuccess || n < 1) {
            (void)hipGetLastError();
            n = 1;
        }
        cached_threads = threads;
        cached_lds = lds;
        cached_per_cu = n;
    }
    int64_t wgs = (int64_t)num_cu() * cached_per_cu;
    if (wgs > rows) wgs = rows;
    hipLaunchKernelGGL(kern, dim3((unsigned)wgs), dim3(threads), lds, stream, static_cast<const uint16_t*>(x), ldx,
                       (int)rows, (int)K, (int)S, perm, codes, scales, flags);
    return check_launch("mx_quantize_rows_kernel");
}

}  // namespace

arcq_status launch_mx_quantize(int mode, const void* x, int64_t rows, int64_t K, int64_t ldx, const int32_t* perm,
                               int64_t S, uint8_t* codes, uint8_t* scales, uint32_t flags, hipStream_t stream) {
    const int nb = (int)(K >> 5);
    const bool stream_in = (uint64_t)rows * (uint64_t)K * 2 > (192ull << 20);   // beyond what the caches can hold
    if (nb <= 512) {
        // two lanes per block (see mx_quantize_pairs_kernel): 2 nb lanes, two row buffers of 64 nb bytes
        const int threads = (2 * nb + 63) / 64 * 64;
        const size_t lds = (size_t)64 * threads;
#define ARCQ_MX_PAIRS(ST) \
    return mode == 0 ? launch_mx_t<1, 0, true, ST, true>(threads, lds, x, rows, K, ldx, perm, S, codes, scales, flags, stream) \
                     : launch_mx_t<1, 1, true, ST, true>(threads, lds, x, rows, K, ldx, perm, S, codes, scales, flags, stream)
        if (stream_in) { ARCQ_MX_PAIRS(true); } else { ARCQ_MX_PAIRS(false); }
#undef ARCQ_MX_PAIRS
    }
    const int bpt = (nb + 1023) / 1024;                       // 1 or 2 for K <= 65536
    const int threads = ((nb + bpt - 1) / bpt + 63) / 64 * 64;
    const size_t stride = (size_t)64 * bpt * threads;
    const bool db = 2 * stride <= 144 * 1024;
    const size_t lds = db ? 2 * stride : stride;
#define ARCQ_MX_CASE2(B, D, ST) \
    return mode == 0 ? launch_mx_t<B, 0, D, ST>(threads, lds, x, rows, K, ldx, perm, S, codes, scales, flags, stream) \
                     : launch_mx_t<B, 1, D, ST>(threads, lds, x, rows, K, ldx, perm, S, codes, scales, flags, stream)
#define ARCQ_MX_CASE(B, D) \
    if (stream_in) { ARCQ_MX_CASE2(B, D, true); } else { ARCQ_MX_CASE2(B, D, false); }
    if (db) {
        if (bpt == 1) { ARCQ_MX_CASE(1, true); }
        ARCQ_MX_CASE(2, true);
    }
    ARCQ_MX_CASE(2, false);
#undef ARCQ_MX_CASE
#undef ARCQ_MX_CASE2
}

}  // namespace arcq
