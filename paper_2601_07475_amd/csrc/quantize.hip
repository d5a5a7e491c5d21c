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

typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(1))) const void global_void_t;

// s_waitcnt that waits only for the vector-memory counter to drop to N (gfx9 encoding:
// vmcnt in bits 3:0 and 15:14, expcnt 6:4 and lgkmcnt 11:8 left at "no wait").
#define ARCQ_WAIT_VMCNT(N) __builtin_amdgcn_s_waitcnt(((N) & 0xF) | (((N) >> 4) << 14) | 0x0F70)

// BPT   16-channel blocks per lane (ceil(K/16 / workgroup size))
// MODE  0: activations, augmented blocks hold the quantized residual
//       1: weights, augmented blocks are copies of the outlier blocks
// DB    two LDS row buffers.  Rows travel HBM -> LDS with global_load_lds_dwordx4 (no
//       register staging): each wave instruction lands 64 x 16 contiguous bytes.  The loads
//       of row r+1 are issued right after the barrier that opens row r and stay in flight
//       during the whole compute phase of row r; one barrier per row.  Vector-memory
//       operations retire in issue order, so waiting until at most 2*BPT of them (this
//       iteration's code/scale stores, issued after the loads) are outstanding is enough to
//       know that the loads have landed, without draining the stores.
//       Without DB (rows too long for two buffers) load, barrier, compute, barrier.
// STREAM the input is far larger than the caches (hundreds of MB): rows are loaded with the
//       non-temporal, system-scope cache policy (each byte is used once), which measured 8 % faster
//       on a 470 MB input and 20 % slower on a cache-resident 42 MB one, hence the switch.
// lds_stride = 32 * BPT * blockDim.x >= 2K: bytes of one row buffer, so that the lanes past
// the end of a row (which re-read its last 16 bytes) land in padding.
template <int BPT, int MODE, bool DB, bool STREAM>
__global__ __launch_bounds__(1024) void quantize_rows_kernel(
    const uint16_t* __restrict__ x, int64_t ldx, int rows, int K, int S,
    const int32_t* __restrict__ perm, float s_T, float ginv,
    uint8_t* __restrict__ codes, uint8_t* __restrict__ scales) {
    extern __shared__ __attribute__((aligned(16))) uint8_t lds_row[];
    constexpr int NPRE = 2 * BPT;           // 16-byte pieces of a row per lane
    const int tid = threadIdx.x;
    const int T = blockDim.x;
    const int nb = K >> 4;                  // primary blocks per row
    const int nbo = S >> 4;                 // outlier blocks per row
    const int first_o = nb - nbo;
    const int n16 = K >> 3;                 // 16-byte pieces per row
    const uint32_t lds_stride = 32u * BPT * (uint32_t)T;
    const int64_t code_pitch = (int64_t)(K + S) >> 1;
    const int64_t scale_pitch = (int64_t)(K + S) >> 4;

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
            // LDS destination of lane l is (wave-uniform base) + 16 * l
            const uint32_t dst = base + 16u * (wave_first + (uint32_t)(p * T));
            // cache policy bits: 2 = nt, 16 = sc1
            __builtin_amdgcn_global_load_lds((global_void_t*)(src + piece[p]), (lds_void_t*)(lds_row + dst), 16, 0, STREAM ? 18 : 0);
        }
    };

    // Lanes past the last block of a row (only when K/16 is not a multiple of the workgroup
    // size) repeat the last block: same values stored to the same addresses, no divergence.
    int blk[BPT];
    uint32_t off[BPT][16];                  // LDS byte offsets of this lane's channels
#pragma unroll
    for (int j = 0; j < BPT; ++j) {
        blk[j] = min(tid + j * T, nb - 1);
        const int4* pp = reinterpret_cast<const int4*>(perm + 16 * blk[j]);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int4 v4 = pp[q];
            off[j][4 * q + 0] = 2u * (uint32_t)v4.x;
            off[j][4 * q + 1] = 2u * (uint32_t)v4.y;
            off[j][4 * q + 2] = 2u * (uint32_t)v4.z;
            off[j][4 * q + 3] = 2u * (uint32_t)v4.w;
        }
    }

    uint32_t base = 0;
    if (DB) {
        issue(row, 0);
        ARCQ_WAIT_VMCNT(0);
    }
    for (; row < rows; row += gridDim.x) {
        if (DB) {
            __syncthreads();                // row landed for every wave; previous compute finished
            const int next = row + gridDim.x;
            issue(next < rows ? next : row, base ^ lds_stride);   // last iteration: harmless re-read
        } else {
            issue(row, 0);
            ARCQ_WAIT_VMCNT(0);
            __syncthreads();
        }

        uint8_t* crow = codes + (int64_t)row * code_pitch;
        uint8_t* srow = scales + (int64_t)row * scale_pitch;
#pragma unroll
        for (int j = 0; j < BPT; ++j) {
            const int b = blk[j];
            float v[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const __half h = *reinterpret_cast<const __half*>(lds_row + base + off[j][i]);
                v[i] = __half2float(h);
            }
            uint32_t sbyte, lo, hi;
            float s;
            quantize_block16(v, s_T, ginv, sbyte, s, lo, hi);
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
        if (DB) {
            ARCQ_WAIT_VMCNT(2 * BPT);       // the next row's loads are older than these stores
            base ^= lds_stride;
        } else {
            __syncthreads();
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

template <int BPT, int MODE, bool DB, bool STREAM>
arcq_status launch_t(int threads, int grid, size_t lds, const void* x, int64_t rows, int64_t K,
                     int64_t ldx, const int32_t* perm, int64_t S, float s_T, float ginv,
                     uint8_t* codes, uint8_t* scales, hipStream_t stream) {
    auto kern = quantize_rows_kernel<BPT, MODE, DB, STREAM>;
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
    const size_t stride = (size_t)32 * bpt * threads;          // one row buffer, >= 2K bytes
    const bool db = 2 * stride <= 144 * 1024;                 // two row buffers fit the 160 KB LDS
    const size_t lds = db ? 2 * stride : stride;
    // enough workgroups to fill every CU, never more than rows
    const int waves = threads / 64;
    int per_cu = 32 / waves;
    const int by_lds = (int)((160 * 1024) / (lds + 512));
    if (per_cu > by_lds) per_cu = by_lds;
    if (per_cu < 1) per_cu = 1;
    int64_t grid = (int64_t)num_cu() * per_cu;
    if (grid > rows) grid = rows;
    // fp32 reciprocal of 6 * s_T, one rounding each (the host computes in IEEE binary32)
    volatile float six_sT = 6.0f * s_T;
    volatile float ginv = 1.0f / six_sT;

    const bool stream_in = (uint64_t)rows * (uint64_t)K * 2 > (192ull << 20);   // beyond what the caches can hold
#define ARCQ_Q_ARGS threads, (int)grid, lds, x, rows, K, ldx, perm, S, s_T, ginv, codes, scales, stream
#define ARCQ_Q_CASE2(B, D, ST)                                               \
    return mode == 0 ? launch_t<B, 0, D, ST>(ARCQ_Q_ARGS) : launch_t<B, 1, D, ST>(ARCQ_Q_ARGS)
#define ARCQ_Q_CASE(B, D)                                                    \
    if (stream_in) { ARCQ_Q_CASE2(B, D, true); } else { ARCQ_Q_CASE2(B, D, false); }
    if (db) {
        switch (bpt) {
            case 1: ARCQ_Q_CASE(1, true);
            case 2: ARCQ_Q_CASE(2, true);
            default: ARCQ_Q_CASE(3, true);                    // K <= 36864 here, so bpt <= 3
        }
    }
    switch (bpt) {
        case 3: ARCQ_Q_CASE(3, false);
        default: ARCQ_Q_CASE(4, false);
    }
#undef ARCQ_Q_CASE2
#undef ARCQ_Q_CASE
#undef ARCQ_Q_ARGS
}

}  // namespace arcq
