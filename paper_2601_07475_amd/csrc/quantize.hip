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
#include "lds_dma.h"
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
// NORM  RMSNorm in front of the quantizer (Section 3.3: the fused kernel integrates it): once a row
//       is in LDS the workgroup sums the squares of the values its lanes gather (the mean of squares is
//       defined with an exact sum, so no summation order enters the result; see the row loop), one wave
//       turns the sum into rstd, and every gathered value is normalised exactly like the reference
//       layer (fp32 multiply by rstd, cast to fp16, times gamma in fp16) before the block statistics.
//       Two more barriers per row.
//       1: gamma is copied once, coalesced, into LDS behind the row buffers and gathered from there
//          (into registers when a lane owns one block, per row otherwise);
//       2: no LDS left for it (very long rows): each lane gathers its gamma from global memory once.
// flags (uniform, see arcq.h): ARCQ_LAYOUT_INTERLEAVED puts the partner block of outlier block i (its
//       residual, or its copy for weights) right behind it, at block positions (K-S)/16 + 2i and + 2i + 1
//       (Appendix D), instead of at K/16 + i; ARCQ_SCALE_ROUND_UP rounds every block scale up.
// lds_stride = 32 * BPT * blockDim.x >= 2K: bytes of one row buffer, so that the lanes past
// the end of a row (which re-read its last 16 bytes) land in padding.
// Sum of v over each row of 16 lanes, in every lane of the row (data-parallel-primitive moves within
// quads, half rows and rows; the additions must be exact for the order not to matter).
template <int CTRL>
__device__ __forceinline__ double dpp_move(double v) {
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, 0xF, 0xF, true);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, 0xF, 0xF, true);
    return __hiloint2double(hi, lo);
}
__device__ __forceinline__ double row16_sum(double v) {
    v += dpp_move<0xB1>(v);     // quad_perm [1,0,3,2]
    v += dpp_move<0x4E>(v);     // quad_perm [2,3,0,1]
    v += dpp_move<0x141>(v);    // row_half_mirror
    v += dpp_move<0x140>(v);    // row_mirror
    return v;
}

template <int BPT, int MODE, bool DB, bool STREAM, int NORM>
__global__ __launch_bounds__(1024) __attribute__((amdgpu_waves_per_eu(BPT == 1 ? (NORM ? 6 : 8) : 4)))
void quantize_rows_kernel(
    const uint16_t* __restrict__ x, int64_t ldx, int rows, int K, int S,
    const int32_t* __restrict__ perm, float s_T, float ginv,
    uint8_t* __restrict__ codes, uint8_t* __restrict__ scales,
    const uint16_t* __restrict__ gamma, float eps, double delta, double inv_K, int force_exact, uint32_t flags) {
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
    const bool interleaved = (flags & ARCQ_LAYOUT_INTERLEAVED) != 0;
    const bool scale_up = (flags & ARCQ_SCALE_ROUND_UP) != 0;

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
    // LDS byte offsets of this lane's channels; the variant that also keeps gamma in registers packs them as
    // 16-bit channel indices, two per register (it would spill otherwise: 128 registers per lane is all a
    // workgroup of more than 512 lanes can have), and unpacks with one instruction per use
    constexpr bool PACK = NORM == 2;
    uint32_t off[PACK ? 1 : BPT][16];
    uint32_t chp[PACK ? BPT : 1][8];
#pragma unroll
    for (int j = 0; j < BPT; ++j) {
        blk[j] = min(tid + j * T, nb - 1);
        const int4* pp = reinterpret_cast<const int4*>(perm + 16 * blk[j]);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int4 v4 = pp[q];
            if constexpr (PACK) {
                chp[j][2 * q] = (uint32_t)v4.x | ((uint32_t)v4.y << 16);
                chp[j][2 * q + 1] = (uint32_t)v4.z | ((uint32_t)v4.w << 16);
            } else {
                off[j][4 * q + 0] = 2u * (uint32_t)v4.x;
                off[j][4 * q + 1] = 2u * (uint32_t)v4.y;
                off[j][4 * q + 2] = 2u * (uint32_t)v4.z;
                off[j][4 * q + 3] = 2u * (uint32_t)v4.w;
            }
        }
    }
    auto off_of = [&](int j, int i) -> uint32_t {
        if constexpr (PACK) {
            uint32_t c = chp[j][i >> 1];
            // keeps the unpacking inside the row loop (hoisted, it is 32 registers again): tied to the row number,
            // and not volatile, which would order the gathers of a lane one behind the other
            asm("" : "+v"(c) : "s"(row));
            return (i & 1) ? (c >> 15) & 0x1FFFEu : (c & 0xFFFFu) << 1;
        } else {
            return off[j][i];
        }
    };

    // NORM: gamma of this lane's channels, fixed for every row
    constexpr bool GAMMA_REGS = NORM == 2;      // fp16, two per register
    const uint8_t* lds_gamma = lds_row + (DB ? 2u : 1u) * lds_stride + 512u;
    uint32_t gam[GAMMA_REGS ? BPT : 1][8];
    if (NORM == 1) {
        uint4* dst = reinterpret_cast<uint4*>(lds_row + (DB ? 2u : 1u) * lds_stride + 512u);
        for (int p = tid; p < n16; p += T) dst[p] = reinterpret_cast<const uint4*>(gamma)[p];
        __syncthreads();
    }
    if (GAMMA_REGS) {
        auto g16 = [&](uint32_t byte_off) -> uint32_t {
            // an index from an unchecked perm may exceed K: keep the global read inside gamma
            return NORM == 1 ? *reinterpret_cast<const uint16_t*>(lds_gamma + byte_off) : gamma[min(byte_off >> 1, (uint32_t)K - 1u)];
        };
#pragma unroll
        for (int j = 0; j < BPT; ++j)
#pragma unroll
            for (int i = 0; i < 8; ++i) gam[j][i] = g16(off_of(j, 2 * i)) | (g16(off_of(j, 2 * i + 1)) << 16);
    }
    // LDS byte address of the statistics words behind the row buffers:
    // +0, +8, +16 integer sums of the exact path; +24 its rstd; +32, +40 fp64 sums of the fast path
    const uint32_t red = lds_address(lds_row) + (DB ? 2u : 1u) * lds_stride;
    if (NORM && tid < 5) lds_write_u64(red + (tid < 3 ? 8u * tid : 8u * tid + 8u), 0);   // the first barrier of the row loop follows
    uint32_t acc = red + 32;                // fp64 accumulator of the current row; rows alternate between +32 and +40

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

        float rstd = 1.0f;
        // KEEP: the lane's gathered values stay in registers (as fp32) from the statistics to the main pass, so the
        // statistics need no second read and conversion of the row (not with the packed channel indices: no room)
        constexpr bool KEEP = NORM == 1 && BPT <= 2;
        float xf[KEEP ? BPT : 1][16];
        if (KEEP) {
#pragma unroll
            for (int j = 0; j < BPT; ++j)
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    xf[j][i] = __half2float(*reinterpret_cast<const __half*>(lds_row + base + off_of(j, i)));
        }
        if (NORM) {
            // Mean of squares, defined with an EXACT sum (no summation order enters the result).
            // Fast path: a plain fp64 sum S^ of the squares (each exact in fp32).  Every term passes through
            // fewer than 150 roundings, so S^ = S (1 + t), |t| < 150 * 2^-53; with delta = (K + 260) 2^-52
            // the fp32 roundings of S^ (1 - delta) / K and S^ (1 + delta) / K (formed with a rounded 1/K:
            // three more roundings) bracket the fp32 rounding of the exactly summed value, because every
            // rounding is monotone.  If the two agree, that is the answer.
            // Otherwise (a row whose mean sits within delta of an fp32 rounding boundary, a few in 10^5)
            // the workgroup redoes the sum in integer arithmetic below.
            if (!force_exact && KEEP) {
                // every channel of the row is gathered by exactly one lane (perm is a permutation)
                double part = 0.0;
#pragma unroll
                for (int j = 0; j < BPT; ++j) {
                    double s16 = 0.0;
#pragma unroll
                    for (int i = 0; i < 16; ++i) s16 = __builtin_fma((double)xf[j][i], (double)xf[j][i], s16);
                    part += tid + j * T < nb ? s16 : 0.0;               // lanes past the last block hold a duplicate
                }
                part = row16_sum(part);
                if ((tid & 15) == 0) lds_add_f64(acc, part);
                wait_lgkmcnt0();
            } else if (!force_exact) {
                // each lane sums the contiguous 16-byte pieces it copied itself: wide, conflict-free reads
                double part = 0.0;
#pragma unroll
                for (int p = 0; p < NPRE; ++p) {
                    const lds_u32x4_t q4 = lds_read_b128(lds_address(lds_row) + base + 16u * (uint32_t)(tid + p * T));
                    double s8 = 0.0;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float lo = __half2float(__ushort_as_half((unsigned short)(q4[e] & 0xFFFFu)));
                        const float hi = __half2float(__ushort_as_half((unsigned short)(q4[e] >> 16)));
                        s8 = __builtin_fma((double)lo, (double)lo, s8);      // the square is exact, one rounding per term
                        s8 = __builtin_fma((double)hi, (double)hi, s8);
                    }
                    part += tid + p * T < n16 ? s8 : 0.0;               // slots past the row hold a duplicate
                }
                part = row16_sum(part);
                if ((tid & 15) == 0) lds_add_f64(acc, part);
                wait_lgkmcnt0();
            }
            wg_barrier();                    // not __syncthreads(): the next row's copy stays in flight
            bool decided = false;
            if (!force_exact) {
                // every wave finishes the statistics for itself: same sum, same operations, same result
                const double sum = lds_read_f64(acc);
                const double q = sum * inv_K;                           // one more rounding than a division would
                                                                        // have; delta has room for it
                const float ms_lo = (float)(q * (1.0 - delta)), ms_hi = (float)(q * (1.0 + delta));
                decided = ms_lo == ms_hi;
                rstd = 1.0f / __builtin_sqrtf(ms_lo + eps);             // IEEE square root and division
            }
            // The other accumulator serves the next row: every wave read it before this row's barriers,
            // and the next additions to it come after the barrier that opens that row.
            if (tid == 0) lds_write_u64(acc ^ 8u, 0);
            acc ^= 8u;
            if (__builtin_amdgcn_readfirstlane(decided ? 1 : 0) == 0) {     // the same in every wave of the workgroup
                // Exact path.  Every channel of the row is gathered by exactly one lane (perm is a
                // permutation), so the lanes' own gathered values cover the row.  x * 2^24 is an integer below 2^40; split as a * 2^20 + b with a, b < 2^20:
                //   (x 2^24)^2 = a^2 2^40 + 2 a b 2^20 + b^2.
                // The three sums stay integers below 2^53 in fp64 up to a row of 16 lanes (64 terms per lane
                // at most, each below 2^40), and go on as 64-bit integers from there (below 2^56 for K <= 65536).
                double d_aa = 0.0, d_ab = 0.0, d_bb = 0.0;
#pragma unroll
                for (int j = 0; j < BPT; ++j) {
                    double p_aa = 0.0, p_ab = 0.0, p_bb = 0.0;
#pragma unroll
                    for (int i = 0; i < 16; ++i) {
                        const float xv = KEEP ? xf[j][i] : __half2float(*reinterpret_cast<const __half*>(lds_row + base + off_of(j, i)));
                        const float s16 = fabsf(xv) * 16.0f;                // exact, < 2^20, a multiple of 2^-20
                        const float fa = truncf(s16);
                        const float fb = (s16 - fa) * 0x1p20f;              // exact
                        const double da = (double)fa, db = (double)fb;
                        p_aa = __builtin_fma(da, da, p_aa);
                        p_ab = __builtin_fma(da, db, p_ab);
                        p_bb = __builtin_fma(db, db, p_bb);
                    }
                    const bool live = tid + j * T < nb;
                    d_aa += live ? p_aa : 0.0;
                    d_ab += live ? p_ab : 0.0;
                    d_bb += live ? p_bb : 0.0;
                }
                d_aa = row16_sum(d_aa);
                d_ab = row16_sum(d_ab);
                d_bb = row16_sum(d_bb);
                if ((tid & 15) == 0) {
                    lds_add_u64(red, (uint64_t)d_aa);
                    lds_add_u64(red + 8, (uint64_t)d_ab);
                    lds_add_u64(red + 16, (uint64_t)d_bb);
                }
                wait_lgkmcnt0();
                wg_barrier();
                if (tid < 64) {
                    const uint64_t s_aa = lds_read_u64(red), s_ab = lds_read_u64(red + 8), s_bb = lds_read_u64(red + 16);
                    if (tid < 3) lds_write_u64(red + 8u * tid, 0);      // ready for the next such row
                    // N = s_aa 2^40 + s_ab 2^21 + s_bb (< 2^97) as six exact doubles, added without error
                    // into (hi, lo); hi + lo then rounds the exact integer once.
                    const double term[6] = {(double)(uint32_t)(s_aa >> 32) * 0x1p72, (double)(uint32_t)s_aa * 0x1p40,
                                            (double)(uint32_t)(s_ab >> 32) * 0x1p53, (double)(uint32_t)s_ab * 0x1p21,
                                            (double)(uint32_t)(s_bb >> 32) * 0x1p32, (double)(uint32_t)s_bb};
                    double hi = term[0], lo = 0.0;
#pragma unroll
                    for (int k = 1; k < 6; ++k) {
                        const double sum = hi + term[k];
                        const double bb = sum - hi;
                        const double err = (hi - (sum - bb)) + (term[k] - bb);   // hi + term = sum + err exactly
                        hi = sum;
                        lo += err;           // integers below 2^53: exact
                    }
                    const double sumsq = (hi + lo) * 0x1p-48;
                    const float ms = (float)(sumsq / (double)K);
                    const float r = 1.0f / __builtin_sqrtf(ms + eps);
                    if (tid == 0) lds_write_f32(red + 24, r);
                    wait_lgkmcnt0();
                }
                wg_barrier();
                rstd = lds_read_f32(red + 24);
            }
        }

        uint8_t* crow = codes + (int64_t)row * code_pitch;
        uint8_t* srow = scales + (int64_t)row * scale_pitch;
#pragma unroll
        for (int j = 0; j < BPT; ++j) {
            const int b = blk[j];
            float v[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                if (NORM) {
                    // t = fl16(fl32(x * rstd)): two roundings, as the reference layer does it.  The product is
                    // pinned to a register between them; left alone the compiler fuses multiply and conversion
                    // into one mixed-precision multiply-add, which rounds once (a different fp16 value once in
                    // some 10^7 elements) and adds +0 (so -0 becomes +0).
                    float prod = (KEEP ? xf[j][i] : __half2float(*reinterpret_cast<const __half*>(lds_row + base + off_of(j, i)))) * rstd;
                    asm("" : "+v"(prod));
                    const __half t16 = __float2half_rn(prod);
                    const __half g = GAMMA_REGS
                        ? __ushort_as_half((unsigned short)((gam[j][i >> 1] >> (16 * (i & 1))) & 0xFFFFu))
                        : *reinterpret_cast<const __half*>(lds_gamma + off_of(j, i));
                    // fp16 times fp16 rounded once to fp16
                    v[i] = __half2float(__hmul(t16, g));
                } else {
                    v[i] = __half2float(*reinterpret_cast<const __half*>(lds_row + base + off_of(j, i)));
                }
            }
            uint32_t sbyte, lo, hi;
            float s;
            quantize_block16(v, s_T, ginv, sbyte, s, lo, hi, scale_up);
            const int io = b - first_o;                 // >= 0: outlier block number
            const int bp = interleaved && io > 0 ? b + io : b;             // position of the primary block
            *reinterpret_cast<uint2*>(crow + 8 * (int64_t)bp) = make_uint2(lo, hi);
            srow[bp] = (uint8_t)sbyte;
            if (io >= 0) {
                const int ba = interleaved ? bp + 1 : nb + io;              // position of its partner
                if (MODE == 0) {
                    float r[16];
                    residual_block16(v, s, lo, hi, r);
                    quantize_block16(r, s_T, ginv, sbyte, s, lo, hi, scale_up);
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

template <int BPT, int MODE, bool DB, bool STREAM, int NORM>
arcq_status launch_t(int threads, int grid /* workgroups per CU, an estimate */, size_t lds, const void* x, int64_t rows, int64_t K,
                     int64_t ldx, const int32_t* perm, int64_t S, float s_T, float ginv,
                     uint8_t* codes, uint8_t* scales, const void* gamma, float eps, uint32_t flags, hipStream_t stream) {
    auto kern = quantize_rows_kernel<BPT, MODE, DB, STREAM, NORM>;
    static std::atomic<uint64_t> lds_raised{0};
    if (arcq_status st = raise_lds_limit(reinterpret_cast<const void*>(kern), lds_raised)) return st;
    // One workgroup per row slot the chip can hold at once (registers and LDS decide; asked of the runtime
    // once per kernel variant and workgroup shape), never more than rows: every workgroup then loops over
    // its rows with the next row's copy in flight, and none waits for a slot.
    static thread_local int cached_threads = 0, cached_per_cu = 0;
    static thread_local size_t cached_lds = 0;
    if (cached_threads != threads || cached_lds != lds) {
        int n = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, kern, threads, lds) != hipSuccess || n < 1) {
            (void)hipGetLastError();
            n = grid;                        // the caller's estimate
        }
        cached_threads = threads;
        cached_lds = lds;
        cached_per_cu = n;
    }
    grid = cached_per_cu;
    int64_t wgs = (int64_t)num_cu() * grid;
    if (wgs > rows) wgs = rows;
    // relative half-width of the fast path's bracket, see the kernel; ARCQ_RMSNORM_EXACT_SUM sends every
    // row through the exact integer sum instead (results are identical)
    const double delta = (double)(K + 260) * 0x1p-52;
    const int force_exact = NORM != 0 && (flags & ARCQ_RMSNORM_EXACT_SUM) != 0;
    hipLaunchKernelGGL(kern, dim3((unsigned)wgs), dim3(threads), lds, stream,
                       static_cast<const uint16_t*>(x), ldx, (int)rows, (int)K, (int)S, perm, s_T,
                       ginv, codes, scales, static_cast<const uint16_t*>(gamma), eps, delta, 1.0 / (double)K, force_exact, flags);
    return check_launch("quantize_rows_kernel");
}

}  // namespace

arcq_status launch_quantize(int mode, const void* x, int64_t rows, int64_t K, int64_t ldx,
                            const int32_t* perm, int64_t S, float s_T,
                            uint8_t* codes, uint8_t* scales, const void* gamma, float eps, uint32_t flags,
                            hipStream_t stream) {
    const int nb = (int)(K >> 4);
    const int bpt = (nb + 1023) / 1024;                       // blocks per lane: 1..4 for K <= 65536
    const int threads = ((nb + bpt - 1) / bpt + 63) / 64 * 64;
    const size_t stride = (size_t)32 * bpt * threads;          // one row buffer, >= 2K bytes
    const bool db = 2 * stride <= 144 * 1024;                 // two row buffers fit the 160 KB LDS
    size_t lds = (db ? 2 * stride : stride) + 512;            // + statistics words of the RMSNorm variant
    int norm = 0;                                             // see the kernel's NORM parameter
    if (gamma) {
        norm = lds + 2 * (size_t)K <= 160 * 1024 ? 1 : 2;
        if (norm == 1) lds += 2 * (size_t)K;
    }
    // workgroups per CU if neither registers nor LDS limit them (refined per kernel variant at launch)
    const int waves = threads / 64;
    int per_cu = 32 / waves;
    const int by_lds = (int)((160 * 1024) / (lds + 512));
    if (per_cu > by_lds) per_cu = by_lds;
    if (per_cu < 1) per_cu = 1;
    const int grid = per_cu;
    // fp32 reciprocal of 6 * s_T, one rounding each (the host computes in IEEE binary32)
    volatile float six_sT = 6.0f * s_T;
    volatile float ginv = 1.0f / six_sT;

    const bool stream_in = (uint64_t)rows * (uint64_t)K * 2 > (192ull << 20);   // beyond what the caches can hold
#define ARCQ_Q_ARGS threads, (int)grid, lds, x, rows, K, ldx, perm, S, s_T, ginv, codes, scales, gamma, eps, flags, stream
#define ARCQ_Q_CASE2(B, D, ST)                                               \
    if (mode == 1) return launch_t<B, 1, D, ST, 0>(ARCQ_Q_ARGS);             \
    if (norm == 0) return launch_t<B, 0, D, ST, 0>(ARCQ_Q_ARGS);             \
    if (norm == 1) return launch_t<B, 0, D, ST, 1>(ARCQ_Q_ARGS);             \
    return launch_t<B, 0, D, ST, 2>(ARCQ_Q_ARGS)
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
