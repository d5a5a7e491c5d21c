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
//
// One 32x32x16 MFMA consumes exactly one NVFP4 block of each operand: a lane supplies 8
// consecutive k of row (lane % 32); lanes 0-31 and 32-63 supply different octets.  A and W use
// the same lane -> k mapping, so any assignment of octets to lanes sums over all of k.
#include "internal.h"
#include "lds_dma.h"

#include <hip/hip_fp16.h>

#include <type_traits>

namespace arcq {

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float float16v __attribute__((ext_vector_type(16)));
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

__device__ __forceinline__ void store_out(float* p, float v) { *p = v; }
__device__ __forceinline__ void store_out(_Float16* p, float v) { *p = (_Float16)v; }

// Accumulates blocks [b_begin, b_end) straight from global memory (no staging): used for the
// K' tail of the staged kernel and as the whole loop of the fallback kernel.  One iteration
// covers 4 blocks: lanes of half h read blocks 4q + 2h and 4q + 2h + 1 of their rows.
template <int WM, int WN>
__device__ __forceinline__ void accumulate_direct(const uint8_t* const (&ac)[WM], const uint8_t* const (&as)[WM],
                                                  const uint8_t* const (&wc)[WN], const uint8_t* const (&ws)[WN],
                                                  int b_begin, int b_end, int h, float16v (&acc)[WM][WN]) {
    for (int q0 = b_begin; q0 < b_end; q0 += 4) {
        const int b0 = q0 + 2 * h;
        uint2 ca[WM][2], cw[WN][2];
        half2v sa[WM][2], sw[WN][2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int b = b0 + t;
            const bool ok = b < b_end;          // blocks past the end contribute zero
#pragma unroll
            for (int i = 0; i < WM; ++i) {
                ca[i][t] = ok ? *reinterpret_cast<const uint2*>(ac[i] + 8 * (int64_t)b) : make_uint2(0, 0);
                sa[i][t] = scale_pair(ok ? as[i][b] : 0);
            }
#pragma unroll
            for (int j = 0; j < WN; ++j) {
                cw[j][t] = ok ? *reinterpret_cast<const uint2*>(wc[j] + 8 * (int64_t)b) : make_uint2(0, 0);
                sw[j][t] = scale_pair(ok ? ws[j][b] : 0);
            }
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            half8 fa[WM], fw[WN];
#pragma unroll
            for (int i = 0; i < WM; ++i) fa[i] = decode8((t & 1) ? ca[i][t >> 1].y : ca[i][t >> 1].x, sa[i][t >> 1]);
#pragma unroll
            for (int j = 0; j < WN; ++j) fw[j] = decode8((t & 1) ? cw[j][t >> 1].y : cw[j][t >> 1].x, sw[j][t >> 1]);
#pragma unroll
            for (int i = 0; i < WM; ++i)
#pragma unroll
                for (int j = 0; j < WN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[i], fw[j], acc[i][j], 0, 0, 0);
        }
    }
}

// D layout of the 32x32 MFMA: lane holds column (lane % 32); register e holds row
// 8 * (e / 4) + 4 * (lane / 32) + e % 4.
template <int WM, int WN, typename OutT>
__device__ __forceinline__ void store_tile(const float16v (&acc)[WM][WN], int m0, int n0, int r, int h, int M,
                                           int N, float alpha, OutT* __restrict__ y, int64_t ldy) {
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j) {
            const int n = n0 + 32 * j + r;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int m = m0 + 32 * i + 8 * (e >> 2) + 4 * h + (e & 3);
                if (m < M && n < N) store_out(y + (int64_t)m * ldy + n, acc[i][j][e] * alpha);
            }
        }
}

// ---------------------------------------------------------------------------------------------
// Fallback: any K' (multiple of 16), operands read straight from global memory.
// Workgroup = 4 waves (2 x 2), tile 128 x 128, each wave 64 x 64.
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
    accumulate_direct<2, 2>(ac, as, wc, ws, 0, nbk, h, acc);
    store_tile<2, 2>(acc, m0, n0, r, h, M, N, alpha, y, ldy);
}

// ---------------------------------------------------------------------------------------------
// Staged kernel for K' % 64 == 0.  Workgroup = 4 waves (2 x 2); each wave owns WM x WN MFMA
// tiles of 32 x 32, so the workgroup tile is BM x BN = 64 WM x 64 WN.
//
// A stage is 128 k (8 blocks): per row 64 bytes of codes and 8 scale bytes, kept PACKED in
// LDS (4.5 bits per element) and decoded in registers after the LDS read.  Stages travel
// global -> LDS with global_load_lds (no register staging) through a ring of 3 buffers: the
// loads of stage s+2 are issued right after the barrier that opens stage s, so they have two
// stage times to land, and one barrier per stage suffices (passing the barrier of stage s
// means every wave has finished stage s-1, whose buffer stage s+2 reuses).
//
// LDS layout of one stage (bytes):  A codes [BM][64] | W codes [BN][64] | A scales [BM][8] |
// W scales [BN][8].  The four 16-byte pieces of a row's codes are stored XOR-swizzled with
// (row >> 1) & 3 so that the 16-byte reads of 8 consecutive rows fall in 8 different bank groups.
// A wave-wide DMA instruction writes lane l to (uniform base) + 16 l, so the swizzle is applied
// by choosing which global piece each lane fetches.
template <int WM, int WN>
struct StagedCfg {
    static constexpr int BM = 64 * WM, BN = 64 * WN;
    static constexpr int A_CODES = 0;
    static constexpr int W_CODES = BM * 64;
    static constexpr int A_SCALES = (BM + BN) * 64;
    static constexpr int W_SCALES = A_SCALES + BM * 8;
    static constexpr int STAGE_BYTES = (BM + BN) * 72;
    static constexpr int NSTAGE = 3;
    static constexpr int LDS_BYTES = NSTAGE * STAGE_BYTES;
    // DMA instructions per thread per stage: 16-byte pieces of codes, 4-byte pieces of scales
    static constexpr int NDMA = (BM + BN) / 64 + (BM + BN) / 128;
};

template <int WM, int WN, typename OutT>
__global__ __launch_bounds__(256) void gemm_staged_kernel(
    const uint8_t* __restrict__ a_codes, const uint8_t* __restrict__ a_scales,
    const uint8_t* __restrict__ w_codes, const uint8_t* __restrict__ w_scales, int M, int N,
    int nbk, float alpha, OutT* __restrict__ y, int64_t ldy, int tiles_m, int tiles_n) {
    using C = StagedCfg<WM, WN>;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

    // ---- workgroup -> tile.  Workgroups are dealt round-robin to the 8 XCDs (each with its
    // own L2); give every XCD a contiguous run of the tile sequence, and walk the sequence in
    // column-major groups of 8 tile rows so that concurrently running tiles share A and W rows.
    const int num_tiles = tiles_m * tiles_n;
    int pid = blockIdx.x;
    if ((num_tiles & 7) == 0) pid = (pid & 7) * (num_tiles >> 3) + (pid >> 3);
    constexpr int GROUP = 8;
    const int group_size = GROUP * tiles_n;
    const int g = pid / group_size;
    const int first_m = g * GROUP;
    const int gm = min(GROUP, tiles_m - first_m);
    const int in_g = pid - g * group_size;
    const int tile_m = first_m + in_g % gm;
    const int tile_n = in_g / gm;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int r = lane & 31, h = lane >> 5;
    const int wg_m0 = tile_m * C::BM, wg_n0 = tile_n * C::BN;
    const int wrow0 = (wave >> 1) * (32 * WM);       // first row of this wave inside the A tile
    const int wcol0 = (wave & 1) * (32 * WN);        // first row of this wave inside the W tile
    const int64_t cpitch = (int64_t)nbk * 8, spitch = nbk;

    // ---- DMA source offsets of this thread (bytes from the operand base, stage 0)
    // When K' is an odd multiple of 64 the last stage is half a stage (4 blocks): the lanes that
    // would fetch its missing second half re-fetch the first half instead (never used), which
    // keeps every access inside the operand.  `half` selects those adjusted offsets.
    const bool has_half = (nbk & 7) != 0;
    const int nstage = (nbk >> 3) + (has_half ? 1 : 0);
    uint32_t src_ac[C::BM / 64], src_wc[C::BN / 64], src_as[C::BM / 128], src_ws[C::BN / 128];
    uint32_t adj_c[2], adj_s;                  // (s & 3) and the row swizzle repeat every 256 slots
    {
        const int row = tid >> 2, lp = (tid & 3) ^ ((row >> 1) & 3);
        adj_c[0] = lp * 16;
        adj_c[1] = (lp & 1) * 16;
        adj_s = (tid & 1) * 4;
    }
#pragma unroll
    for (int p = 0; p < C::BM / 64; ++p)
        src_ac[p] = (uint32_t)(min(wg_m0 + ((p * 256 + tid) >> 2), M - 1) * cpitch);
#pragma unroll
    for (int p = 0; p < C::BN / 64; ++p)
        src_wc[p] = (uint32_t)(min(wg_n0 + ((p * 256 + tid) >> 2), N - 1) * cpitch);
#pragma unroll
    for (int p = 0; p < C::BM / 128; ++p)
        src_as[p] = (uint32_t)(min(wg_m0 + ((p * 256 + tid) >> 1), M - 1) * spitch);
#pragma unroll
    for (int p = 0; p < C::BN / 128; ++p)
        src_ws[p] = (uint32_t)(min(wg_n0 + ((p * 256 + tid) >> 1), N - 1) * spitch);
    const uint32_t wave_slot = (uint32_t)(tid & ~63);   // lane l of a DMA writes slot wave_slot + l
    const uint32_t lds0 = lds_address(lds);
    auto issue = [&](int stage, int buf) {
        const uint32_t base = lds0 + buf * C::STAGE_BYTES;
        const bool half = has_half && stage == nstage - 1;
        const uint32_t oc = (uint32_t)stage * 64u + (half ? adj_c[1] : adj_c[0]);
        const uint32_t os = (uint32_t)stage * 8u + (half ? 0u : adj_s);
#pragma unroll
        for (int p = 0; p < C::BM / 64; ++p)
            dma16(a_codes, src_ac[p] + oc, base + C::A_CODES + 16u * (p * 256 + wave_slot));
#pragma unroll
        for (int p = 0; p < C::BN / 64; ++p)
            dma16(w_codes, src_wc[p] + oc, base + C::W_CODES + 16u * (p * 256 + wave_slot));
#pragma unroll
        for (int p = 0; p < C::BM / 128; ++p)
            dma4(a_scales, src_as[p] + os, base + C::A_SCALES + 4u * (p * 256 + wave_slot));
#pragma unroll
        for (int p = 0; p < C::BN / 128; ++p)
            dma4(w_scales, src_ws[p] + os, base + C::W_SCALES + 4u * (p * 256 + wave_slot));
    };

    // ---- LDS read offsets of this lane inside a stage (piece index still to be swizzled)
    uint32_t rd_ac[WM], rd_wc[WN], rd_as[WM], rd_ws[WN], sw_a[WM], sw_w[WN];
#pragma unroll
    for (int i = 0; i < WM; ++i) {
        const int row = wrow0 + 32 * i + r;
        rd_ac[i] = C::A_CODES + row * 64;
        rd_as[i] = C::A_SCALES + row * 8 + 2 * h;
        sw_a[i] = (row >> 1) & 3;
    }
#pragma unroll
    for (int j = 0; j < WN; ++j) {
        const int row = wcol0 + 32 * j + r;
        rd_wc[j] = C::W_CODES + row * 64;
        rd_ws[j] = C::W_SCALES + row * 8 + 2 * h;
        sw_w[j] = (row >> 1) & 3;
    }

    float16v acc[WM][WN];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    // ---- per-stage compute, software-pipelined by hand.
    // A k-step (one block, 16 k) is WM*WN MFMAs fed by WM + WN fragments of 8 fp16 per lane.
    // While the MFMAs of step x run, the fragments of step x+1 are decoded: after every pair of
    // MFMAs the decode of one (or two) fragments is placed, and scheduling barriers keep the
    // compiler from regrouping them, so the matrix pipe (32 clocks per MFMA) stays busy while
    // the vector ALU decodes.  Raw codes for the second half of a stage are read from LDS
    // during the first k-step.
    constexpr int G = WM + WN;                 // fragments per k-step
    constexpr int P = (WM * WN) / 2;           // MFMA pairs per k-step
    uint4 ca[2][WM], cw[2][WN];
    uint32_t sa[2][WM], sw[2][WN];
    half8 fa[2][WM], fw[2][WN];
    const uint8_t* st = lds;
    auto read_raw = [&](int u) {
#pragma unroll
        for (int i = 0; i < WM; ++i) {
            ca[u][i] = *reinterpret_cast<const uint4*>(st + rd_ac[i] + 16u * ((2 * u + h) ^ sw_a[i]));
            sa[u][i] = *reinterpret_cast<const uint16_t*>(st + rd_as[i] + 4 * u);
        }
#pragma unroll
        for (int j = 0; j < WN; ++j) {
            cw[u][j] = *reinterpret_cast<const uint4*>(st + rd_wc[j] + 16u * ((2 * u + h) ^ sw_w[j]));
            sw[u][j] = *reinterpret_cast<const uint16_t*>(st + rd_ws[j] + 4 * u);
        }
    };
    auto decode_frag = [&](int gidx, int x) {   // fragment gidx of k-step x (0..7) into slot x & 1
        const int u = x >> 2, t = x & 3, d = x & 1;
        if (gidx < WM) {
            const uint4 c4 = ca[u][gidx];
            const uint32_t c = t == 0 ? c4.x : t == 1 ? c4.y : t == 2 ? c4.z : c4.w;
            fa[d][gidx] = decode8(c, scale_pair((t < 2) ? (sa[u][gidx] & 0xFFu) : (sa[u][gidx] >> 8)));
        } else {
            const int j = gidx - WM;
            const uint4 c4 = cw[u][j];
            const uint32_t c = t == 0 ? c4.x : t == 1 ? c4.y : t == 2 ? c4.z : c4.w;
            fw[d][j] = decode8(c, scale_pair((t < 2) ? (sw[u][j] & 0xFFu) : (sw[u][j] >> 8)));
        }
    };

    // One stage: wait for its copies, open it with a barrier, start the copies two stages ahead,
    // then NSTEPS k-steps (8, or 4 for the half stage that ends an odd multiple of 64).
    int buf = 0;
    auto run_stage = [&](int s, auto nsteps_tag) {
        constexpr int NSTEPS = decltype(nsteps_tag)::value;
        // vector-memory operations retire in issue order: at most NDMA outstanding means
        // everything older than the youngest stage has landed
        if (s + 1 < nstage) wait_vmcnt<C::NDMA>();
        else wait_vmcnt<0>();
        wg_barrier();
        if (s + 2 < nstage) issue(s + 2, buf >= 1 ? buf - 1 : 2);     // (buf + 2) % 3
        st = lds + buf * C::STAGE_BYTES;
        read_raw(0);
#pragma unroll
        for (int gidx = 0; gidx < G; ++gidx) decode_frag(gidx, 0);
        if (NSTEPS > 4) read_raw(1);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int x = 0; x < NSTEPS; ++x) {
#pragma unroll
            for (int p = 0; p < P; ++p) {
                if (x + 1 < NSTEPS) {
#pragma unroll
                    for (int gidx = (p * G) / P; gidx < ((p + 1) * G) / P; ++gidx) decode_frag(gidx, x + 1);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int q = 2 * p; q < 2 * p + 2; ++q) {
                    const int i = q / WN, j = q % WN;
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fa[x & 1][i], fw[x & 1][j], acc[i][j], 0, 0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        buf = buf == 2 ? 0 : buf + 1;
    };

    if (nstage > 0) issue(0, 0);
    if (nstage > 1) issue(1, 1);
    const int nfull = nbk >> 3;
    for (int s = 0; s < nfull; ++s) run_stage(s, std::integral_constant<int, 8>{});
    if (has_half) run_stage(nfull, std::integral_constant<int, 4>{});

    const int m0 = wg_m0 + wrow0, n0 = wg_n0 + wcol0;
    store_tile<WM, WN>(acc, m0, n0, r, h, M, N, alpha, y, ldy);
}

template <int WM, int WN, typename OutT>
arcq_status launch_staged(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* w_codes,
                          const uint8_t* w_scales, int M, int N, int nbk, float alpha, OutT* y, int64_t ldy,
                          hipStream_t stream) {
    using C = StagedCfg<WM, WN>;
    auto kern = gemm_staged_kernel<WM, WN, OutT>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
    if (e != hipSuccess) return fail(ARCQ_HIP_ERROR, "hipFuncSetAttribute(LDS=%d): %s", C::LDS_BYTES, hipGetErrorString(e));
    const int tiles_m = (M + C::BM - 1) / C::BM, tiles_n = (N + C::BN - 1) / C::BN;
    hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(256), C::LDS_BYTES, stream, a_codes, a_scales, w_codes,
                       w_scales, M, N, nbk, alpha, y, ldy, tiles_m, tiles_n);
    return check_launch("gemm_staged_kernel");
}

template <typename OutT>
arcq_status launch_typed(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* w_codes,
                         const uint8_t* w_scales, int64_t M, int64_t N, int64_t Kp, float alpha, OutT* y,
                         int64_t ldy, hipStream_t stream) {
    const int nbk = (int)(Kp >> 4);
    const bool offsets_fit = (uint64_t)M * (uint64_t)nbk * 8 < 0xFFFF0000ull && (uint64_t)N * (uint64_t)nbk * 8 < 0xFFFF0000ull;
    const bool aligned16 = ((reinterpret_cast<uintptr_t>(a_codes) | reinterpret_cast<uintptr_t>(w_codes)) & 15) == 0 &&
                           ((reinterpret_cast<uintptr_t>(a_scales) | reinterpret_cast<uintptr_t>(w_scales)) & 3) == 0;
    if ((nbk & 3) == 0 && nbk >= 8 && offsets_fit && aligned16) {
        // big tiles when they still give every CU work; otherwise smaller ones
        const int64_t t256 = ((M + 255) / 256) * ((N + 255) / 256);
        if (t256 >= 256)
            return launch_staged<4, 4>(a_codes, a_scales, w_codes, w_scales, (int)M, (int)N, nbk, alpha, y, ldy, stream);
        const int64_t t128x256 = ((M + 127) / 128) * ((N + 255) / 256);
        if (t128x256 >= 192)
            return launch_staged<2, 4>(a_codes, a_scales, w_codes, w_scales, (int)M, (int)N, nbk, alpha, y, ldy, stream);
        return launch_staged<2, 2>(a_codes, a_scales, w_codes, w_scales, (int)M, (int)N, nbk, alpha, y, ldy, stream);
    }
    dim3 grid((unsigned)((N + 127) / 128), (unsigned)((M + 127) / 128));
    hipLaunchKernelGGL(gemm_direct_kernel<OutT>, grid, dim3(256), 0, stream, a_codes, a_scales, w_codes, w_scales,
                       (int)M, (int)N, nbk, alpha, y, ldy);
    return check_launch("gemm_direct_kernel");
}

}  // namespace

size_t gemm_workspace_bytes(int64_t, int64_t, int64_t) { return 0; }

arcq_status launch_gemm(const uint8_t* a_codes, const uint8_t* a_scales,
                        const uint8_t* w_codes, const uint8_t* w_scales,
                        int64_t M, int64_t N, int64_t Kp, float alpha,
                        void* y, int y_dtype, int64_t ldy,
                        void*, size_t, hipStream_t stream) {
    if (y_dtype == ARCQ_DTYPE_F16)
        return launch_typed<_Float16>(a_codes, a_scales, w_codes, w_scales, M, N, Kp, alpha,
                                      static_cast<_Float16*>(y), ldy, stream);
    return launch_typed<float>(a_codes, a_scales, w_codes, w_scales, M, N, Kp, alpha, static_cast<float*>(y), ldy, stream);
}

}  // namespace arcq
