// GEMM over K' = K + S for MXFP4 operands (Section 3.2 "Unified GEMM Execution", eq. (2), in the MXFP4
// variant of the format): y[m,n] = sum_b 2^(sa[m,b]-127) 2^(sw[n,b]-127) sum_{i<32} qa[m,32b+i] qw[n,32b+i].
//
// This is the format gfx950 multiplies natively: v_mfma_scale_f32_32x32x64_f8f6f4 takes 32 E2M1 values
// per lane and operand (one 16-byte register quad = exactly one MX block of one row) plus one E8M0
// scale byte per lane and operand; a lane holds row (lane % 32) and the k range 32 (lane / 32) .. + 31
// of the 64-k step (checked on the GPU with random codes and scales against this formula).  Products
// of E2M1 values and powers of two are exact; the only rounding is the fp32 accumulation.
// No decode: packed operands go global -> LDS -> registers -> matrix core unchanged.
#include "gemm_epilogue.h"
#include "internal.h"
#include "gemm_decode.h"
#include "lds_dma.h"

#include <type_traits>

namespace arcq {

namespace {

typedef int int8v __attribute__((ext_vector_type(8)));

__device__ __forceinline__ float16v mfma_mx(const uint4& a, const uint4& b, const float16v& c, int sa, int sb, int t) {
    const int8v va = {(int)a.x, (int)a.y, (int)a.z, (int)a.w, 0, 0, 0, 0};
    const int8v vb = {(int)b.x, (int)b.y, (int)b.z, (int)b.w, 0, 0, 0, 0};
    // cbsz = blgp = 4: both operands FP4; the scale of a lane is byte 2t of its scale register
    return t == 0 ? __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(va, vb, c, 4, 4, 0, sa, 0, sb)
                  : __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(va, vb, c, 4, 4, 2, sa, 2, sb);
}

// Staged kernel for K' % 128 == 0.  A unit is 256 k: per row 128 bytes of codes (eight 16-byte pieces =
// eight MX blocks) and 8 scale bytes, so that a copy instruction asks for whole 128-byte cache lines
// (8 lanes per row): the texture-address unit of a CU spends about 34 cycles on a copy that touches
// sixteen 64-byte segments and 17.5 on one that touches eight full lines (measured), and with FP4
// MFMAs the copies of a 256 x 256 tile would otherwise take as long as its arithmetic.  Units travel
// global -> LDS with global_load_lds through a ring of NUNIT buffers (2 for the 256 x 256 tile: 2 x 68 KB),
// one barrier per unit.  LDS layout of one unit: A codes [BM][128] | W codes [BN][128] | A scales [BM][8] |
// W scales [BN][8] (regions padded to whole workgroup-wide copies).  The eight pieces of a row are stored
// XOR-swizzled with (row >> 1) & 7: the LDS serves a 16-byte read of 16 consecutive lanes per clock from
// 64 banks, rows are 128 bytes apart, so 16 consecutive rows must land on 16 different 16-byte bank groups
// (measured: a swizzle with a period of 8 rows spent 44 % of its LDS cycles on bank conflicts); applied by
// choosing which global piece a lane fetches (a wave-wide copy writes lane l to base + 16 l).
// When K' is an odd multiple of 128 the last unit is half a unit: its copies re-fetch the first half
// for the missing second half (never used, in bounds).
// BF16: the same skeleton for plain bf16 operands (the comparison kernel arcq_ref_gemm_bf16): a row of a unit is 128
// bytes = 64 bf16 values, there are no scale bytes, and a k-step is one v_mfma_f32_32x32x16_bf16.
template <int WM, int WN, int GM, int GN, bool BF16 = false>
struct MxCfg {
    static constexpr int BM = 32 * WM * GM, BN = 32 * WN * GN;
    static constexpr int NT = 64 * GM * GN;
    static constexpr int NA = (BM * 8 + NT - 1) / NT, NW = (BN * 8 + NT - 1) / NT;       // 16-byte pieces of codes
    static constexpr int NAS = BF16 ? 0 : (BM * 2 + NT - 1) / NT, NWS = BF16 ? 0 : (BN * 2 + NT - 1) / NT;     // 4-byte words of scales
    static constexpr int NDMA = NA + NW + NAS + NWS;
    static constexpr int A_CODES = 0;
    static constexpr int W_CODES = NA * NT * 16;
    static constexpr int A_SCALES = W_CODES + NW * NT * 16;
    static constexpr int W_SCALES = A_SCALES + NAS * NT * 4;
    static constexpr int UNIT_BYTES = W_SCALES + NWS * NT * 4;
    static constexpr int NUNIT = (160 * 1024) / UNIT_BYTES >= 3 ? 3 : 2;
    static constexpr int LDS_BYTES = NUNIT * UNIT_BYTES;
    static_assert(NDMA * (NUNIT - 1) < 64, "the counted wait needs the copies of NUNIT - 1 units to fit the counter");
};

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

//
// REG: the same tiles, LDS layout and schedule for shapes the direct-to-LDS copies do not serve: any number of
// blocks per row (K' a multiple of 32 only: rows of scale bytes then start at odd addresses) and operands at the
// interface's minimum alignment.  A thread fetches its pieces of unit u+2 into registers with ordinary loads
// (declared with the alignment the interface guarantees), all at once right after the barrier that opens unit u+1,
// and writes them to LDS just before the barrier that opens their unit; blocks past the end of a row become zero
// codes (a scale word that would reach past the end is fetched from further left and shifted), so every unit is a
// whole unit.
template <int WM, int WN, int GM, int GN, typename OutT, bool BF16 = false, bool REG = false>
__global__ __launch_bounds__(64 * GM * GN) void mx_gemm_staged_kernel(
    const uint8_t* __restrict__ a_codes, const uint8_t* __restrict__ a_scales,
    const uint8_t* __restrict__ w_codes, const uint8_t* __restrict__ w_scales, int M, int N, int nb,
    OutT* __restrict__ y, int64_t ldy, int tiles_m, int tiles_n, int splits, int64_t split_stride) {
    using C = MxCfg<WM, WN, GM, GN, BF16>;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

    // workgroup -> tile: a contiguous run of the tile sequence per XCD, column-major groups of 8 tile rows
    // With splits > 1 the units of the reduction dimension are cut into `splits` runs: workgroup
    // blockIdx.x = split * num_tiles + tile accumulates its run and stores an fp32 partial tile at
    // y + split * split_stride (a reduction kernel adds the partial results in index order).
    const int num_tiles = tiles_m * tiles_n;
    const int split = (int)blockIdx.x / num_tiles;
    int pid = (int)blockIdx.x - split * num_tiles;
    if ((num_tiles & 7) == 0) pid = (pid & 7) * (num_tiles >> 3) + (pid >> 3);
    constexpr int GROUP = 8;
    const int group_size = GROUP * tiles_n;
    const int g = pid / group_size;
    const int first_m = g * GROUP;
    const int gm = min(GROUP, tiles_m - first_m);
    const int in_g = pid - g * group_size;
    const int tile_m = first_m + in_g % gm;
    const int tile_n = in_g / gm;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane & 31, h = lane >> 5;
    const int wg_m0 = tile_m * C::BM, wg_n0 = tile_n * C::BN;
    const int wrow0 = (wave / GN) * (32 * WM), wcol0 = (wave % GN) * (32 * WN);

    const bool has_half = !REG && (nb & 7) != 0;            // nb % 8 == 4
    const int nunit = REG ? (nb + 7) >> 3 : (nb >> 3) + (has_half ? 1 : 0);

    // ---- copies: thread -> (row, piece) of a workgroup-wide copy; 8 lanes fetch one row's 128 bytes
    const uint32_t cpitch = (uint32_t)nb * 16u, spitch = (uint32_t)nb;
    const uint32_t lp = (uint32_t)((tid & 7) ^ ((tid >> 4) & 7));               // global piece this lane fetches
    const int crow = tid >> 3, srow = tid >> 1;
    const uint32_t wave_slot = __builtin_amdgcn_readfirstlane((uint32_t)(tid & ~63));
    const uint32_t lds0 = lds_address(lds);
    auto issue_one = [&](int d, int unit, int buf) {
        const uint32_t base = lds0 + buf * C::UNIT_BYTES;
        constexpr int NA = C::NA, NW = C::NW, NAS = C::NAS, NT = C::NT;
        const bool half = has_half && unit == nunit - 1;
        const uint32_t oc = (uint32_t)unit * 128u + (half ? (lp & 3u) : lp) * 16u;
        const uint32_t os = (uint32_t)unit * 8u + (half ? 0u : (uint32_t)(tid & 1) * 4u);
        // rows past the edge of the operand re-read its last row (never stored)
        if (d < NA) {
            const uint32_t row = (uint32_t)min(wg_m0 + d * (NT / 8) + crow, M - 1);
            dma16(a_codes, row * cpitch + oc, base + C::A_CODES + 16u * (d * NT + wave_slot));
        } else if (d < NA + NW) {
            const int p = d - NA;
            const uint32_t row = (uint32_t)min(wg_n0 + p * (NT / 8) + crow, N - 1);
            dma16(w_codes, row * cpitch + oc, base + C::W_CODES + 16u * (p * NT + wave_slot));
        } else if (d < NA + NW + NAS) {
            const int p = d - NA - NW;
            const uint32_t row = (uint32_t)min(wg_m0 + p * (NT / 2) + srow, M - 1);
            dma4(a_scales, row * spitch + os, base + C::A_SCALES + 4u * (p * NT + wave_slot));
        } else {
            const int p = d - NA - NW - NAS;
            const uint32_t row = (uint32_t)min(wg_n0 + p * (NT / 2) + srow, N - 1);
            dma4(w_scales, row * spitch + os, base + C::W_SCALES + 4u * (p * NT + wave_slot));
        }
    };

    // ---- REG: the same pieces through registers (piece d of a thread lands where copy d puts it); needs nb >= 4
    constexpr int NCP = C::NA + C::NW, NSP = C::NAS + C::NWS;
    uint4 rc[REG ? NCP : 1];
    uint32_t rs[REG && NSP > 0 ? NSP : 1];
    auto reg_issue = [&](int unit) {
        const uint32_t oc = 16u * (uint32_t)min(8 * unit + (int)lp, nb - 1);
#pragma unroll
        for (int d = 0; d < NCP; ++d) {
            const bool is_a = d < C::NA;
            const int p = is_a ? d : d - C::NA;
            const uint32_t row = (uint32_t)(is_a ? min(wg_m0 + p * (C::NT / 8) + crow, M - 1) : min(wg_n0 + p * (C::NT / 8) + crow, N - 1));
            rc[d] = load16_a4((is_a ? a_codes : w_codes) + (size_t)(row * cpitch + oc));
        }
        const uint32_t os = (uint32_t)min(8 * unit + 4 * (tid & 1), nb - 4);
#pragma unroll
        for (int d = 0; d < NSP; ++d) {
            const bool is_a = d < C::NAS;
            const int p = is_a ? d : d - C::NAS;
            const uint32_t row = (uint32_t)(is_a ? min(wg_m0 + p * (C::NT / 2) + srow, M - 1) : min(wg_n0 + p * (C::NT / 2) + srow, N - 1));
            rs[d] = load4_a1((is_a ? a_scales : w_scales) + (size_t)(row * spitch + os));
        }
    };
    auto reg_commit = [&](int unit, int buf) {
        uint8_t* st = lds + buf * C::UNIT_BYTES;
        const bool ok = 8 * unit + (int)lp < nb;       // this piece's block exists
#pragma unroll
        for (int d = 0; d < NCP; ++d) {
            const uint4 v = uint4{ok ? rc[d].x : 0u, ok ? rc[d].y : 0u, ok ? rc[d].z : 0u, ok ? rc[d].w : 0u};
            const int at = d < C::NA ? C::A_CODES + 16 * (d * C::NT + tid) : C::W_CODES + 16 * ((d - C::NA) * C::NT + tid);
            *reinterpret_cast<uint4*>(st + at) = v;
        }
        const int sb0 = 8 * unit + 4 * (tid & 1);       // this word: blocks sb0 .. sb0 + 3
        const int skip = sb0 - min(sb0, nb - 4);        // bytes of the fetched word that belong to earlier blocks
#pragma unroll
        for (int d = 0; d < NSP; ++d) {
            const uint32_t word = skip >= 4 ? 0u : rs[d] >> (8 * skip);
            const int at = d < C::NAS ? C::A_SCALES + 4 * (d * C::NT + tid) : C::W_SCALES + 4 * ((d - C::NAS) * C::NT + tid);
            *reinterpret_cast<uint32_t*>(st + at) = word;
        }
    };

    // ---- LDS read offsets of this lane: k-step t of a unit takes piece 2t + h of its rows, stored at
    // physical position (2t + h) ^ ((row >> 1) & 7), which only depends on r because the other terms of the
    // row are multiples of 32
    const uint32_t swz = (uint32_t)(r >> 1) & 7u;
    const uint32_t rd_a = C::A_CODES + (wrow0 + r) * 128, rd_w = C::W_CODES + (wcol0 + r) * 128;
    const uint32_t rd_as = C::A_SCALES + (wrow0 + r) * 8, rd_ws = C::W_SCALES + (wcol0 + r) * 8;
    uint32_t pc[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) pc[t] = 16u * ((uint32_t)(2 * t + h) ^ swz);

    float16v acc[WM][WN];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    uint4 fa[2][WM], fw[2][WN];             // fragments of the k-step being computed and of the next one
    uint2 sa[WM], sw[WN], sa_n[WM], sw_n[WN];   // scale bytes of the unit (.x: blocks 0-3, .y: 4-7), shifted so
                                                // that bytes 0 and 2 of each word are this lane's
    auto read_codes = [&](int slot, int t, const uint8_t* st) {
#pragma unroll
        for (int i = 0; i < WM; ++i) fa[slot][i] = *reinterpret_cast<const uint4*>(st + rd_a + i * 4096 + pc[t]);
#pragma unroll
        for (int j = 0; j < WN; ++j) fw[slot][j] = *reinterpret_cast<const uint4*>(st + rd_w + j * 4096 + pc[t]);
    };
    auto read_scales = [&](const uint8_t* st, uint2 (&da)[WM], uint2 (&dw)[WN]) {
        if (BF16) return;
#pragma unroll
        for (int i = 0; i < WM; ++i) {
            const uint2 v = *reinterpret_cast<const uint2*>(st + rd_as + i * 256);
            da[i] = make_uint2(v.x >> (8 * h), v.y >> (8 * h));
        }
#pragma unroll
        for (int j = 0; j < WN; ++j) {
            const uint2 v = *reinterpret_cast<const uint2*>(st + rd_ws + j * 256);
            dw[j] = make_uint2(v.x >> (8 * h), v.y >> (8 * h));
        }
    };

    // ---- pipeline, scheduled by hand (one wave per SIMD: nothing else hides a stall).  A unit is
    // NSTEPS WM WN MFMAs.  The copies of unit u + NUNIT - 1 are issued one at a time between the first
    // MFMAs of unit u (its buffer was last read in unit u-1, which every wave left before the barrier
    // inside unit u-1); the fragments of k-step t+1 are read while k-step t is computed; the barrier
    // that opens unit u+1 and the reads of its first fragments sit before the last half k-step.
    constexpr int NM = WM * WN;               // MFMAs per k-step
    constexpr int DIST = C::NUNIT - 1;
    int buf = 0;
    auto run_unit = [&](int u, auto nsteps_tag) {
        constexpr int NSTEPS = decltype(nsteps_tag)::value;
        constexpr int LAST_Q = NSTEPS * NM - NM / 2;
        constexpr int COMMIT_Q = LAST_Q - NM / 2;     // REG: the pieces of unit u+1 go to LDS half a k-step before its barrier
        const uint8_t* st = lds + buf * C::UNIT_BYTES;
        const int buf1 = buf + 1 == C::NUNIT ? 0 : buf + 1, bufd = buf == 0 ? C::NUNIT - 1 : buf - 1;
        const int fetch = min(u + DIST, nunit - 1);
#pragma unroll
        for (int t = 0; t < NSTEPS; ++t) {
            if (t + 1 < NSTEPS) {
                read_codes((t + 1) & 1, t + 1, st);
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int i = 0; i < WM; ++i)
#pragma unroll
                for (int j = 0; j < WN; ++j) {
                    const int q = t * NM + i * WN + j;
                    if (REG && q == COMMIT_Q) {
                        reg_commit(min(u + 1, nunit - 1), buf1);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    if (q == LAST_Q) {
                        // unit u+1 must have landed: the copies of the DIST - 1 later units are younger
                        // (REG: this wave's LDS writes of unit u+1 must have completed)
                        if constexpr (REG) wait_lgkmcnt0();
                        else wait_vmcnt<(DIST - 1) * C::NDMA>();
                        wg_barrier();
                        read_codes(0, 0, lds + buf1 * C::UNIT_BYTES);
                        read_scales(lds + buf1 * C::UNIT_BYTES, sa_n, sw_n);
                        if constexpr (REG) reg_issue(min(u + 2, nunit - 1));
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    // weights as the row operand: see store_tile_swapped
                    if constexpr (BF16)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fw[t & 1][j]),
                                                                            __builtin_bit_cast(bf16x8, fa[t & 1][i]), acc[i][j], 0, 0, 0);
                    else
                        acc[i][j] = mfma_mx(fw[t & 1][j], fa[t & 1][i], acc[i][j], (int)(t < 2 ? sw[j].x : sw[j].y),
                                            (int)(t < 2 ? sa[i].x : sa[i].y), t & 1);
                    __builtin_amdgcn_sched_barrier(0);
                    if (!REG && NSTEPS == 4 && q < C::NDMA) {
                        issue_one(q, fetch, bufd);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
        }
        if constexpr (!BF16) {
#pragma unroll
            for (int i = 0; i < WM; ++i) sa[i] = sa_n[i];
#pragma unroll
            for (int j = 0; j < WN; ++j) sw[j] = sw_n[j];
        }
        buf = buf1;
    };
    static_assert(C::NDMA <= 3 * NM, "copies are issued during the first three k-steps of a unit");

    // this workgroup's run of units [u0, u1); copies past the run fetch units the run never uses (in bounds)
    const int u0 = (int)((int64_t)split * nunit / splits), u1 = (int)((int64_t)(split + 1) * nunit / splits);
    if constexpr (REG) {
        reg_issue(u0);
        reg_commit(u0, 0);
        reg_issue(min(u0 + 1, nunit - 1));
        wait_lgkmcnt0();
    } else {
#pragma unroll
        for (int u = 0; u < DIST; ++u)
#pragma unroll
            for (int d = 0; d < C::NDMA; ++d) issue_one(d, min(u0 + u, nunit - 1), u);
        wait_vmcnt<(DIST - 1) * C::NDMA>();
    }
    wg_barrier();
    read_codes(0, 0, lds);
    read_scales(lds, sa, sw);
    const int nfull = REG ? nunit : nb >> 3;
    for (int u = u0; u < min(u1, nfull); ++u) run_unit(u, std::integral_constant<int, 4>{});
    if (has_half && u1 == nunit) run_unit(nfull, std::integral_constant<int, 2>{});
    wait_vmcnt<0>();                            // no copy may still be in flight when the LDS is released

    const int m0 = wg_m0 + wrow0, n0 = wg_n0 + wcol0;
    if constexpr (std::is_same<OutT, _Float16>::value) {
        static_assert(epilogue_lds_bytes(WN) * GM * GN <= C::LDS_BYTES, "one epilogue region per wave must fit the operand ring");
        wg_barrier();                           // every wave has read its last operands: the ring is free
        const bool vec_ok = (ldy & 7) == 0 && (reinterpret_cast<uintptr_t>(y) & 15) == 0;
        store_tile_f16_via_lds<WM, WN>(acc, lds + wave * epilogue_lds_bytes(WN), m0, n0, lane, M, N, 1.0f, y, ldy, vec_ok);
    } else {
        const bool vec_ok = (ldy & 3) == 0 && (reinterpret_cast<uintptr_t>(y) & 15) == 0;
        store_tile_swapped<WM, WN>(acc, m0, n0, r, h, M, N, 1.0f, y + (int64_t)split * split_stride, ldy, vec_ok);
    }
}

// Fallback for any K' (multiple of 32) and any alignment the API admits: operands straight from global
// memory, one 64 x 64 tile per wave.  A k-step is two blocks; when the block count is odd the upper
// half of the lanes contributes zero codes in the last step.
template <typename OutT>
__global__ __launch_bounds__(256) void mx_gemm_direct_kernel(
    const uint8_t* __restrict__ a_codes, const uint8_t* __restrict__ a_scales,
    const uint8_t* __restrict__ w_codes, const uint8_t* __restrict__ w_scales, int M, int N, int nb,
    OutT* __restrict__ y, int64_t ldy) {
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));   // scalar: see gemm.hip
    const int r = lane & 31, h = lane >> 5;
    const int m0 = blockIdx.y * 128 + (wave >> 1) * 64, n0 = blockIdx.x * 128 + (wave & 1) * 64;
    const int64_t cpitch = (int64_t)nb * 16, spitch = nb;
    const uint8_t *ac[2], *as[2], *wc[2], *ws[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int m = min(m0 + 32 * i + r, M - 1), n = min(n0 + 32 * i + r, N - 1);
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
    for (int b0 = 0; b0 < nb; b0 += 2) {
        const int b = b0 + h;
        const bool ok = b < nb;
        const int bb = ok ? b : 0;
        uint4 fa[2], fw[2];
        int sa[2], sw[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            // 4-byte loads: the API only guarantees 4-byte alignment of the codes on this path
            const uint32_t* pa = reinterpret_cast<const uint32_t*>(ac[i] + 16 * (int64_t)bb);
            const uint32_t* pw = reinterpret_cast<const uint32_t*>(wc[i] + 16 * (int64_t)bb);
            fa[i] = ok ? make_uint4(pa[0], pa[1], pa[2], pa[3]) : make_uint4(0, 0, 0, 0);
            fw[i] = ok ? make_uint4(pw[0], pw[1], pw[2], pw[3]) : make_uint4(0, 0, 0, 0);
            sa[i] = ok ? as[i][bb] : 127;
            sw[i] = ok ? ws[i][bb] : 127;
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) acc[i][j] = mfma_mx(fw[j], fa[i], acc[i][j], sw[j], sa[i], 0);
    }
    store_tile_swapped<2, 2>(acc, m0, n0, r, h, M, N, 1.0f, y, ldy, false);
}

// Weight-streaming kernel for M <= 64 (decode, batched decode), any K' (a multiple of 32): bound by
// reading the packed weights once (17/32 byte per weight).  v_mfma_scale_f32_16x16x128_f8f6f4: lane
// (i = lane % 16, q = lane / 16) supplies the 32 values of block 4c + q of row i for the 128-k chunk c,
// with that block's scale byte.  A lane loads 16 bytes of codes per row and chunk (a wave: 16 rows x 64
// contiguous bytes) and its block's scale byte.  Blocks past the end of a row (a last chunk of one to three
// blocks) count as zero codes.  Loads are declared with the alignment the interface guarantees (codes 4 bytes,
// scale bytes 1); global memory serves them in one request at any address.  MT tiles of 16 activation rows share every weight fragment; the WAVES
// waves of a workgroup split K' and add their partial tiles through LDS.  Everything is loaded straight
// into registers; latency is hidden by occupancy.
typedef float float4v __attribute__((ext_vector_type(4)));

// GRP: whole chunks are taken four at a time (512 k) with the scale bytes of the four chunks fetched by ONE
// four-byte load per lane: the four lanes of a row read 16 contiguous bytes, and a 4 x 4 byte transpose
// across the four lane groups (two lane-swap instructions and two byte permutes with per-lane selectors)
// leaves every lane with the scale bytes of its block for the four chunks, which the matrix instruction
// picks with its byte selector.  The address unit of a CU spends about two cycles per (row, 64-byte
// segment) an instruction touches, so a four-byte scale load per chunk costs as much as the code load.
typedef unsigned uint2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t transpose_scale_bytes(uint32_t s, uint32_t sel_half, uint32_t sel_byte) {
    const uint2v x = __builtin_amdgcn_permlane32_swap(s, s, false, false);     // (q, q ^ 2): own and partner word
    const uint32_t pair = __builtin_amdgcn_perm(x[1], x[0], sel_half);         // bytes {0,1} or {2,3} of chunks (q & 1), (q & 1) + 2
    const uint2v t = __builtin_amdgcn_permlane16_swap(pair, pair, false, false);   // (q, q ^ 1)
    return __builtin_amdgcn_perm(t[1], t[0], sel_byte);                        // byte q of chunks 0, 1, 2, 3
}

template <int MT, int NT, int WAVES, int U, bool GRP, typename OutT>
__global__ __launch_bounds__(WAVES * 64) void mx_gemm_skinny_kernel(
    const uint8_t* __restrict__ a_codes, const uint8_t* __restrict__ a_scales,
    const uint8_t* __restrict__ w_codes, const uint8_t* __restrict__ w_scales, int M, int N, int nb,
    OutT* __restrict__ y, int64_t ldy) {
    __shared__ float red[WAVES][MT * NT][4][64];
    static_assert(sizeof(float) * WAVES * MT * NT * 256 <= 64 * 1024, "partial tiles must fit the static LDS limit");
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));   // scalar: see gemm.hip
    const int i = lane & 15, q = lane >> 4;
    const int n0 = blockIdx.x * (16 * NT);
    const int64_t cpitch = (int64_t)nb * 16, spitch = nb;
    const int nchunk = (nb + 3) >> 2;                            // the last chunk may hold fewer than four blocks

    const uint8_t *ac[MT], *as[MT];
#pragma unroll
    for (int r = 0; r < MT; ++r) {
        const int m = min(16 * r + i, M - 1);                    // rows past M repeat row M-1 and are not stored
        ac[r] = a_codes + (int64_t)m * cpitch;
        as[r] = a_scales + (int64_t)m * spitch;
    }
    const uint8_t *wc[NT], *ws[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int n = min(n0 + 16 * t + i, N - 1);
        wc[t] = w_codes + n * cpitch;
        ws[t] = w_scales + n * spitch;
    }
    float4v acc[MT][NT];
#pragma unroll
    for (int r = 0; r < MT; ++r)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[r][t] = float4v{0.f, 0.f, 0.f, 0.f};

    int cbase = 0, first_wave = 0;              // first chunk and first wave of the chunk-at-a-time loop
    if constexpr (GRP) {
        const int ngroup = nb >> 4;             // groups of four whole chunks
        const uint32_t sel_half = q < 2 ? 0x05040100u : 0x07060302u;
        const uint32_t sel_byte = (q & 1) ? 0x07030501u : 0x06020400u;
        for (int g = wave; g < ngroup; g += WAVES) {
            uint4 ca[4][MT], cw[4][NT];
            uint32_t sa[MT], sw[NT];
            // the scale bytes are needed first (their transpose precedes the first matrix instruction) and loads retire
            // in issue order: asked for first, they do not make the wave wait for the whole group's codes; the
            // scheduling barrier keeps every load of the group ahead of its first use
#pragma unroll
            for (int r = 0; r < MT; ++r) sa[r] = load4_a1(as[r] + 16 * (int64_t)g + 4 * q);
#pragma unroll
            for (int t = 0; t < NT; ++t) sw[t] = load4_a1(ws[t] + 16 * (int64_t)g + 4 * q);
#pragma unroll
            for (int m = 0; m < 4; ++m) {
#pragma unroll
                for (int r = 0; r < MT; ++r) ca[m][r] = load16_a4(ac[r] + 256 * (int64_t)g + 64 * m + 16 * q);
#pragma unroll
                for (int t = 0; t < NT; ++t) cw[m][t] = load16_a4(wc[t] + 256 * (int64_t)g + 64 * m + 16 * q);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int r = 0; r < MT; ++r) sa[r] = transpose_scale_bytes(sa[r], sel_half, sel_byte);
#pragma unroll
            for (int t = 0; t < NT; ++t) sw[t] = transpose_scale_bytes(sw[t], sel_half, sel_byte);
            auto step = [&](auto mtag) {
                constexpr int m = decltype(mtag)::value;
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    const int8v vw = {(int)cw[m][t].x, (int)cw[m][t].y, (int)cw[m][t].z, (int)cw[m][t].w, 0, 0, 0, 0};
#pragma unroll
                    for (int r = 0; r < MT; ++r) {
                        const int8v va = {(int)ca[m][r].x, (int)ca[m][r].y, (int)ca[m][r].z, (int)ca[m][r].w, 0, 0, 0, 0};
                        // byte m of the scale registers belongs to chunk m
                        acc[r][t] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(va, vw, acc[r][t], 4, 4, m, (int)sa[r], m, (int)sw[t]);
                    }
                }
            };
            step(std::integral_constant<int, 0>{});
            step(std::integral_constant<int, 1>{});
            step(std::integral_constant<int, 2>{});
            step(std::integral_constant<int, 3>{});
        }
        cbase = 4 * ngroup;
        first_wave = ngroup % WAVES;            // the waves that took one group less come first
    }
    for (int c0 = cbase + ((wave - first_wave + WAVES) % WAVES) * U; c0 < nchunk; c0 += WAVES * U) {
        uint4 ca[U][MT], cw[U][NT];
        uint32_t sa[U][MT], sw[U][NT];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            // a block past the end of the row: the lane re-reads block 0 and the block counts as zero (codes zeroed where
            // they are used, not here: a select behind a load would make the wave wait for it at once)
            const int64_t b = 4 * (c0 + u) + q < nb ? 4 * (c0 + u) + q : 0;
#pragma unroll
            for (int r = 0; r < MT; ++r) {
                ca[u][r] = load16_a4(ac[r] + 16 * b);
                sa[u][r] = as[r][b];
            }
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                cw[u][t] = load16_a4(wc[t] + 16 * b);
                sw[u][t] = ws[t][b];
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bool ok = 4 * (c0 + u) + q < nb;
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const int8v vw = {ok ? (int)cw[u][t].x : 0, ok ? (int)cw[u][t].y : 0, ok ? (int)cw[u][t].z : 0, ok ? (int)cw[u][t].w : 0, 0, 0, 0, 0};
#pragma unroll
                for (int r = 0; r < MT; ++r) {
                    const int8v va = {ok ? (int)ca[u][r].x : 0, ok ? (int)ca[u][r].y : 0, ok ? (int)ca[u][r].z : 0, ok ? (int)ca[u][r].w : 0, 0, 0, 0, 0};
                    // activations as the 16-row operand: lane holds column n = lane % 16, register e row 4 (lane / 16) + e
                    acc[r][t] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(va, vw, acc[r][t], 4, 4, 0, (int)sa[u][r], 0, (int)sw[u][t]);
                }
            }
        }
    }
#pragma unroll
    for (int r = 0; r < MT; ++r)
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int e = 0; e < 4; ++e) red[wave][r * NT + t][e][lane] = acc[r][t][e];
    __syncthreads();
    for (int idx = threadIdx.x; idx < MT * NT * 4 * 64; idx += WAVES * 64) {
        const int rt = idx >> 8, e = (idx >> 6) & 3, l = idx & 63;
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < WAVES; ++w) sum += red[w][rt][e][l];
        const int m = 16 * (rt / NT) + 4 * (l >> 4) + e, n = n0 + 16 * (rt % NT) + (l & 15);
        if (m < M && n < N) store_out(y + (int64_t)m * ldy + n, sum);
    }
}

template <int MT, int NT, int WAVES, int U, typename OutT>
arcq_status launch_mx_skinny(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* w_codes,
                             const uint8_t* w_scales, int M, int N, int nb, OutT* y, int64_t ldy, hipStream_t stream) {
    hipLaunchKernelGGL((mx_gemm_skinny_kernel<MT, NT, WAVES, U, (MT <= 4), OutT>), dim3((N + 16 * NT - 1) / (16 * NT)),
                       dim3(WAVES * 64), 0, stream, a_codes, a_scales, w_codes, w_scales, M, N, nb, y, ldy);
    return check_launch("mx_gemm_skinny_kernel");
}

template <int WM, int WN, int GM, int GN, typename OutT, bool BF16 = false, bool REG = false>
arcq_status launch_mx_staged(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* w_codes,
                             const uint8_t* w_scales, int M, int N, int nb, OutT* y, int64_t ldy, hipStream_t stream,
                             int splits = 1, float* partial = nullptr) {
    using C = MxCfg<WM, WN, GM, GN, BF16>;
    const int tiles_m = (M + C::BM - 1) / C::BM, tiles_n = (N + C::BN - 1) / C::BN;
    if (splits > 1) {
        // fp32 partial results [splits, M, N] in the workspace, then one pass that adds them
        auto kern = mx_gemm_staged_kernel<WM, WN, GM, GN, float, BF16, REG>;
        static std::atomic<uint64_t> lds_raised{0};
        if (arcq_status st = raise_lds_limit(reinterpret_cast<const void*>(kern), lds_raised)) return st;
        hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n * splits), dim3(C::NT), C::LDS_BYTES, stream, a_codes, a_scales,
                           w_codes, w_scales, M, N, nb, partial, (int64_t)N, tiles_m, tiles_n, splits, (int64_t)M * N);
        if (arcq_status st = check_launch("mx_gemm_staged_kernel (split K)")) return st;
        return launch_splitk_reduce(partial, splits, M, N, 1.0f, y, std::is_same<OutT, _Float16>::value ? ARCQ_DTYPE_F16 : ARCQ_DTYPE_F32,
                                    ldy, stream);
    }
    auto kern = mx_gemm_staged_kernel<WM, WN, GM, GN, OutT, BF16, REG>;
    static std::atomic<uint64_t> lds_raised{0};
    if (arcq_status st = raise_lds_limit(reinterpret_cast<const void*>(kern), lds_raised)) return st;
    hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(C::NT), C::LDS_BYTES, stream, a_codes, a_scales, w_codes,
                       w_scales, M, N, nb, y, ldy, tiles_m, tiles_n, 1, (int64_t)0);
    return check_launch("mx_gemm_staged_kernel");
}

// Number of runs the units of the reduction dimension are cut into when the caller provides a workspace (1: no
// split): a function of the shape alone.  Only the 128 x 128 tiles of few-tile problems split; the cost, in
// microseconds, is rounds of workgroups over the 256 CUs times the units of a run at about 0.65 us a unit, plus,
// when split, the write and read of the fp32 partial results at about 3 TB/s and 5.5 us for the shorter runs'
// pipeline fill and the second launch (fitted to measurements over N = 2048 .. 8192, K' = 4352 .. 29696).
// Shapes the weight-streaming kernel serves: up to 64 rows while the tiled kernels (with K' split across workgroups
// where tiles are few) are not faster already.  Measured over N = 1024 .. 28672, K' = 4352 .. 28928: up to 16 rows
// below 2 * 10^8 weights (10^8 when K' >= 16384: 5120 x 27904 27.5 us streamed, 19 us tiled); 17 to 32 rows below
// 1.2 * 10^8 (5120 x 27904: 40 us streamed, 19 us tiled); 33 to 64
// rows below 2.2 * 10^7 and fewer than 8192 weight rows (6144 x 4352: 13.2 against 11.2 us).  On the FP4 instruction a 128- or 256-row tile costs no
// more than a 16-row one, so the tiled kernels win as soon as their tiles fill the chip.
static bool mx_streaming_shape(int64_t M, int64_t N, int64_t Kp) {
    const int64_t weights = N * Kp;
    if (M <= 16) return weights < 200000000 && !(Kp >= 16384 && weights >= 100000000);
    return M <= 32 ? weights < 120000000 : M <= 64 && N < 8192 && weights < 22000000;
}

int mx_split_k(int64_t M, int64_t N, int64_t Kp) {
    const int64_t nb = Kp >> 5;
    const bool streaming = mx_streaming_shape(M, N, Kp);
    if (streaming || nb < 8) return 1;
    if (((M + 255) / 256) * ((N + 255) / 256) >= 256 || ((M + 127) / 128) * ((N + 255) / 256) >= 192) return 1;
    const int64_t tiles = ((M + 127) / 128) * ((N + 127) / 128);
    if (tiles > 256 && ((M + 191) / 192) * ((N + 127) / 128) <= 256) return 1;      // one round of 192 x 128 tiles
    const int64_t nunit = (nb + 7) >> 3;
    const int64_t max_splits = std::min<int64_t>(8, nunit / 2);
    int best = 1;
    double best_cost = 0.0;
    for (int64_t sp = 1; sp <= max_splits; ++sp) {
        const double rounds = (double)((tiles * sp + 255) / 256);
        double cost = rounds * (double)((nunit + sp - 1) / sp) * 0.65;
        if (sp > 1) cost += (double)sp * (double)M * (double)N * 8.0 / 3.0e6 + 5.5;
        if (sp == 1 || cost < best_cost) {
            best = (int)sp;
            best_cost = cost;
        }
    }
    return best;
}

template <typename OutT>
arcq_status launch_mx_typed(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* w_codes,
                            const uint8_t* w_scales, int64_t M, int64_t N, int64_t Kp, OutT* y, int64_t ldy,
                            float* workspace, hipStream_t stream) {
    const int nb = (int)(Kp >> 5);
    const bool offsets_fit = (uint64_t)M * (uint64_t)nb * 16 < 0xFFFF0000ull && (uint64_t)N * (uint64_t)nb * 16 < 0xFFFF0000ull;
    const bool aligned16 = ((reinterpret_cast<uintptr_t>(a_codes) | reinterpret_cast<uintptr_t>(w_codes)) & 15) == 0 &&
                           ((reinterpret_cast<uintptr_t>(a_scales) | reinterpret_cast<uintptr_t>(w_scales)) & 3) == 0;
    // up to 64 rows the tiled kernels only win where they can split K' across workgroups, which needs the workspace
    const bool streaming = mx_streaming_shape(M, N, Kp) || (M <= 64 && workspace == nullptr && mx_split_k(M, N, Kp) > 1);
    if (streaming) {
        const int64_t tiles = (N + 15) / 16;
#define ARCQ_MX_SKINNY(MT_, NT_, W_, U_) \
    return launch_mx_skinny<MT_, NT_, W_, U_>(a_codes, a_scales, w_codes, w_scales, (int)M, (int)N, nb, y, ldy, stream)
        // weight tiles per wave: as few as keep the launch at one workgroup per compute unit, up to four (measured with
        // weights from HBM, 32 rows: 640 tiles 14.8 us with three per wave against 21.7 with one, 896 tiles 10.4 us
        // with four against 13.0 with two, 320 tiles over K' = 8448 11.2 us with two against 15.2 with one)
        if (M <= 16) {
            if (tiles >= 769) ARCQ_MX_SKINNY(1, 4, 8, 1);
            if (tiles >= 513) ARCQ_MX_SKINNY(1, 3, 8, 1);
            if (tiles >= 257) ARCQ_MX_SKINNY(1, 2, 8, 2);
            ARCQ_MX_SKINNY(1, 1, 8, 2);
        }
        if (M <= 32) {
            if (tiles >= 769) ARCQ_MX_SKINNY(2, 4, 8, 1);
            if (tiles >= 513) ARCQ_MX_SKINNY(2, 3, 8, 1);
            if (tiles >= 257) ARCQ_MX_SKINNY(2, 2, 8, 1);
            ARCQ_MX_SKINNY(2, 1, 8, 2);
        }
        if (tiles >= 257) ARCQ_MX_SKINNY(4, 2, 8, 1);
        ARCQ_MX_SKINNY(4, 1, 8, 1);
#undef ARCQ_MX_SKINNY
    }
    // Tiles of 256 weight rows by 256, 192 or 128 activation rows when there is work for them: workgroups run in rounds
    // of one per compute unit, a round lasts as long as one tile, and a tile's time follows the bytes it copies per
    // unit, 136 (rows of A + rows of W): the height that minimises rounds x (height + 256) wins (e.g. 1024 x 10240:
    // 240 tiles of 192 rows in one round instead of 320 of 128 rows in two).
    const int64_t tn256 = (N + 255) / 256, t128x256 = ((M + 127) / 128) * tn256;
    auto tile_cost = [&](int64_t bm) { return ((((M + bm - 1) / bm) * tn256 + 255) / 256) * (bm + 256); };
    const int tile_rows = t128x256 < 192 ? 0
                          : tile_cost(256) <= tile_cost(192) && tile_cost(256) <= tile_cost(128) ? 256
                          : tile_cost(192) <= tile_cost(128) ? 192 : 128;
    if ((nb & 3) == 0 && offsets_fit && aligned16) {
        if (tile_rows == 256)
            return launch_mx_staged<4, 4, 2, 2>(a_codes, a_scales, w_codes, w_scales, (int)M, (int)N, nb, y, ldy, stream);
        if (tile_rows == 192)
            return launch_mx_staged<3, 4, 2, 2>(a_codes, a_scales, w_codes, w_scales, (int)M, (int)N, nb, y, ldy, stream);
        if (tile_rows == 128)
            return launch_mx_staged<2, 4, 2, 2>(a_codes, a_scales, w_codes, w_scales, (int)M, (int)N, nb, y, ldy, stream);
        // more than 256 tiles of 128 x 128 but at most 256 of 192 x 128: one round of the taller tile instead of two
        // workgroups on some compute units (512 x 10240 over K' = 8448: 48 -> 37 us; 1024 x 5120 over 27904: 144 -> 105 us)
        {
            const int64_t t128 = ((M + 127) / 128) * ((N + 127) / 128), t192 = ((M + 191) / 192) * ((N + 127) / 128);
            if (t128 > 256 && t192 <= 256)
                return launch_mx_staged<3, 2, 2, 2>(a_codes, a_scales, w_codes, w_scales, (int)M, (int)N, nb, y, ldy, stream);
        }
        return launch_mx_staged<2, 2, 2, 2>(a_codes, a_scales, w_codes, w_scales, (int)M, (int)N, nb, y, ldy, stream,
                                            workspace ? mx_split_k(M, N, Kp) : 1, workspace);
    }
    if (nb >= 8 && offsets_fit) {
        // any K' that is a multiple of 32, operands at their minimum alignment: units through registers
        if (tile_rows == 256)
            return launch_mx_staged<4, 4, 2, 2, OutT, false, true>(a_codes, a_scales, w_codes, w_scales, (int)M, (int)N, nb, y, ldy, stream);
        if (tile_rows == 192)
            return launch_mx_staged<3, 4, 2, 2, OutT, false, true>(a_codes, a_scales, w_codes, w_scales, (int)M, (int)N, nb, y, ldy, stream);
        if (tile_rows == 128)
            return launch_mx_staged<2, 4, 2, 2, OutT, false, true>(a_codes, a_scales, w_codes, w_scales, (int)M, (int)N, nb, y, ldy, stream);
        return launch_mx_staged<2, 2, 2, 2, OutT, false, true>(a_codes, a_scales, w_codes, w_scales, (int)M, (int)N, nb, y, ldy, stream,
                                                               workspace ? mx_split_k(M, N, Kp) : 1, workspace);
    }
    dim3 grid((unsigned)((N + 127) / 128), (unsigned)((M + 127) / 128));
    hipLaunchKernelGGL(mx_gemm_direct_kernel<OutT>, grid, dim3(256), 0, stream, a_codes, a_scales, w_codes, w_scales,
                       (int)M, (int)N, nb, y, ldy);
    return check_launch("mx_gemm_direct_kernel");
}

}  // namespace

// Comparison kernel: y = x w^T for plain bf16 operands (x [M, K], w [N, K], row-major, 16-byte aligned, K % 32 == 0)
// on the tiled skeleton above, fp32 accumulation, fp16 output.  nb counts 16-byte pieces of a row.
arcq_status launch_ref_gemm_bf16(const void* x, const void* w, int64_t M, int64_t N, int64_t K, _Float16* y, int64_t ldy,
                                 hipStream_t stream) {
    const uint8_t* a = static_cast<const uint8_t*>(x);
    const uint8_t* b = static_cast<const uint8_t*>(w);
    const int nb = (int)(K >> 3);
    const int64_t t256 = ((M + 255) / 256) * ((N + 255) / 256);
    if (t256 >= 256) return launch_mx_staged<4, 4, 2, 2, _Float16, true>(a, nullptr, b, nullptr, (int)M, (int)N, nb, y, ldy, stream);
    const int64_t t128x256 = ((M + 127) / 128) * ((N + 255) / 256);
    if (t128x256 >= 192) return launch_mx_staged<2, 4, 2, 2, _Float16, true>(a, nullptr, b, nullptr, (int)M, (int)N, nb, y, ldy, stream);
    return launch_mx_staged<2, 2, 2, 2, _Float16, true>(a, nullptr, b, nullptr, (int)M, (int)N, nb, y, ldy, stream);
}

size_t mx_gemm_workspace_bytes(int64_t M, int64_t N, int64_t Kp) {
    const int splits = mx_split_k(M, N, Kp);
    return splits > 1 ? (size_t)splits * (size_t)M * (size_t)N * sizeof(float) : 0;
}

arcq_status launch_mx_gemm(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* w_codes,
                           const uint8_t* w_scales, int64_t M, int64_t N, int64_t Kp, void* y, int y_dtype, int64_t ldy,
                           void* workspace, hipStream_t stream) {
    float* ws = static_cast<float*>(workspace);
    if (y_dtype == ARCQ_DTYPE_F16)
        return launch_mx_typed<_Float16>(a_codes, a_scales, w_codes, w_scales, M, N, Kp, static_cast<_Float16*>(y), ldy, ws, stream);
    return launch_mx_typed<float>(a_codes, a_scales, w_codes, w_scales, M, N, Kp, static_cast<float*>(y), ldy, ws, stream);
}

}  // namespace arcq
