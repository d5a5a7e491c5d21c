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
#include "gemm_decode.h"
#include "gemm_epilogue.h"
#include "lds_dma.h"

#include <hip/hip_fp16.h>

#include <algorithm>
#include <atomic>
#include <type_traits>

namespace arcq {

namespace {

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
// Staged kernel for K' % 64 == 0.  Workgroup = GM x GN waves; each wave owns WM x WN MFMA tiles
// of 32 x 32, so the workgroup tile is BM x BN = 32 WM GM x 32 WN GN.  With 4 waves (one per
// SIMD, up to 256 accumulator registers) the hand-made schedule has to hide every stall.  8 waves
// (two per SIMD, 128 accumulator registers each, <2,4,4,2> / <4,2,2,4>) let the hardware interleave
// two waves but decode every fragment for more waves; on the large shapes they measure the same as
// 2 x 2 waves to within 1 % (the loop is limited by the vector and matrix work itself, not by
// stalls: removing the waits or the barrier from a timing build gains 2 %), so 2 x 2 waves are
// dispatched there; on a 128 x 256 tile, 2 x 4 waves of 64 x 64 are 5 % faster than 2 x 2 of 64 x 128.
//
// A stage is 128 k (8 blocks): per row 64 bytes of codes and 8 scale bytes, kept PACKED in
// LDS (4.5 bits per element) and decoded in registers after the LDS read.  Stages travel
// global -> LDS with global_load_lds (no register staging) through a ring of NSTAGE (3 to 5)
// buffers: the loads of stage s + NSTAGE - 1 are issued right after the barrier that opens stage s,
// so they have NSTAGE - 1 stage times to land, and one barrier per stage suffices (passing the
// barrier of stage s means every wave has finished stage s-1, whose buffer the new stage reuses).
//
// LDS layout of one stage (bytes):  A codes [BM][64] | W codes [BN][64] | A scales [BM][8] |
// W scales [BN][8].  The four 16-byte pieces of a row's codes are stored XOR-swizzled with
// (row >> 2) & 3: the LDS serves a 16-byte read of 16 consecutive lanes per clock from 64 banks, rows
// are 64 bytes apart, so 16 consecutive rows must land on 16 different 16-byte bank groups (measured: a
// swizzle with a period of 8 rows spent half of the LDS-active cycles on bank conflicts).
// A wave-wide DMA instruction writes lane l to (uniform base) + 16 l, so the swizzle is applied
// by choosing which global piece each lane fetches.
template <int WM, int WN, int GM, int GN>
struct StagedCfg {
    static constexpr int BM = 32 * WM * GM, BN = 32 * WN * GN;
    static constexpr int NT = 64 * GM * GN;              // threads
    // DMA instructions per thread per stage: 16-byte pieces of codes, 4-byte pieces of scales.  A copy
    // always involves the whole workgroup; when an operand has fewer pieces than threads the surplus
    // lanes re-fetch its last rows into padding behind the region (so every wave issues the same
    // number of copies, which the counted waits rely on).
    static constexpr int NA = (BM * 4 + NT - 1) / NT, NW = (BN * 4 + NT - 1) / NT;
    static constexpr int NAS = (BM * 2 + NT - 1) / NT, NWS = (BN * 2 + NT - 1) / NT;
    static constexpr int NDMA = NA + NW + NAS + NWS;
    static constexpr int A_CODES = 0;
    static constexpr int W_CODES = NA * NT * 16;
    static constexpr int A_SCALES = W_CODES + NW * NT * 16;
    static constexpr int W_SCALES = A_SCALES + NAS * NT * 4;
    static constexpr int STAGE_BYTES = W_SCALES + NWS * NT * 4;
    // Ring depth: a stage is fetched NSTAGE - 1 stages before it is computed (3 measured as good as 5).
    static constexpr int NSTAGE = 3;
    static constexpr int DIST = NSTAGE - 1;
    static constexpr int LDS_BYTES = NSTAGE * STAGE_BYTES;
};

//
// REG: the same tiles, LDS layout and compute schedule for operands the direct-to-LDS copies cannot serve: any
// number of blocks per row (K' a multiple of 16 only) and rows that are only 8-byte aligned.  A thread fetches
// its pieces of a stage into registers (loads declared with the alignment the interface guarantees, 8 bytes
// for codes and 1 for scale bytes), all at once right after the barrier that opens
// stage s+1, and writes them to LDS seven k-steps later, just before the barrier that opens the stage they
// belong to, with blocks past the end of the row replaced by zeros: every stage is then a whole stage.
template <int WM, int WN, int GM, int GN, typename OutT, bool REG = false>
__global__ __launch_bounds__(64 * GM * GN) void gemm_staged_kernel(
    const uint8_t* __restrict__ a_codes, const uint8_t* __restrict__ a_scales,
    const uint8_t* __restrict__ w_codes, const uint8_t* __restrict__ w_scales, int M, int N,
    int nbk, float alpha, OutT* __restrict__ y, int64_t ldy, int tiles_m, int tiles_n, int splits,
    int64_t split_stride) {
    using C = StagedCfg<WM, WN, GM, GN>;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

    // ---- workgroup -> tile.  Workgroups are dealt round-robin to the 8 XCDs (each with its
    // own L2); give every XCD a contiguous run of the tile sequence, and walk the sequence in
    // column-major groups of 8 tile rows so that concurrently running tiles share A and W rows.
    // With splits > 1 the reduction dimension is cut into `splits` runs of whole stages: workgroup
    // blockIdx.x = split * num_tiles + tile accumulates its run and stores an fp32 partial tile at
    // y + split * split_stride (a reduction kernel adds the partial results).
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

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int r = lane & 31, h = lane >> 5;
    const int wg_m0 = tile_m * C::BM, wg_n0 = tile_n * C::BN;
    const int wrow0 = (wave / GN) * (32 * WM);       // first row of this wave inside the A tile
    const int wcol0 = (wave % GN) * (32 * WN);       // first row of this wave inside the W tile

    // ---- DMA source offsets of this thread (bytes from the operand base)
    // When K' is an odd multiple of 64 the last stage is half a stage (4 blocks): the lanes that
    // would fetch its missing second half re-fetch the first half instead (never used), which
    // keeps every access inside the operand.  `half` selects those adjusted offsets.
    const bool has_half = !REG && (nbk & 7) != 0;
    const int nstage = REG ? (nbk + 7) >> 3 : (nbk >> 3) + (has_half ? 1 : 0);   // of the whole reduction dimension
    const int per_split = nstage / splits, extra = nstage % splits;
    const int s_begin = split * per_split + min(split, extra);  // this workgroup's stages [s_begin, s_end)
    const int s_end = s_begin + per_split + (split < extra ? 1 : 0);
    // Offsets are recomputed per copy (a handful of ALU operations per stage) rather than kept
    // in registers: the accumulators leave this kernel 256 registers and it needs most of them.
    // (s & 3) and the row swizzle repeat every 64 slots, so one value serves every copy
    const uint32_t lp_ = (uint32_t)((tid & 3) ^ ((tid >> 4) & 3));
    const uint32_t adj_c0 = lp_ * 16u, adj_c1 = (lp_ & 1u) * 16u, adj_s = (uint32_t)(tid & 1) * 4u;
    const int crow = tid >> 2, srow = tid >> 1; // row of this thread inside a copy of NT/4 code rows / NT/2 scale rows
    const uint32_t cpitch32 = (uint32_t)nbk * 8u, spitch32 = (uint32_t)nbk;
    // lane l of a DMA writes slot wave_slot + l; made a scalar once so that the LDS destinations
    // of all copies are computed on the scalar unit
    const uint32_t wave_slot = __builtin_amdgcn_readfirstlane((uint32_t)(tid & ~63));
    const uint32_t lds0 = lds_address(lds);
    // DMA instruction d (0 .. NDMA-1) of a stage: A code pieces, W code pieces, A scales, W scales.
    auto issue_one = [&](int d, int stage, int buf) {
        const uint32_t base = lds0 + buf * C::STAGE_BYTES;
        const bool half = has_half && stage == nstage - 1;
        const uint32_t oc = (uint32_t)stage * 64u + (half ? adj_c1 : adj_c0);
        const uint32_t os = (uint32_t)stage * 8u + (half ? 0u : adj_s);
        constexpr int NA = C::NA, NW = C::NW, NAS = C::NAS, NT = C::NT;
        // rows past the edge of the operand re-read its last row (never stored)
        if (d < NA) {
            const uint32_t row = (uint32_t)min(wg_m0 + d * (NT / 4) + crow, M - 1);
            dma16(a_codes, row * cpitch32 + oc, base + C::A_CODES + 16u * (d * NT + wave_slot));
        } else if (d < NA + NW) {
            const int p = d - NA;
            const uint32_t row = (uint32_t)min(wg_n0 + p * (NT / 4) + crow, N - 1);
            dma16(w_codes, row * cpitch32 + oc, base + C::W_CODES + 16u * (p * NT + wave_slot));
        } else if (d < NA + NW + NAS) {
            const int p = d - NA - NW;
            const uint32_t row = (uint32_t)min(wg_m0 + p * (NT / 2) + srow, M - 1);
            dma4(a_scales, row * spitch32 + os, base + C::A_SCALES + 4u * (p * NT + wave_slot));
        } else {
            const int p = d - NA - NW - NAS;
            const uint32_t row = (uint32_t)min(wg_n0 + p * (NT / 2) + srow, N - 1);
            dma4(w_scales, row * spitch32 + os, base + C::W_SCALES + 4u * (p * NT + wave_slot));
        }
    };
    auto issue_all = [&](int stage, int buf) {
#pragma unroll
        for (int d = 0; d < C::NDMA; ++d) issue_one(d, stage, buf);
    };
    // ---- REG: the same pieces through registers (piece d of a thread lands where DMA instruction d puts it).
    // A piece that would reach past the end of its row is fetched from further left, so that it ends with the row
    // (needs nbk >= 4), and shifted into place when it is written to LDS.
    constexpr int NCP = C::NA + C::NW, NSP = C::NAS + C::NWS;
    uint4 rc[REG ? NCP : 1];
    uint32_t rs[REG ? NSP : 1];
    auto reg_issue = [&](int stage) {
        const uint32_t oc = 8u * (uint32_t)min(8 * stage + 2 * (int)lp_, nbk - 2);
#pragma unroll
        for (int d = 0; d < NCP; ++d) {
            const bool is_a = d < C::NA;
            const int p = is_a ? d : d - C::NA;
            const uint32_t row = (uint32_t)(is_a ? min(wg_m0 + p * (C::NT / 4) + crow, M - 1) : min(wg_n0 + p * (C::NT / 4) + crow, N - 1));
            rc[d] = load16_a8((is_a ? a_codes : w_codes) + (size_t)(row * cpitch32 + oc));
        }
        const uint32_t os = (uint32_t)min(8 * stage + 4 * (tid & 1), nbk - 4);
#pragma unroll
        for (int d = 0; d < NSP; ++d) {
            const bool is_a = d < C::NAS;
            const int p = is_a ? d : d - C::NAS;
            const uint32_t row = (uint32_t)(is_a ? min(wg_m0 + p * (C::NT / 2) + srow, M - 1) : min(wg_n0 + p * (C::NT / 2) + srow, N - 1));
            rs[d] = load4_a1((is_a ? a_scales : w_scales) + (size_t)(row * spitch32 + os));
        }
    };
    auto reg_commit = [&](int stage, int buf) {
        uint8_t* st = lds + buf * C::STAGE_BYTES;
        const int b0 = 8 * stage + 2 * (int)lp_;       // this piece: blocks b0, b0 + 1
        const bool both = b0 + 1 < nbk, one = b0 < nbk;
#pragma unroll
        for (int d = 0; d < NCP; ++d) {
            const uint4 v = uint4{both ? rc[d].x : one ? rc[d].z : 0u, both ? rc[d].y : one ? rc[d].w : 0u, both ? rc[d].z : 0u, both ? rc[d].w : 0u};
            const int at = d < C::NA ? C::A_CODES + 16 * (d * C::NT + tid) : C::W_CODES + 16 * ((d - C::NA) * C::NT + tid);
            *reinterpret_cast<uint4*>(st + at) = v;
        }
        const int sb0 = 8 * stage + 4 * (tid & 1);      // this word: blocks sb0 .. sb0 + 3
        const int skip = sb0 - min(sb0, nbk - 4);       // bytes of the fetched word that belong to earlier blocks
#pragma unroll
        for (int d = 0; d < NSP; ++d) {
            const uint32_t word = skip >= 4 ? 0u : rs[d] >> (8 * skip);
            const int at = d < C::NAS ? C::A_SCALES + 4 * (d * C::NT + tid) : C::W_SCALES + 4 * ((d - C::NAS) * C::NT + tid);
            *reinterpret_cast<uint32_t*>(st + at) = word;
        }
    };

    // ---- LDS read offsets of this lane inside a stage.  Fragment i of a wave is 32 rows (2048
    // bytes of codes, 256 of scales) further on, a constant folded into the instruction; the
    // swizzle (row >> 2) & 3 only depends on lane % 32 because the other terms are multiples of 32.
    const uint32_t swz = (uint32_t)(r >> 2) & 3u;
    const uint32_t rd_a = C::A_CODES + (wrow0 + r) * 64, rd_w = C::W_CODES + (wcol0 + r) * 64;
    // a lane reads the whole 4-byte scale word of its row and 64-k half stage (both halves of the wave read
    // the same word, which the LDS broadcasts; two-byte reads of its two halves count as a bank conflict)
    // and picks its two bytes with the byte selector of the permute
    const uint32_t rd_as = C::A_SCALES + (wrow0 + r) * 8, rd_ws = C::W_SCALES + (wcol0 + r) * 8;
    const uint32_t scale_sel = h ? 0x0C030C02u : 0x0C010C00u;
    const uint32_t piece0 = 16u * ((uint32_t)h ^ swz), piece1 = 16u * ((2u + (uint32_t)h) ^ swz);

    float16v acc[WM][WN];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    // ---- per-stage compute, software-pipelined by hand (with one or two waves per SIMD little else
    // hides a stall, so every wait is placed where its data has long been ready).
    // A k-step (one block, 16 k) is WM*WN MFMAs fed by WM + WN fragments of 8 fp16 per lane.
    // While the MFMAs of step x run, the fragments of step x+1 are decoded: after every group of
    // MFMAs (see MPG) the decode of its share of the fragments is placed, and scheduling barriers keep
    // the compiler from regrouping them, so the matrix pipe stays busy while the vector ALU decodes.
    // The pipeline runs ACROSS stages: the barrier that opens stage s+1 sits before step 6 of
    // stage s; step 6 reads the first raw codes of stage s+1 from LDS and step 7 decodes its
    // first fragments.  The copies for stage s + NSTAGE - 1 are issued two per k-step during steps 0-5 of
    // stage s (its buffer was last read in stage s-1, which every wave left before the barrier
    // that opened stage s), so no wave ever queues a burst of memory instructions.
    constexpr int G = WM + WN;                 // fragments per k-step
    // MFMAs per group: after every group the decode of G / P fragments is placed.  With few MFMAs per
    // fragment (2 x 2 fragments: nine vector instructions per MFMA) single MFMAs interleave best with the
    // vector work (a register-only model of this loop ran 10 % faster with singles than with pairs);
    // with 4 x 4 fragments pairs and singles measure the same in that model, and singles spill here.
    constexpr int MPG = (WM * WN >= 16) ? 2 : 1;
    constexpr int P = (WM * WN) / MPG;         // groups per k-step
    uint4 ca[2][WM], cw[2][WN];
    uint32_t sa[2][WM], sw[2][WN];
    half8 fa[2][WM], fw[2][WN];
    auto read_raw = [&](int u, const uint8_t* st) {
        const uint8_t* pa = st + rd_a + (u ? piece1 : piece0);
        const uint8_t* pw = st + rd_w + (u ? piece1 : piece0);
        const uint8_t* psa = st + rd_as + 4 * u;
        const uint8_t* psw = st + rd_ws + 4 * u;
#pragma unroll
        for (int i = 0; i < WM; ++i) {
            ca[u][i] = *reinterpret_cast<const uint4*>(pa + i * 2048);
            sa[u][i] = scale_halves(*reinterpret_cast<const uint32_t*>(psa + i * 256), scale_sel);
        }
#pragma unroll
        for (int j = 0; j < WN; ++j) {
            cw[u][j] = *reinterpret_cast<const uint4*>(pw + j * 2048);
            sw[u][j] = scale_halves(*reinterpret_cast<const uint32_t*>(psw + j * 256), scale_sel);
        }
    };
    auto decode_frag = [&](int gidx, int x) {   // fragment gidx of k-step x (0..7) into slot x & 1
        const int u = x >> 2, t = x & 3, d = x & 1;
        if (gidx < WM) {
            const uint4 c4 = ca[u][gidx];
            const uint32_t c = t == 0 ? c4.x : t == 1 ? c4.y : t == 2 ? c4.z : c4.w;
            fa[d][gidx] = decode8_half(c, sa[u][gidx], t >> 1);
        } else {
            const int j = gidx - WM;
            const uint4 c4 = cw[u][j];
            const uint32_t c = t == 0 ? c4.x : t == 1 ? c4.y : t == 2 ? c4.z : c4.w;
            fw[d][j] = decode8_half(c, sw[u][j], t >> 1);
        }
    };

    // The steady-state stage is free of branches (they would split the hand-made schedule):
    // past the end of K' it keeps issuing copies (of the last stage, into a free ring slot) and
    // keeps reading and decoding a "next" stage whose values are never used.
    int buf = 0;                                // ring slot of the stage being computed
    auto ring_next = [](int b) { return b == C::NSTAGE - 1 ? 0 : b + 1; };
    auto run_stage = [&](int s, auto nsteps_tag) {
        constexpr int NSTEPS = decltype(nsteps_tag)::value;
        constexpr bool FULL = NSTEPS == 8;      // a half stage is always the last one
        const uint8_t* st = lds + buf * C::STAGE_BYTES;
        // the copies issued during this stage go to the slot of the stage computed before this one
        const int buf1 = ring_next(buf), buf2 = buf == 0 ? C::NSTAGE - 1 : buf - 1;
        const int fetch = min(s + C::DIST, s_end - 1);
#pragma unroll
        for (int x = 0; x < NSTEPS; ++x) {
            if (x == 0 && FULL) read_raw(1, st);
            if (x == 6) {
                // stage s+1 must have landed: the copies of the DIST - 1 later stages are younger, and
                // everything older has retired once at most that many operations are outstanding
                // (REG: this wave's LDS writes of stage s+1 must have completed)
                if constexpr (REG) wait_lgkmcnt0();
                else wait_vmcnt<(C::DIST - 1) * C::NDMA>();
                wg_barrier();
                read_raw(0, lds + buf1 * C::STAGE_BYTES);
                if constexpr (REG) reg_issue(min(s + 2, s_end - 1));
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int p = 0; p < P; ++p) {
#pragma unroll
                for (int gidx = (p * G) / P; gidx < ((p + 1) * G) / P; ++gidx) {
                    if (x + 1 < NSTEPS) decode_frag(gidx, x + 1);
                    else if (FULL) decode_frag(gidx, 0);          // first step of stage s+1
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int q = MPG * p; q < MPG * p + MPG; ++q) {
                    const int i = q / WN, j = q % WN;
                    // weights as the row operand: see store_tile_swapped
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fw[x & 1][j], fa[x & 1][i], acc[i][j], 0, 0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
                if (!REG && FULL && x < 6) {    // copies of stage s + NSTAGE - 1, spread over steps 0..5
#pragma unroll
                    for (int d = 0; d < C::NDMA; ++d)
                        if ((d * 6) / C::NDMA == x && (d - (x * C::NDMA + 5) / 6) == p) issue_one(d, fetch, buf2);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            if constexpr (REG)
                if (x == 5) {                   // stage s+1, fetched since step 6 of the stage before
                    reg_commit(min(s + 1, s_end - 1), buf1);
                    __builtin_amdgcn_sched_barrier(0);
                }
        }
        buf = buf1;
    };

    if constexpr (REG) {
        reg_issue(s_begin);
        reg_commit(s_begin, 0);
        reg_issue(min(s_begin + 1, s_end - 1));
        wait_lgkmcnt0();
    } else {
#pragma unroll
        for (int d = 0; d < C::DIST; ++d) issue_all(min(s_begin + d, s_end - 1), d);
        wait_vmcnt<(C::DIST - 1) * C::NDMA>();
    }
    wg_barrier();
    read_raw(0, lds);
#pragma unroll
    for (int gidx = 0; gidx < G; ++gidx) decode_frag(gidx, 0);
    const int nfull = REG ? nstage : nbk >> 3;
    for (int s = s_begin; s < min(s_end, nfull); ++s) run_stage(s, std::integral_constant<int, 8>{});
    if (has_half && s_end == nstage) run_stage(nfull, std::integral_constant<int, 4>{});
    wait_vmcnt<0>();                            // no copy may still be in flight when the LDS is released

    const int m0 = wg_m0 + wrow0, n0 = wg_n0 + wcol0;
    if constexpr (std::is_same<OutT, _Float16>::value) {
        static_assert(epilogue_lds_bytes(WN) * GM * GN <= C::LDS_BYTES, "one epilogue region per wave must fit the operand ring");
        wg_barrier();                           // every wave has read its last operands: the ring is free
        const bool vec_ok = (ldy & 7) == 0 && (reinterpret_cast<uintptr_t>(y) & 15) == 0;
        store_tile_f16_via_lds<WM, WN>(acc, lds + wave * epilogue_lds_bytes(WN), m0, n0, lane, M, N, alpha,
                                       y + (int64_t)split * split_stride, ldy, vec_ok);
    } else {
        const bool vec_ok = (ldy & 3) == 0 && (reinterpret_cast<uintptr_t>(y) & 15) == 0;
        store_tile_swapped<WM, WN>(acc, m0, n0, r, h, M, N, alpha, y + (int64_t)split * split_stride, ldy, vec_ok);
    }
}

// ---------------------------------------------------------------------------------------------
// 128 x 256 tiles for problems with about one such tile per CU (2048 x 4096 has 256 of them).
// Same tile, stage ring and copies as gemm_staged_kernel<2, 2, 2, 4>, but the eight waves form a
// 2 (rows) x 2 (columns) x 2 (k) grid: a wave computes a 64 x 128 sub-tile (2 x 4 fragments: six fragment
// decodes per eight MFMAs instead of four per four, the decode being what keeps this tile shape from the
// matrix rate of the bigger ones) over one half of every stage: four of its eight k-steps, exactly the
// 16-byte piece of codes a lane reads per row and stage.  The two waves of a pair (w and w + 4) share a
// SIMD, so the matrix pipe still draws from two instruction streams; at the end they add their partial
// tiles through the LDS and each stores one of the two fragment rows.  Needs K' % 128 == 0.
template <typename OutT>
__global__ __launch_bounds__(512) void gemm_kpair_kernel(
    const uint8_t* __restrict__ a_codes, const uint8_t* __restrict__ a_scales,
    const uint8_t* __restrict__ w_codes, const uint8_t* __restrict__ w_scales, int M, int N,
    int nbk, float alpha, OutT* __restrict__ y, int64_t ldy, int tiles_m, int tiles_n) {
    using C = StagedCfg<2, 2, 2, 4>;
    constexpr int WM = 2, WN = 4;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

    // workgroup -> tile as in gemm_staged_kernel
    const int num_tiles = tiles_m * tiles_n;
    int pid = (int)blockIdx.x;
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
    const int kh = wave >> 2;                        // k half: k-steps 4 kh .. 4 kh + 3 of every stage
    const int wq = wave & 3;
    const int wg_m0 = tile_m * C::BM, wg_n0 = tile_n * C::BN;
    const int wrow0 = (wq >> 1) * 64;                // first row of this wave inside the A tile
    const int wcol0 = (wq & 1) * 128;                // first row of this wave inside the W tile
    const int nstage = nbk >> 3;

    // ---- copies (see gemm_staged_kernel)
    const uint32_t lp_ = (uint32_t)((tid & 3) ^ ((tid >> 4) & 3));
    const uint32_t adj_c0 = lp_ * 16u, adj_s = (uint32_t)(tid & 1) * 4u;
    const int crow = tid >> 2, srow = tid >> 1;
    const uint32_t cpitch32 = (uint32_t)nbk * 8u, spitch32 = (uint32_t)nbk;
    const uint32_t wave_slot = __builtin_amdgcn_readfirstlane((uint32_t)(tid & ~63));
    const uint32_t lds0 = lds_address(lds);
    auto issue_one = [&](int d, int stage, int buf) {
        const uint32_t base = lds0 + buf * C::STAGE_BYTES;
        const uint32_t oc = (uint32_t)stage * 64u + adj_c0;
        const uint32_t os = (uint32_t)stage * 8u + adj_s;
        constexpr int NA = C::NA, NW = C::NW, NAS = C::NAS, NT = C::NT;
        if (d < NA) {
            const uint32_t row = (uint32_t)min(wg_m0 + d * (NT / 4) + crow, M - 1);
            dma16(a_codes, row * cpitch32 + oc, base + C::A_CODES + 16u * (d * NT + wave_slot));
        } else if (d < NA + NW) {
            const int p = d - NA;
            const uint32_t row = (uint32_t)min(wg_n0 + p * (NT / 4) + crow, N - 1);
            dma16(w_codes, row * cpitch32 + oc, base + C::W_CODES + 16u * (p * NT + wave_slot));
        } else if (d < NA + NW + NAS) {
            const int p = d - NA - NW;
            const uint32_t row = (uint32_t)min(wg_m0 + p * (NT / 2) + srow, M - 1);
            dma4(a_scales, row * spitch32 + os, base + C::A_SCALES + 4u * (p * NT + wave_slot));
        } else {
            const int p = d - NA - NW - NAS;
            const uint32_t row = (uint32_t)min(wg_n0 + p * (NT / 2) + srow, N - 1);
            dma4(w_scales, row * spitch32 + os, base + C::W_SCALES + 4u * (p * NT + wave_slot));
        }
    };

    // ---- LDS read offsets: this wave's half of a stage is piece 2 kh + h of a row's codes and bytes
    // 4 kh + 2 h, 4 kh + 2 h + 1 of its scale bytes
    const uint32_t swz = (uint32_t)(r >> 2) & 3u;
    const uint32_t piece = 16u * ((uint32_t)(2 * kh + h) ^ swz);
    const uint32_t rd_a = C::A_CODES + (wrow0 + r) * 64 + piece, rd_w = C::W_CODES + (wcol0 + r) * 64 + piece;
    const uint32_t rd_as = C::A_SCALES + (wrow0 + r) * 8 + 4 * kh, rd_ws = C::W_SCALES + (wcol0 + r) * 8 + 4 * kh;
    const uint32_t scale_sel = h ? 0x0C030C02u : 0x0C010C00u;

    float16v acc[WM][WN];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    constexpr int G = WM + WN;                 // fragments per k-step
    constexpr int P = WM * WN;                 // MFMAs per k-step, one per group
    uint4 ca[WM], cw[WN];
    uint32_t sa[WM], sw[WN];
    half8 fa[2][WM], fw[2][WN];
    auto read_raw = [&](const uint8_t* st) {
#pragma unroll
        for (int i = 0; i < WM; ++i) {
            ca[i] = *reinterpret_cast<const uint4*>(st + rd_a + i * 2048);
            sa[i] = scale_halves(*reinterpret_cast<const uint32_t*>(st + rd_as + i * 256), scale_sel);
        }
#pragma unroll
        for (int j = 0; j < WN; ++j) {
            cw[j] = *reinterpret_cast<const uint4*>(st + rd_w + j * 2048);
            sw[j] = scale_halves(*reinterpret_cast<const uint32_t*>(st + rd_ws + j * 256), scale_sel);
        }
    };
    auto decode_frag = [&](int gidx, int t) {   // fragment gidx of this wave's k-step t (0..3) into slot t & 1
        const int d = t & 1;
        if (gidx < WM) {
            const uint4 c4 = ca[gidx];
            const uint32_t c = t == 0 ? c4.x : t == 1 ? c4.y : t == 2 ? c4.z : c4.w;
            fa[d][gidx] = decode8_half(c, sa[gidx], t >> 1);
        } else {
            const int j = gidx - WM;
            const uint4 c4 = cw[j];
            const uint32_t c = t == 0 ? c4.x : t == 1 ? c4.y : t == 2 ? c4.z : c4.w;
            fw[d][j] = decode8_half(c, sw[j], t >> 1);
        }
    };

    // One stage = four k-steps of this wave.  During step t the fragments of step t + 1 are decoded, one
    // group of fragments after every MFMA; the raw codes of the next stage are read at the start of step 3
    // (every fragment of this stage has been decoded by then) behind the barrier that opens that stage, and
    // step 3 decodes its first fragments.  The copies of stage s + DIST are issued during steps 0..2.
    int buf = 0;
    auto ring_next = [](int b) { return b == C::NSTAGE - 1 ? 0 : b + 1; };
    auto run_stage = [&](int s) {
        const int buf1 = ring_next(buf), buf2 = buf == 0 ? C::NSTAGE - 1 : buf - 1;
        const int fetch = min(s + C::DIST, nstage - 1);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            if (t == 3) {
                wait_vmcnt<(C::DIST - 1) * C::NDMA>();
                wg_barrier();
                read_raw(lds + buf1 * C::STAGE_BYTES);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int p = 0; p < P; ++p) {
#pragma unroll
                for (int gidx = (p * G) / P; gidx < ((p + 1) * G) / P; ++gidx) decode_frag(gidx, (t + 1) & 3);
                __builtin_amdgcn_sched_barrier(0);
                const int i = p / WN, j = p % WN;
                // weights as the row operand: see store_tile_swapped
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fw[t & 1][j], fa[t & 1][i], acc[i][j], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (t < 3) {
#pragma unroll
                    for (int d = 0; d < C::NDMA; ++d)
                        if ((d * 3) / C::NDMA == t && (d - (t * C::NDMA + 2) / 3) == p) issue_one(d, fetch, buf2);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
        buf = buf1;
    };

#pragma unroll
    for (int d = 0; d < C::DIST; ++d)
#pragma unroll
        for (int q = 0; q < C::NDMA; ++q) issue_one(q, min(d, nstage - 1), d);
    wait_vmcnt<(C::DIST - 1) * C::NDMA>();
    wg_barrier();
    read_raw(lds);
#pragma unroll
    for (int gidx = 0; gidx < G; ++gidx) decode_frag(gidx, 0);
    for (int s = 0; s < nstage; ++s) run_stage(s);
    wait_vmcnt<0>();                            // no copy may still be in flight when the LDS is released

    // ---- the pair adds its partial tiles: in two rounds (columns 0-63, 64-127 of the sub-tile) every wave
    // hands the partner the fragment row the partner will store, 16 bytes per lane and register group
    static_assert(8 * 8192 <= C::LDS_BYTES && 8 * epilogue_lds_bytes(WN) / 2 <= C::LDS_BYTES, "epilogue regions must fit the ring");
    float* xch = reinterpret_cast<float*>(lds);
    const int mine = kh, other = kh ^ 1;        // fragment row this wave stores / gives away
#pragma unroll
    for (int round = 0; round < 2; ++round) {
        wait_lgkmcnt0();                        // this wave's reads of the ring / of the previous round have returned
        wg_barrier();                           // ring (or the previous round's regions) no longer read
#pragma unroll
        for (int jj = 0; jj < 2; ++jj)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int j = 2 * round + jj;
                const float16v& src = other == 0 ? acc[0][j] : acc[1][j];
                *reinterpret_cast<float4*>(xch + wave * 2048 + ((jj * 4 + q) * 64 + lane) * 4) =
                    make_float4(src[4 * q], src[4 * q + 1], src[4 * q + 2], src[4 * q + 3]);
            }
        wait_lgkmcnt0();
        wg_barrier();
#pragma unroll
        for (int jj = 0; jj < 2; ++jj)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int j = 2 * round + jj;
                const float4 v = *reinterpret_cast<const float4*>(xch + (wave ^ 4) * 2048 + ((jj * 4 + q) * 64 + lane) * 4);
                if (mine == 0) {
                    acc[0][j][4 * q] += v.x; acc[0][j][4 * q + 1] += v.y; acc[0][j][4 * q + 2] += v.z; acc[0][j][4 * q + 3] += v.w;
                } else {
                    acc[1][j][4 * q] += v.x; acc[1][j][4 * q + 1] += v.y; acc[1][j][4 * q + 2] += v.z; acc[1][j][4 * q + 3] += v.w;
                }
            }
    }
    wait_lgkmcnt0();
    wg_barrier();                               // every wave has read its partner's last round
    const int m0 = wg_m0 + wrow0, n0 = wg_n0 + wcol0;
    if constexpr (std::is_same<OutT, _Float16>::value) {
        const bool vec_ok = (ldy & 7) == 0 && (reinterpret_cast<uintptr_t>(y) & 15) == 0;
        uint8_t* region = lds + wave * (epilogue_lds_bytes(WN) / 2);
        if (mine == 0)
            store_fragment_rows_f16_via_lds<WM, WN, 0, 1>(acc, region, m0, n0, lane, M, N, alpha, y, ldy, vec_ok);
        else
            store_fragment_rows_f16_via_lds<WM, WN, 1, 1>(acc, region, m0, n0, lane, M, N, alpha, y, ldy, vec_ok);
    } else {
        const bool vec_ok = (ldy & 3) == 0 && (reinterpret_cast<uintptr_t>(y) & 15) == 0;
        if (mine == 0)
            store_fragment_row_swapped<WM, WN, 0>(acc, m0, n0, r, h, M, N, alpha, y, ldy, vec_ok);
        else
            store_fragment_row_swapped<WM, WN, 1>(acc, m0, n0, r, h, M, N, alpha, y, ldy, vec_ok);
    }
}

// y = alpha * (sum of the `splits` fp32 partial results [M, N], added in index order).
template <typename OutT>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ part, int splits,
                                                            int64_t split_stride, int M, int N, float alpha,
                                                            OutT* __restrict__ y, int64_t ldy, int vec4) {
    const int64_t total = vec4 ? (int64_t)M * (N >> 2) : (int64_t)M * N;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * blockDim.x) {
        if (vec4) {
            const int64_t m = idx / (N >> 2), n = 4 * (idx % (N >> 2));
            float4 sum = *reinterpret_cast<const float4*>(part + m * N + n);
            for (int sp = 1; sp < splits; ++sp) {
                const float4 v = *reinterpret_cast<const float4*>(part + sp * split_stride + m * N + n);
                sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
            }
            store4(y + m * ldy + n, sum.x * alpha, sum.y * alpha, sum.z * alpha, sum.w * alpha);
        } else {
            const int64_t m = idx / N, n = idx % N;
            float sum = part[m * N + n];
            for (int sp = 1; sp < splits; ++sp) sum += part[sp * split_stride + m * N + n];
            store_out(y + m * ldy + n, sum * alpha);
        }
    }
}

template <int WM, int WN, int GM, int GN, bool REG = false, typename OutT>
arcq_status launch_staged(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* w_codes,
                          const uint8_t* w_scales, int M, int N, int nbk, float alpha, OutT* y, int64_t ldy,
                          hipStream_t stream, int splits = 1, float* partial = nullptr) {
    using C = StagedCfg<WM, WN, GM, GN>;
    const int tiles_m = (M + C::BM - 1) / C::BM, tiles_n = (N + C::BN - 1) / C::BN;
    if (splits > 1) {
        // fp32 partial results [splits, M, N] in the workspace, then one pass that adds them
        auto kern = gemm_staged_kernel<WM, WN, GM, GN, float, REG>;
        static std::atomic<uint64_t> lds_raised{0};
        if (arcq_status st = raise_lds_limit(reinterpret_cast<const void*>(kern), lds_raised)) return st;
        const int64_t stride = (int64_t)M * N;
        hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n * splits), dim3(C::NT), C::LDS_BYTES, stream, a_codes, a_scales,
                           w_codes, w_scales, M, N, nbk, 1.0f, partial, (int64_t)N, tiles_m, tiles_n, splits, stride);
        if (arcq_status st = check_launch("gemm_staged_kernel (split K)")) return st;
        return launch_splitk_reduce(partial, splits, M, N, alpha, y, std::is_same<OutT, _Float16>::value ? ARCQ_DTYPE_F16 : ARCQ_DTYPE_F32,
                                    ldy, stream);
    }
    auto kern = gemm_staged_kernel<WM, WN, GM, GN, OutT, REG>;
    static std::atomic<uint64_t> lds_raised{0};
    if (arcq_status st = raise_lds_limit(reinterpret_cast<const void*>(kern), lds_raised)) return st;
    hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(C::NT), C::LDS_BYTES, stream, a_codes, a_scales, w_codes,
                       w_scales, M, N, nbk, alpha, y, ldy, tiles_m, tiles_n, 1, (int64_t)0);
    return check_launch("gemm_staged_kernel");
}

// ---------------------------------------------------------------------------------------------
// Skinny kernel for M <= 128 (decode, batched decode, short prefill): bound by streaming the packed
// weights once from HBM (9/16 byte per weight), so the layout of the work follows the weight rows.
//
// v_mfma_f32_16x16x32_f16: lane (i = lane % 16, q = lane / 16) supplies 8 consecutive k of row i;
// the four lane groups q supply different octets.  The activations are the 16-row operand, the
// weights the 16-column operand.  A lane loads 16 bytes (32 codes, blocks 8c+2q and 8c+2q+1 of
// chunk c = 128 k) of its weight row, which feed 4 MFMAs; the 16 rows of a tile make each wave
// load 16 x 64 contiguous bytes.  Rows of the activation operand past M repeat row M-1 and are
// not stored.
//
// Everything is loaded straight into registers, U chunks at a time, and latency is hidden by
// occupancy (about 64 registers per lane, so more than twenty waves per CU) rather than by
// prefetching: variants that staged the activations and scale bytes in LDS or double-buffered
// the weight stream in registers measured 1.4-1.6x slower at the decode shapes.  Every wave
// handles NT tiles of 16 weight rows for the same chunks, which shares the loads and the decode
// of the activation operand; the WAVES waves of a workgroup split K' (wave w takes chunks
// w*U .. w*U+U-1, then strides on) and add their partial tiles through LDS at the end.
typedef float float4v __attribute__((ext_vector_type(4)));

// MT tiles of 16 activation rows (M <= 16 MT) share every weight fragment a wave loads and decodes:
// batched decode and short prefills (M up to 128) stay on the weight-streaming path.
// GRP: whole chunks are taken four at a time (512 k) with the scale bytes of the four chunks fetched by ONE
// load per tile: the four lanes of a row read 8 bytes each, 32 contiguous bytes of the row, and a 4 x 4
// transpose of 16-bit pairs across the four lane groups (two lane-swap instructions and two byte permutes)
// hands every lane the two bytes it needs for each chunk.  The address unit of a CU spends about two cycles
// per (row, 64-byte segment) an instruction touches, whatever it fetches from the segment, so the two-byte
// scale loads of the chunk-at-a-time loop cost as much as the code loads: without any scale loads the
// kernel ran 18-23 % faster (timing build).  Chunks past the last whole group go through that loop.
typedef unsigned uint2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void transpose_scale_pairs(uint2 s, uint32_t& even_chunks, uint32_t& odd_chunks) {
    // lane group q holds the 8 scale bytes of chunk q as four 16-bit pairs (pair p: blocks 2p, 2p+1);
    // afterwards it holds pair q of chunks 0 and 2 (even_chunks: low, high half) and of chunks 1 and 3
    const uint2v x = __builtin_amdgcn_permlane32_swap(s.x, s.y, false, false);
    const uint32_t lo = __builtin_amdgcn_perm(x[1], x[0], 0x05040100u);   // low halves of both words
    const uint32_t hi = __builtin_amdgcn_perm(x[1], x[0], 0x07060302u);   // high halves
    const uint2v t = __builtin_amdgcn_permlane16_swap(lo, hi, false, false);
    even_chunks = t[0];
    odd_chunks = t[1];
}

// Rows need not start on 16-byte boundaries (K' / 16 odd, or operands that are only 8-byte aligned): every load
// is declared with the alignment the interface guarantees (codes 8 bytes, scale bytes 1), which the memory
// path serves in one request like an aligned one.  With an odd number of blocks the last block of a row has no
// partner: the pairs of the main loops stop before it and the last wave handles it by itself at the end, with
// 8-byte loads.
template <int MT, int NT, int WAVES, int U, bool GRP, typename OutT>
__global__ __launch_bounds__(WAVES * 64) void gemm_skinny_kernel(
    const uint8_t* __restrict__ a_codes, const uint8_t* __restrict__ a_scales,
    const uint8_t* __restrict__ w_codes, const uint8_t* __restrict__ w_scales, int M, int N,
    int nbk, float alpha, OutT* __restrict__ y, int64_t ldy) {
    __shared__ float red[WAVES][MT * NT][4][64];
    static_assert(sizeof(float) * WAVES * MT * NT * 256 <= 64 * 1024, "partial tiles must fit the static LDS limit");
    // the wave number as a scalar: conditions on it become scalar branches (a matrix instruction inside a branch on a
    // vector condition would still execute: it does not honour the lane mask)
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int i = lane & 15, q = lane >> 4;
    const int n0 = blockIdx.x * (16 * NT);
    const int64_t cpitch = (int64_t)nbk * 8, spitch = nbk;
    const int nchunk = (nbk + 7) >> 3;                       // chunks of 8 blocks, the last may be partial

    const uint8_t *ac[MT], *as[MT];
#pragma unroll
    for (int r = 0; r < MT; ++r) {
        const int m = min(16 * r + i, M - 1);
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

    // ---- operand registers of one group of four whole chunks, and of the U chunks of one pass of the chunk loop
    struct Group {
        uint4 ca[4][MT], cw[4][NT];
        uint2 sa2[MT], sw2[NT];
    };
    struct Chunks {
        uint4 ca[U][MT], cw[U][NT];
        uint32_t sa[U][MT], sw[U][NT];
    };
    // Every load of a group is issued before any of it is used, the scale bytes (used first) first: loads retire
    // in issue order, so chunk m is decoded as soon as it has landed while the later chunks are still in flight.
    // (Left to itself the compiler sinks the loads of the later chunks behind the decode of the earlier ones to
    // save registers, which turns one trip to memory into three; the scheduling barriers behind the calls of
    // these functions keep the loads where they are written.)
    auto load_group = [&](int g, Group& G) {
        const int64_t co = 256 * (int64_t)g + 16 * q, so = 32 * (int64_t)g + 8 * q;
#pragma unroll
        for (int r = 0; r < MT; ++r) G.sa2[r] = load8_a1(as[r] + so);
#pragma unroll
        for (int t = 0; t < NT; ++t) G.sw2[t] = load8_a1(ws[t] + so);
#pragma unroll
        for (int m = 0; m < 4; ++m) {
#pragma unroll
            for (int r = 0; r < MT; ++r) G.ca[m][r] = load16_a8(ac[r] + co + 64 * m);
#pragma unroll
            for (int t = 0; t < NT; ++t) G.cw[m][t] = load16_a8(wc[t] + co + 64 * m);
        }
    };
    auto compute_group = [&](const Group& G) {
        uint32_t ea[2][MT], ew[2][NT];     // [chunk parity][tile]: pairs of chunks (0, 2) / (1, 3)
#pragma unroll
        for (int r = 0; r < MT; ++r) transpose_scale_pairs(G.sa2[r], ea[0][r], ea[1][r]);
#pragma unroll
        for (int t = 0; t < NT; ++t) transpose_scale_pairs(G.sw2[t], ew[0][t], ew[1][t]);
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const uint32_t sel = (m >> 1) ? 0x0C030C02u : 0x0C010C00u;
            uint32_t ha[MT], hw[NT];       // fp16 scales of the lane's two blocks of chunk m
#pragma unroll
            for (int r = 0; r < MT; ++r) ha[r] = scale_halves(ea[m & 1][r], sel);
#pragma unroll
            for (int t = 0; t < NT; ++t) hw[t] = scale_halves(ew[m & 1][t], sel);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                half8 fa[MT];
#pragma unroll
                for (int r = 0; r < MT; ++r) {
                    const uint32_t a32 = k == 0 ? G.ca[m][r].x : k == 1 ? G.ca[m][r].y : k == 2 ? G.ca[m][r].z : G.ca[m][r].w;
                    fa[r] = decode8_half(a32, ha[r], k >> 1);
                }
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    const uint32_t w32 = k == 0 ? G.cw[m][t].x : k == 1 ? G.cw[m][t].y : k == 2 ? G.cw[m][t].z : G.cw[m][t].w;
                    const half8 fw = decode8_half(w32, hw[t], k >> 1);
#pragma unroll
                    for (int r = 0; r < MT; ++r)
                        acc[r][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fa[r], fw, acc[r][t], 0, 0, 0);
                }
            }
        }
    };
    // the lane's two blocks 8c + 2q, 8c + 2q + 1 of chunk c both exist, or the pair counts as zero (codes and scale
    // bytes, so that no stray scale pattern meets a zero) and the lane reads the start of its row instead.  The
    // zeroing happens at the use, not at the load: a select behind a load would make the wave wait for it at once.
    auto load_chunks = [&](int c0, Chunks& T) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int b0 = 8 * (c0 + u) + 2 * q;
            const bool ok = b0 + 1 < nbk;
            const int64_t co = ok ? 8 * (int64_t)b0 : 0, so = ok ? b0 : 0;
#pragma unroll
            for (int r = 0; r < MT; ++r) {
                T.ca[u][r] = load16_a8(ac[r] + co);
                T.sa[u][r] = load2_a1(as[r] + so);
            }
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                T.cw[u][t] = load16_a8(wc[t] + co);
                T.sw[u][t] = load2_a1(ws[t] + so);
            }
        }
    };
    auto compute_chunks = [&](int c0, const Chunks& T) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const bool ok = 8 * (c0 + u) + 2 * q + 1 < nbk;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                half8 fa[MT];
#pragma unroll
                for (int r = 0; r < MT; ++r) {
                    const uint32_t a32 = k == 0 ? T.ca[u][r].x : k == 1 ? T.ca[u][r].y : k == 2 ? T.ca[u][r].z : T.ca[u][r].w;
                    fa[r] = decode8(ok ? a32 : 0u, scale_pair(!ok ? 0u : k < 2 ? (T.sa[u][r] & 0xFFu) : (T.sa[u][r] >> 8)));
                }
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    const uint32_t w32 = k == 0 ? T.cw[u][t].x : k == 1 ? T.cw[u][t].y : k == 2 ? T.cw[u][t].z : T.cw[u][t].w;
                    const half8 fw = decode8(ok ? w32 : 0u, scale_pair(!ok ? 0u : k < 2 ? (T.sw[u][t] & 0xFFu) : (T.sw[u][t] >> 8)));
#pragma unroll
                    for (int r = 0; r < MT; ++r)
                        acc[r][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fa[r], fw, acc[r][t], 0, 0, 0);
                }
            }
        }
    };
    bool grouped = false;
    if constexpr (GRP) grouped = nbk >= 32;
    if (grouped) {
        // Whole chunks in groups of four, dealt round-robin to the waves; the up to four chunks behind the last
        // group go to the waves that took one group less.  With one group per wave and four tiles (the up-projection
        // shapes) such a wave asks for its left-over chunk FIRST and decodes it last, so that it costs no trip to
        // memory of its own (1 us of 12 there); with few tiles per wave and several groups the same change made the
        // kernel 10 % slower (measured), so those variants load it where they use it.  (Dealing the left-over chunks
        // out as (chunk, tile) units, one per wave, balances the waves but decodes the activation chunk once per unit:
        // 11.7 against 10.5 us on the 16 x 14336 x 4352 shape, not kept.)
        constexpr bool HOIST = MT == 1 && NT == 4;
        const int ngroup = nbk >> 5;
        const int tail_c = 4 * ngroup + (wave - ngroup % WAVES + WAVES) % WAVES * U;
        const bool has_tail = tail_c < nchunk;
        Chunks tail;
        if (HOIST && has_tail) load_chunks(tail_c, tail);
        for (int g = wave; g < ngroup; g += WAVES) {
            Group ga;
            load_group(g, ga);
            __builtin_amdgcn_sched_barrier(0);
            compute_group(ga);
        }
        if (!HOIST && has_tail) load_chunks(tail_c, tail);
        if (has_tail) compute_chunks(tail_c, tail);
    } else {
        for (int c0 = wave * U; c0 < nchunk; c0 += WAVES * U) {
            Chunks T;
            load_chunks(c0, T);
            compute_chunks(c0, T);
        }
    }
    // the last block of a row with an odd number of blocks: lane group 0 supplies its two octets, the others zeros
    if ((nbk & 1) != 0 && wave == WAVES - 1) {
        uint2 oa[MT], ow[NT];
        uint32_t osa[MT], osw[NT];
#pragma unroll
        for (int r = 0; r < MT; ++r) {
            oa[r] = load8_a8(ac[r] + 8 * (int64_t)(nbk - 1));
            osa[r] = as[r][nbk - 1];
        }
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            ow[t] = load8_a8(wc[t] + 8 * (int64_t)(nbk - 1));
            osw[t] = ws[t][nbk - 1];
        }
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            half8 fa[MT];
#pragma unroll
            for (int r = 0; r < MT; ++r) fa[r] = decode8(q ? 0u : k ? oa[r].y : oa[r].x, scale_pair(q ? 0u : osa[r]));
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const half8 fw = decode8(q ? 0u : k ? ow[t].y : ow[t].x, scale_pair(q ? 0u : osw[t]));
#pragma unroll
                for (int r = 0; r < MT; ++r)
                    acc[r][t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(fa[r], fw, acc[r][t], 0, 0, 0);
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
        if (m < M && n < N) store_out(y + (int64_t)m * ldy + n, sum * alpha);
    }
}

template <int MT, int NT, int WAVES, int U, bool GRP, typename OutT>
arcq_status launch_skinny(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* w_codes,
                                 const uint8_t* w_scales, int M, int N, int nbk, float alpha, OutT* y, int64_t ldy,
                                 hipStream_t stream) {
    hipLaunchKernelGGL((gemm_skinny_kernel<MT, NT, WAVES, U, GRP, OutT>), dim3((N + 16 * NT - 1) / (16 * NT)),
                       dim3(WAVES * 64), 0, stream, a_codes, a_scales, w_codes, w_scales, M, N, nbk, alpha, y, ldy);
    return check_launch("gemm_skinny_kernel");
}

// Shapes the weight-streaming kernel serves (alignment permitting): up to 64 rows always; up to 128 rows
// unless the problem is big enough for the tiled kernels with split K to be faster (measured over
// N = 1024 .. 28672, K' = 1088 .. 14592 at M = 80, 96, 128: the eight-row-tile variant of the streaming kernel
// takes about 1 us per 10^6 weights, the tiled path 20-30 us for everything up to 6 * 10^7 weights, more with
// a short K' that cannot be split).
static bool skinny_shape(int64_t M, int64_t N, int64_t Kp) {
    if (M <= 64) return true;
    if (M > 128) return false;
    const int64_t weights = N * Kp;
    return !((Kp >= 4096 && weights >= 20000000) || (Kp >= 8192 && weights >= 12000000));
}

// Number of runs the reduction dimension is cut into (1: no split).  A function of the shape alone,
// so that the workspace a caller sizes beforehand matches what the launch uses.  Problems off the
// weight-streaming path with too few 128 x 128 tiles to occupy the chip split K' into runs of at least four
// stages (256 k).  The number of runs minimises a cost in units of one stage time of a tile (about
// 1.3 us): rounds of workgroups over the 256 CUs times the stages of a run, plus, when split, the
// write and read of the fp32 partial results at about 3 TB/s.
int split_k(int64_t M, int64_t N, int64_t Kp) {
    const int64_t nbk = Kp >> 4;
    if (skinny_shape(M, N, Kp) || nbk < 8) return 1;
    if (gemm_ksplit_variant(M, N, Kp) != 0) return 1;      // the k split happens inside the workgroups
    if (((M + 255) / 256) * ((N + 255) / 256) >= 256 || ((M + 127) / 128) * ((N + 255) / 256) >= 192) return 1;
    const int64_t tiles = ((M + 127) / 128) * ((N + 127) / 128);
    if (tiles > 128) return 1;
    const int64_t nstage = (nbk + 7) >> 3;
    const int64_t max_splits = std::min<int64_t>(8, nstage / 4);
    int best = 1;
    double best_cost = 0.0;
    for (int64_t sp = 1; sp <= max_splits; ++sp) {
        const double rounds = (double)((tiles * sp + 255) / 256);
        double cost = rounds * (double)((nstage + sp - 1) / sp);
        if (sp > 1) cost += (double)sp * (double)M * (double)N * 8.0 / 4.0e6;
        if (sp == 1 || cost < best_cost) {
            best = (int)sp;
            best_cost = cost;
        }
    }
    return best;
}

template <typename OutT>
arcq_status launch_typed(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* w_codes,
                         const uint8_t* w_scales, int64_t M, int64_t N, int64_t Kp, float alpha, OutT* y,
                         int64_t ldy, float* workspace, hipStream_t stream) {
    const int nbk = (int)(Kp >> 4);
    const bool aligned16 = ((reinterpret_cast<uintptr_t>(a_codes) | reinterpret_cast<uintptr_t>(w_codes)) & 15) == 0 &&
                           ((reinterpret_cast<uintptr_t>(a_scales) | reinterpret_cast<uintptr_t>(w_scales)) & 3) == 0;
    // 33 to 64 rows against many weight rows: 64 x 64 tiles with the k split inside the workgroup decode every activation
    // fragment once per tile, the weight-streaming kernel once per 32 weight rows
    // (measured with weights from HBM, 64 rows: 14336 x 4352 15.8 us against 21.8, 9216 x 4352 15.3 against 25.3,
    // 12288 x 8448 25.0 against 44.8; 33 rows gain as long as the tiles are 64 x 64)
    const int ks_variant = M > 32 ? gemm_ksplit_variant(M, N, Kp) : 0;
    const bool tiles_instead = ks_variant == 1 || ks_variant == 6 || (ks_variant != 0 && M > 48);
    if (skinny_shape(M, N, Kp) && !tiles_instead) {
        // Weight-streaming path.  Enough waves to keep the weight stream in flight, as few as that allows
        // so that each wave has several KB to request at once: with many weight rows several tiles per
        // wave share the activation operand; with few, one tile per wave so that every CU still gets a
        // workgroup (measured at the decode shapes).
        const int64_t tiles = (N + 15) / 16;
        // tiles per wave: as few as give the chip at most one workgroup per compute unit (256), up to four (three with
        // 17 to 32 activation rows); measured with weights from HBM at 16 rows: 640 tiles (N = 10240, K' = 8448) 13.7 us
        // with three tiles per wave against 18.1 us with two (320 workgroups: two rounds), 576 tiles 8.7 against 10.6
        // (257 to 399 tiles used to run one tile per wave, two workgroups sharing a CU: 320 tiles over K' = 27904 33.7 us
        // against 27.3 us with two tiles per wave, over K' = 4352 7.6 against 6.9)
        const int64_t T2 = 257, T3 = 513, T4 = 769;
#define ARCQ_SKINNY_W(MT_, NT_, W_, U_) \
    return launch_skinny<MT_, NT_, W_, U_, (MT_ <= 4)>(a_codes, a_scales, w_codes, w_scales, (int)M, (int)N, nbk, alpha, y, ldy, stream)
#define ARCQ_SKINNY(MT_, NT_, U_) ARCQ_SKINNY_W(MT_, NT_, 8, U_)
        if (M <= 16) {
            if (tiles >= T4) ARCQ_SKINNY(1, 4, 1);
            if (tiles >= T3) ARCQ_SKINNY(1, 3, 1);
            if (tiles >= T2) ARCQ_SKINNY(1, 2, 2);
            ARCQ_SKINNY(1, 1, 2);
        }
        if (M <= 32) {
            // (32 rows, weights from HBM: 640 tiles 17.2 us with three tiles per wave against 24.0 with one, 512 tiles
            // 14.7 with two against 17.9, 896 tiles 12.4 with four against 15.7 with two)
            if (tiles >= T4) ARCQ_SKINNY(2, 4, 1);
            if (tiles >= T3) ARCQ_SKINNY(2, 3, 1);
            if (tiles >= T2) ARCQ_SKINNY(2, 2, 1);
            ARCQ_SKINNY(2, 1, 2);
        }
        if (M <= 64) {
            // (64 rows, weights from HBM: 512 tiles over K' = 8464 23.2 us with two tiles per wave against 34.6 with one)
            if (tiles >= T2) ARCQ_SKINNY(4, 2, 1);
            ARCQ_SKINNY(4, 1, 1);
        }
        if (tiles >= T2) ARCQ_SKINNY_W(8, 2, 4, 1);    // 128 rows, 512 tiles over K' = 2064: 16.2 us against 20.0
        ARCQ_SKINNY(8, 1, 1);
#undef ARCQ_SKINNY
#undef ARCQ_SKINNY_W
    }
    const bool offsets_fit = (uint64_t)M * (uint64_t)nbk * 8 < 0xFFFF0000ull && (uint64_t)N * (uint64_t)nbk * 8 < 0xFFFF0000ull;
    if (const int variant = gemm_ksplit_variant(M, N, Kp))
        return launch_gemm_ksplit(variant, a_codes, a_scales, w_codes, w_scales, M, N, Kp, alpha, y,
                                  std::is_same<OutT, _Float16>::value ? ARCQ_DTYPE_F16 : ARCQ_DTYPE_F32, ldy, stream);
    if ((nbk & 3) == 0 && nbk >= 8 && offsets_fit && aligned16) {
        // Tiles of 256 weight rows by 256, 192 or 128 activation rows when there is work for them.  Workgroups run in
        // rounds of one per compute unit and a round lasts as long as one tile, so the tile height that minimises
        // rounds x (time of a stage of that tile) wins: 2.96, 2.59 and 1.96 us measured per 128-k stage (the bigger
        // tile decodes fewer fragments per matrix instruction: 45, 53 and 60 ps per output element and stage).
        // E.g. 768 x 14336: 224 tiles of 192 rows in one round 88 us, 336 tiles of 128 rows in two rounds 113 us,
        // 168 tiles of 256 rows 100 us; 1024 x 14336: 224 tiles of 256 rows 106 us against 120 us.
        const int64_t tn256 = (N + 255) / 256;
        const int64_t t128x256 = ((M + 127) / 128) * tn256;
        if (t128x256 >= 192) {
            auto cost = [&](int bm, double t_stage) { return (double)((((M + bm - 1) / bm) * tn256 + 255) / 256) * t_stage; };
            const double c256 = cost(256, 2.96), c192 = cost(192, 2.59), c128 = cost(128, 1.96);
            if (c256 <= c192 && c256 <= c128)
                return launch_staged<4, 4, 2, 2>(a_codes, a_scales, w_codes, w_scales, (int)M, (int)N, nbk, alpha, y, ldy, stream);
            if (c192 <= c128)
                return launch_staged<3, 4, 2, 2>(a_codes, a_scales, w_codes, w_scales, (int)M, (int)N, nbk, alpha, y, ldy, stream);
        }
        // 128 x 256 tiles with 8 waves of 64 x 64 (two per SIMD): 5 % faster than 4 waves of 64 x 128 on the
        // 2048 x 4096 x 4352 problem; on the large shapes 4 and 8 waves measure the same
        if (t128x256 >= 192) {
            // whole stages: the variant whose wave pairs split every stage (6 % faster on the 2048 x 4096 x 4352 problem)
            {
                if ((nbk & 7) == 0 && nbk >= 16) {
                    using C = StagedCfg<2, 2, 2, 4>;
                    auto kern = gemm_kpair_kernel<OutT>;
                    static std::atomic<uint64_t> lds_raised{0};
                    if (arcq_status st = raise_lds_limit(reinterpret_cast<const void*>(kern), lds_raised)) return st;
                    const int tiles_m = (int)((M + 127) / 128), tiles_n = (int)((N + 255) / 256);
                    hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(512), C::LDS_BYTES, stream, a_codes, a_scales, w_codes,
                                       w_scales, (int)M, (int)N, nbk, alpha, y, ldy, tiles_m, tiles_n);
                    return check_launch("gemm_kpair_kernel");
                }
            }
            return launch_staged<2, 2, 2, 4>(a_codes, a_scales, w_codes, w_scales, (int)M, (int)N, nbk, alpha, y, ldy, stream);
        }
        // More than 256 tiles of 128 x 128 (two workgroups on some compute units, one on the others) but at most 256 of
        // 192 x 128: one round of the taller tile, which also decodes five fragments per six matrix instructions
        // instead of four per four (1.52 against 1.3 us per stage and tile): 512 x 10240 over K' = 8448 116 -> 100 us,
        // 1024 x 5120 over 27904 365 -> 297 us, 1280 x 4096 over 4352 61 -> 49 us.
        {
            const int64_t t128 = ((M + 127) / 128) * ((N + 127) / 128), t192 = ((M + 191) / 192) * ((N + 127) / 128);
            if (t128 > 256 && t192 <= 256)
                return launch_staged<3, 2, 2, 2>(a_codes, a_scales, w_codes, w_scales, (int)M, (int)N, nbk, alpha, y, ldy, stream);
        }
        return launch_staged<2, 2, 2, 2>(a_codes, a_scales, w_codes, w_scales, (int)M, (int)N, nbk, alpha, y, ldy, stream,
                                         split_k(M, N, Kp), workspace);
    }
    if (offsets_fit && nbk >= 8) {
        // any K' that is a multiple of 16, operands that are only 8-byte aligned: stages through registers (no 256 x 256
        // tiles: the staging registers do not fit beside 256 accumulators); the same choice by rounds x stage time
        // (3.5 and 2.4 us measured per stage for 192 x 256 and 128 x 256 tiles: 768 x 14336 over K' = 4368 118 us instead of 163)
        const int64_t tn256 = (N + 255) / 256;
        if (((M + 127) / 128) * tn256 >= 192) {
            auto cost = [&](int bm, double t_stage) { return (double)((((M + bm - 1) / bm) * tn256 + 255) / 256) * t_stage; };
            if (cost(192, 3.5) <= cost(128, 2.4))
                return launch_staged<3, 4, 2, 2, true>(a_codes, a_scales, w_codes, w_scales, (int)M, (int)N, nbk, alpha, y, ldy, stream);
            return launch_staged<2, 2, 2, 4, true>(a_codes, a_scales, w_codes, w_scales, (int)M, (int)N, nbk, alpha, y, ldy, stream);
        }
        const int64_t t128 = ((M + 127) / 128) * ((N + 127) / 128), t192 = ((M + 191) / 192) * ((N + 127) / 128);
        if (t128 > 256 && t192 <= 256)
            return launch_staged<3, 2, 2, 2, true>(a_codes, a_scales, w_codes, w_scales, (int)M, (int)N, nbk, alpha, y, ldy, stream);
        return launch_staged<2, 2, 2, 2, true>(a_codes, a_scales, w_codes, w_scales, (int)M, (int)N, nbk, alpha, y, ldy, stream,
                                               split_k(M, N, Kp), workspace);
    }
    dim3 grid((unsigned)((N + 127) / 128), (unsigned)((M + 127) / 128));
    hipLaunchKernelGGL(gemm_direct_kernel<OutT>, grid, dim3(256), 0, stream, a_codes, a_scales, w_codes, w_scales,
                       (int)M, (int)N, nbk, alpha, y, ldy);
    return check_launch("gemm_direct_kernel");
}

}  // namespace

arcq_status launch_splitk_reduce(const float* partial, int splits, int M, int N, float alpha, void* y, int y_dtype,
                                 int64_t ldy, hipStream_t stream) {
    const int64_t stride = (int64_t)M * N;
    const int vec4 = (N & 3) == 0 && (ldy & 3) == 0 && (reinterpret_cast<uintptr_t>(y) & 15) == 0;
    const int64_t work = vec4 ? stride / 4 : stride;
    const int blocks = (int)std::min<int64_t>((work + 255) / 256, 4096);
    if (y_dtype == ARCQ_DTYPE_F16)
        hipLaunchKernelGGL(splitk_reduce_kernel<_Float16>, dim3(blocks), dim3(256), 0, stream, partial, splits, stride, M, N,
                           alpha, static_cast<_Float16*>(y), ldy, vec4);
    else
        hipLaunchKernelGGL(splitk_reduce_kernel<float>, dim3(blocks), dim3(256), 0, stream, partial, splits, stride, M, N,
                           alpha, static_cast<float*>(y), ldy, vec4);
    return check_launch("splitk_reduce_kernel");
}

size_t gemm_workspace_bytes(int64_t M, int64_t N, int64_t Kp) {
    const int splits = split_k(M, N, Kp);
    return splits > 1 ? (size_t)splits * (size_t)M * (size_t)N * sizeof(float) : 0;
}

// ---------------------------------------------------------------------------------------------
// Scratch memory of arcq_gemm_noalloc: the fp32 partial results of a split reduction dimension for
// callers that cannot allocate a workspace.  Every GPU the library runs on holds its own copy of this
// array, at its own address, until the process ends.  In host code the array's name is only a stand-in
// for hipGetSymbolAddress; launches get the per-device address kept in g_scratch_ptr.
static __device__ __align__(256) unsigned char scratch[ARCQ_NOALLOC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];
}  // namespace

// Device address of `scratch` on the current device; looked up once per device.
arcq_status gemm_scratch_pointer(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(ARCQ_HIP_ERROR, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fail(ARCQ_HIP_ERROR, "device index %d beyond the %d this library keeps scratch for", dev, kMaxDevices);
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return fail(ARCQ_HIP_ERROR, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
        g_scratch_ptr[dev].store(p, std::memory_order_release);     // the same value from whichever thread gets here first
    }
    *out = p;
    return ARCQ_OK;
}

arcq_status launch_gemm(const uint8_t* a_codes, const uint8_t* a_scales,
                        const uint8_t* w_codes, const uint8_t* w_scales,
                        int64_t M, int64_t N, int64_t Kp, float alpha,
                        void* y, int y_dtype, int64_t ldy,
                        void* workspace, size_t, hipStream_t stream) {
    float* ws = static_cast<float*>(workspace);
    if (y_dtype == ARCQ_DTYPE_F16)
        return launch_typed<_Float16>(a_codes, a_scales, w_codes, w_scales, M, N, Kp, alpha,
                                      static_cast<_Float16*>(y), ldy, ws, stream);
    return launch_typed<float>(a_codes, a_scales, w_codes, w_scales, M, N, Kp, alpha, static_cast<float*>(y), ldy, ws, stream);
}

}  // namespace arcq
