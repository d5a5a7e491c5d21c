// Tiled W4A4 GEMM for problems with few output tiles (a few hundred activation rows; Section 3.2 eq. (2)): the waves
// of a workgroup split every stage along k INSIDE the compute unit, so a small output tile still keeps all four
// SIMDs busy and the chip gets one tile per compute unit without a round trip of fp32 partial results through
// HBM and a second launch (which is what splitting K' across workgroups costs).
//
// Workgroup tile BM x BN = 32 WM GM x 32 WN GN, computed by GM x GN x KS waves: wave (wq, kh) accumulates the
// WM x WN fragments of sub-tile wq over the k-quarter kh of every stage.  A stage is 64 KS k (256 for KS = 4): per
// row 32 KS code bytes (2 KS pieces of 16 bytes) and 4 KS scale bytes, kept packed in LDS and decoded in registers
// (gemm_decode.h); wave kh reads pieces 2 kh and 2 kh + 1 of a row (lanes 0-31 the first, lanes 32-63 the second:
// four k-steps, as in the wave-pair kernel of gemm.hip, whose schedule this kernel shares) and the scale word at
// byte 4 kh.  Stages travel global -> LDS with global_load_lds through a ring of three buffers.  The 16-byte
// pieces of a row are XOR-swizzled so that 16 consecutive rows fall on 16 different bank groups (rows are 128
// bytes apart for KS = 4: swizzle (row >> 1) & 7; 64 bytes for KS = 2: (row >> 2) & 3).
// At the end the KS partial tiles are added through the LDS in KS - 1 rounds; fragment f of a sub-tile is owned
// (finished and stored) by wave kh = f % KS (with six fragments and four waves two waves own two, two own one).
#include "internal.h"
#include "gemm_decode.h"
#include "gemm_epilogue.h"
#include "lds_dma.h"

#include <type_traits>

namespace arcq {

namespace {

template <int WM, int WN, int GM, int GN, int KS>
struct KsplitCfg {
    static_assert(KS == 2 || KS == 4, "k halves or quarters");
    static constexpr int BM = 32 * WM * GM, BN = 32 * WN * GN;
    static constexpr int NWAVE = GM * GN * KS, NT = 64 * NWAVE;
    static constexpr int ROWB = 32 * KS;            // code bytes of a row per stage
    static constexpr int PPR = 2 * KS;              // 16-byte pieces of a row per stage
    static constexpr int SROWB = 4 * KS;            // scale bytes of a row per stage
    // copy instructions per thread and stage (a copy always involves the whole workgroup; surplus lanes re-fetch
    // the operand's last rows into padding behind its region, so that every wave issues the same number)
    static constexpr int NA = (BM * PPR + NT - 1) / NT, NW = (BN * PPR + NT - 1) / NT;
    static constexpr int NAS = (BM * KS + NT - 1) / NT, NWS = (BN * KS + NT - 1) / NT;
    static constexpr int NDMA = NA + NW + NAS + NWS;
    static constexpr int A_CODES = 0;
    static constexpr int W_CODES = NA * NT * 16;
    static constexpr int A_SCALES = W_CODES + NW * NT * 16;
    static constexpr int W_SCALES = A_SCALES + NAS * NT * 4;
    static constexpr int STAGE_BYTES = W_SCALES + NWS * NT * 4;
    static constexpr int NSTAGE = 3, DIST = 2;
    static constexpr int OWN = (WM * WN + KS - 1) / KS;  // fragments a wave finishes and stores (at most)
    static constexpr int LDS_BYTES = NSTAGE * STAGE_BYTES;
    static_assert(NWAVE * OWN * 4096 <= LDS_BYTES, "the exchange regions must fit the operand ring");
    static_assert((NT / PPR) % 16 == 0 && (NT / KS) % 1 == 0, "row swizzle must not depend on the copy index");
    static_assert((DIST - 1) * NDMA < 64, "the vector-memory counter has 6 bits");
};

// One 32 x 32 fragment computed with the weights as the row operand: lane holds output row m0 + lane % 32, register
// e holds column n0 + 8 (e / 4) + 4 (lane / 32) + e % 4.
template <typename OutT>
__device__ __forceinline__ void store_fragment(const float16v& a, int m0, int n0, int r, int h, int M, int N, float alpha,
                                               OutT* __restrict__ y, int64_t ldy, bool vec_ok) {
    const int m = m0 + r;
    if (m >= M) return;
    OutT* yrow = y + (int64_t)m * ldy;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const int n = n0 + 8 * g + 4 * h;
        const float v0 = a[4 * g] * alpha, v1 = a[4 * g + 1] * alpha, v2 = a[4 * g + 2] * alpha, v3 = a[4 * g + 3] * alpha;
        if (vec_ok && n + 3 < N) {
            store4(yrow + n, v0, v1, v2, v3);
        } else {
            if (n < N) store_out(yrow + n, v0);
            if (n + 1 < N) store_out(yrow + n + 1, v1);
            if (n + 2 < N) store_out(yrow + n + 2, v2);
            if (n + 3 < N) store_out(yrow + n + 3, v3);
        }
    }
}

// REG: any K' (a multiple of 16) and operands that are only 8-byte aligned: a thread fetches its pieces of stage s + 2
// into registers with ordinary loads (declared with the alignment the interface guarantees), right after the barrier
// that opens stage s + 1, and writes them to LDS before the barrier that opens their stage; blocks past the end of a row
// become zero codes and zero scale bytes (a piece that would reach past the row's end is fetched from further left and
// shifted), so the last stage needs no special case.
template <int WM, int WN, int GM, int GN, int KS, typename OutT, bool REG = false>
__global__ __launch_bounds__(64 * GM * GN * KS) void gemm_ksplit_kernel(
    const uint8_t* __restrict__ a_codes, const uint8_t* __restrict__ a_scales,
    const uint8_t* __restrict__ w_codes, const uint8_t* __restrict__ w_scales, int M, int N,
    int nbk, float alpha, OutT* __restrict__ y, int64_t ldy, int tiles_m, int tiles_n) {
    using C = KsplitCfg<WM, WN, GM, GN, KS>;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

    // workgroup -> tile: workgroups are dealt round-robin to the 8 XCDs (each with its own L2); every XCD gets a
    // contiguous run of the tile sequence, walked in column-major groups of 8 tile rows
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
    const int kh = wave / (GM * GN);                 // k share: k-steps 4 kh .. 4 kh + 3 of every stage
    const int wq = wave % (GM * GN);
    const int wg_m0 = tile_m * C::BM, wg_n0 = tile_n * C::BN;
    const int wrow0 = (wq / GN) * (32 * WM);         // first row of this wave inside the A tile
    const int wcol0 = (wq % GN) * (32 * WN);         // first row of this wave inside the W tile
    // stages of 4 KS blocks; the last one may hold only `part` k shares (K' is a multiple of 64, not of 64 KS): the
    // copies of its missing shares re-fetch the first share (in bounds, never used) and the waves of those shares read
    // their scale bytes as zero, so that their fragments decode to zeros
    const int nstage = (nbk + 4 * KS - 1) / (4 * KS);
    const int part = REG ? 0 : (nbk % (4 * KS)) / 4; // 0: the last stage is whole (REG: made whole with zeros)

    // ---- copies
    auto swz = [](int row) -> uint32_t { return KS == 4 ? (uint32_t)(row >> 1) & 7u : (uint32_t)(row >> 2) & 3u; };
    const int crow = tid / C::PPR, srow = tid / KS;  // row of this thread inside a copy of NT / PPR code rows / NT / KS scale rows
    const uint32_t adj_c = 16u * ((uint32_t)(tid % C::PPR) ^ swz(crow));
    const uint32_t adj_s = 4u * (uint32_t)(tid % KS);
    const uint32_t cpitch32 = (uint32_t)nbk * 8u, spitch32 = (uint32_t)nbk;
    const uint32_t wave_slot = __builtin_amdgcn_readfirstlane((uint32_t)(tid & ~63));
    const uint32_t lds0 = lds_address(lds);
    const uint32_t piece_g = (uint32_t)(tid % C::PPR) ^ swz(crow);      // global piece this lane fetches
    const bool piece_missing = part != 0 && (int)(piece_g >> 1) >= part, scale_missing = part != 0 && tid % KS >= part;
    const uint32_t adj_c_last = piece_missing ? 16u * (piece_g & 1u) : adj_c, adj_s_last = scale_missing ? 0u : adj_s;
    auto issue_one = [&](int d, int stage, int buf) {
        const uint32_t base = lds0 + buf * C::STAGE_BYTES;
        const bool last = stage == nstage - 1;
        const uint32_t oc = (uint32_t)stage * C::ROWB + (last ? adj_c_last : adj_c);
        const uint32_t os = (uint32_t)stage * C::SROWB + (last ? adj_s_last : adj_s);
        constexpr int NA = C::NA, NW = C::NW, NAS = C::NAS, NT = C::NT;
        // rows past the edge of the operand re-read its last row (never stored)
        if (d < NA) {
            const uint32_t row = (uint32_t)min(wg_m0 + d * (NT / C::PPR) + crow, M - 1);
            dma16(a_codes, row * cpitch32 + oc, base + C::A_CODES + 16u * (d * NT + wave_slot));
        } else if (d < NA + NW) {
            const int p = d - NA;
            const uint32_t row = (uint32_t)min(wg_n0 + p * (NT / C::PPR) + crow, N - 1);
            dma16(w_codes, row * cpitch32 + oc, base + C::W_CODES + 16u * (p * NT + wave_slot));
        } else if (d < NA + NW + NAS) {
            const int p = d - NA - NW;
            const uint32_t row = (uint32_t)min(wg_m0 + p * (NT / KS) + srow, M - 1);
            dma4(a_scales, row * spitch32 + os, base + C::A_SCALES + 4u * (p * NT + wave_slot));
        } else {
            const int p = d - NA - NW - NAS;
            const uint32_t row = (uint32_t)min(wg_n0 + p * (NT / KS) + srow, N - 1);
            dma4(w_scales, row * spitch32 + os, base + C::W_SCALES + 4u * (p * NT + wave_slot));
        }
    };

    // ---- REG: the same pieces through registers (piece d of a thread lands where copy d puts it); needs nbk >= 4
    constexpr int NCP = C::NA + C::NW, NSP = C::NAS + C::NWS;
    uint4 rc[REG ? NCP : 1];
    uint32_t rs[REG ? NSP : 1];
    auto reg_issue = [&](int stage) {
        const uint32_t oc = 8u * (uint32_t)min(4 * KS * stage + 2 * (int)piece_g, nbk - 2);
#pragma unroll
        for (int d = 0; d < NCP; ++d) {
            const bool is_a = d < C::NA;
            const int p = is_a ? d : d - C::NA;
            const uint32_t row = (uint32_t)(is_a ? min(wg_m0 + p * (C::NT / C::PPR) + crow, M - 1) : min(wg_n0 + p * (C::NT / C::PPR) + crow, N - 1));
            rc[d] = load16_a8((is_a ? a_codes : w_codes) + (size_t)(row * cpitch32 + oc));
        }
        const uint32_t os = (uint32_t)min(4 * KS * stage + 4 * (tid % KS), nbk - 4);
#pragma unroll
        for (int d = 0; d < NSP; ++d) {
            const bool is_a = d < C::NAS;
            const int p = is_a ? d : d - C::NAS;
            const uint32_t row = (uint32_t)(is_a ? min(wg_m0 + p * (C::NT / KS) + srow, M - 1) : min(wg_n0 + p * (C::NT / KS) + srow, N - 1));
            rs[d] = load4_a1((is_a ? a_scales : w_scales) + (size_t)(row * spitch32 + os));
        }
    };
    auto reg_commit = [&](int stage, int buf) {
        uint8_t* st = lds + buf * C::STAGE_BYTES;
        const int b0 = 4 * KS * stage + 2 * (int)piece_g;      // this piece: blocks b0, b0 + 1
        const bool both = b0 + 1 < nbk, one = b0 < nbk;
#pragma unroll
        for (int d = 0; d < NCP; ++d) {
            const uint4 v = uint4{both ? rc[d].x : one ? rc[d].z : 0u, both ? rc[d].y : one ? rc[d].w : 0u, both ? rc[d].z : 0u, both ? rc[d].w : 0u};
            const int at = d < C::NA ? C::A_CODES + 16 * (d * C::NT + tid) : C::W_CODES + 16 * ((d - C::NA) * C::NT + tid);
            *reinterpret_cast<uint4*>(st + at) = v;
        }
        const int sb0 = 4 * KS * stage + 4 * (tid % KS);       // this word: blocks sb0 .. sb0 + 3
        const int skip = sb0 - min(sb0, nbk - 4);               // bytes of the fetched word that belong to earlier blocks
#pragma unroll
        for (int d = 0; d < NSP; ++d) {
            const uint32_t word = skip >= 4 ? 0u : rs[d] >> (8 * skip);
            const int at = d < C::NAS ? C::A_SCALES + 4 * (d * C::NT + tid) : C::W_SCALES + 4 * ((d - C::NAS) * C::NT + tid);
            *reinterpret_cast<uint32_t*>(st + at) = word;
        }
    };

    // ---- LDS read offsets: this wave's share of a stage is piece 2 kh + h of a row's codes and the scale word at
    // byte 4 kh; fragment i of a wave is 32 rows further on (the swizzle only depends on lane % 32 because the other
    // terms are multiples of 32)
    const uint32_t piece = 16u * ((uint32_t)(2 * kh + h) ^ swz(r));
    const uint32_t rd_a = C::A_CODES + (wrow0 + r) * C::ROWB + piece, rd_w = C::W_CODES + (wcol0 + r) * C::ROWB + piece;
    const uint32_t rd_as = C::A_SCALES + (wrow0 + r) * C::SROWB + 4 * kh, rd_ws = C::W_SCALES + (wcol0 + r) * C::SROWB + 4 * kh;
    const uint32_t scale_sel = h ? 0x0C030C02u : 0x0C010C00u;

    float16v acc[WM][WN];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    constexpr int G = WM + WN;                 // fragments per k-step
    constexpr int MPG = (WM * WN >= 16) ? 2 : 1;   // MFMAs per group (singles spill with 4 x 4 fragments)
    constexpr int P = WM * WN / MPG;           // groups per k-step: after every group the decode of G / P fragments
    uint4 ca[WM], cw[WN];
    uint32_t sa[WM], sw[WN];
    half8 fa[2][WM], fw[2][WN];
    const bool share_missing = part != 0 && kh >= part;     // this wave has nothing in the last stage
    auto read_raw = [&](const uint8_t* st, bool zero) {
#pragma unroll
        for (int i = 0; i < WM; ++i) {
            ca[i] = *reinterpret_cast<const uint4*>(st + rd_a + i * (32 * C::ROWB));
            const uint32_t word = *reinterpret_cast<const uint32_t*>(st + rd_as + i * (32 * C::SROWB));
            sa[i] = scale_halves(zero ? 0u : word, scale_sel);
        }
#pragma unroll
        for (int j = 0; j < WN; ++j) {
            cw[j] = *reinterpret_cast<const uint4*>(st + rd_w + j * (32 * C::ROWB));
            const uint32_t word = *reinterpret_cast<const uint32_t*>(st + rd_ws + j * (32 * C::SROWB));
            sw[j] = scale_halves(zero ? 0u : word, scale_sel);
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

    // One stage = four k-steps of this wave.  During step t the fragments of step t + 1 are decoded, one group of
    // fragments after every MFMA; the raw codes of the next stage are read at the start of step 3 (every fragment of
    // this stage has been decoded by then) behind the barrier that opens that stage, and step 3 decodes its first
    // fragments.  The copies of stage s + DIST are issued during steps 0..2, into the buffer of stage s - 1, which
    // every wave left before the barrier that opened stage s.
    int buf = 0;
    auto ring_next = [](int b) { return b == C::NSTAGE - 1 ? 0 : b + 1; };
    auto run_stage = [&](int s) {
        const int buf1 = ring_next(buf), buf2 = buf == 0 ? C::NSTAGE - 1 : buf - 1;
        const int fetch = min(s + C::DIST, nstage - 1);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            if (t == 3) {
                if constexpr (REG) {
                    reg_commit(min(s + 1, nstage - 1), buf1);       // fetched since step 3 of the stage before
                    wait_lgkmcnt0();
                } else {
                    wait_vmcnt<(C::DIST - 1) * C::NDMA>();
                }
                wg_barrier();
                read_raw(lds + buf1 * C::STAGE_BYTES, share_missing && s + 1 >= nstage - 1);
                if constexpr (REG) reg_issue(min(s + 2, nstage - 1));
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int p = 0; p < P; ++p) {
#pragma unroll
                for (int gidx = (p * G) / P; gidx < ((p + 1) * G) / P; ++gidx) decode_frag(gidx, (t + 1) & 3);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int q = MPG * p; q < MPG * p + MPG; ++q) {
                    const int i = q / WN, j = q % WN;
                    // weights as the row operand: see store_fragment
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(fw[t & 1][j], fa[t & 1][i], acc[i][j], 0, 0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
                if (!REG && t < 3) {
#pragma unroll
                    for (int d = 0; d < C::NDMA; ++d)
                        if ((d * 3) / C::NDMA == t && (d - (t * C::NDMA + 2) / 3) == p) issue_one(d, fetch, buf2);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
        buf = buf1;
    };
    static_assert((C::NDMA + 2) / 3 <= P, "the copies of a stage are spread over the MFMAs of three k-steps");

    if constexpr (REG) {
        reg_issue(0);
        reg_commit(0, 0);
        reg_issue(min(1, nstage - 1));
        wait_lgkmcnt0();
    } else {
#pragma unroll
        for (int d = 0; d < C::DIST; ++d)
#pragma unroll
            for (int q = 0; q < C::NDMA; ++q) issue_one(q, min(d, nstage - 1), d);
        wait_vmcnt<(C::DIST - 1) * C::NDMA>();
    }
    wg_barrier();
    read_raw(lds, share_missing && nstage == 1);
#pragma unroll
    for (int gidx = 0; gidx < G; ++gidx) decode_frag(gidx, 0);
    for (int s = 0; s < nstage; ++s) run_stage(s);
    wait_vmcnt<0>();                            // no copy may still be in flight when the LDS is released

    // ---- the KS partial tiles of a sub-tile are added through the LDS: in round rho every wave hands the fragments
    // owned by wave kh + rho (same sub-tile) over and adds what wave kh - rho left for it
    float* xch = reinterpret_cast<float*>(lds);
    auto region = [&](int k_share) { return xch + ((k_share * (GM * GN) + wq) * C::OWN) * 1024; };
#pragma unroll
    for (int rho = 1; rho < KS; ++rho) {
        const int dst = (kh + rho) % KS, src = (kh + KS - rho) % KS;
        wait_lgkmcnt0();                        // this wave's reads of the ring / of the previous round have returned
        wg_barrier();                           // ring (or the previous round's regions) no longer read by anyone
#pragma unroll
        for (int f = 0; f < WM * WN; ++f)
            if (f % KS == dst) {                // uniform over the wave
                float* slot = region(kh) + (f / KS) * 1024;
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    *reinterpret_cast<float4*>(slot + (q * 64 + lane) * 4) =
                        make_float4(acc[f / WN][f % WN][4 * q], acc[f / WN][f % WN][4 * q + 1], acc[f / WN][f % WN][4 * q + 2],
                                    acc[f / WN][f % WN][4 * q + 3]);
            }
        wait_lgkmcnt0();
        wg_barrier();
#pragma unroll
        for (int f = 0; f < WM * WN; ++f)
            if (f % KS == kh) {
                const float* slot = region(src) + (f / KS) * 1024;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float4 v = *reinterpret_cast<const float4*>(slot + (q * 64 + lane) * 4);
                    acc[f / WN][f % WN][4 * q] += v.x;
                    acc[f / WN][f % WN][4 * q + 1] += v.y;
                    acc[f / WN][f % WN][4 * q + 2] += v.z;
                    acc[f / WN][f % WN][4 * q + 3] += v.w;
                }
            }
    }
    const int m0 = wg_m0 + wrow0, n0 = wg_n0 + wcol0;
    const bool vec_ok = (ldy & (std::is_same<OutT, _Float16>::value ? 3 : 3)) == 0 &&
                        (reinterpret_cast<uintptr_t>(y) & (std::is_same<OutT, _Float16>::value ? 7 : 15)) == 0;
#pragma unroll
    for (int f = 0; f < WM * WN; ++f)
        if (f % KS == kh) store_fragment(acc[f / WN][f % WN], m0 + 32 * (f / WN), n0 + 32 * (f % WN), r, h, M, N, alpha, y, ldy, vec_ok);
}

template <int WM, int WN, int GM, int GN, int KS, bool REG, typename OutT>
arcq_status launch_ksplit(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* w_codes, const uint8_t* w_scales,
                          int M, int N, int nbk, float alpha, OutT* y, int64_t ldy, hipStream_t stream) {
    using C = KsplitCfg<WM, WN, GM, GN, KS>;
    auto kern = gemm_ksplit_kernel<WM, WN, GM, GN, KS, OutT, REG>;
    static std::atomic<uint64_t> lds_raised{0};
    if (arcq_status st = raise_lds_limit(reinterpret_cast<const void*>(kern), lds_raised)) return st;
    const int tiles_m = (M + C::BM - 1) / C::BM, tiles_n = (N + C::BN - 1) / C::BN;
    hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(C::NT), C::LDS_BYTES, stream, a_codes, a_scales, w_codes, w_scales,
                       M, N, nbk, alpha, y, ldy, tiles_m, tiles_n);
    return check_launch("gemm_ksplit_kernel");
}

template <bool REG, typename OutT>
arcq_status launch_ksplit_typed(int variant, const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* w_codes,
                                const uint8_t* w_scales, int M, int N, int nbk, float alpha, OutT* y, int64_t ldy,
                                hipStream_t stream) {
    switch (variant) {
        case 1: return launch_ksplit<2, 2, 1, 1, 4, REG>(a_codes, a_scales, w_codes, w_scales, M, N, nbk, alpha, y, ldy, stream);   // 64 x 64
        case 2: return launch_ksplit<4, 2, 1, 1, 4, REG>(a_codes, a_scales, w_codes, w_scales, M, N, nbk, alpha, y, ldy, stream);   // 128 x 64
        case 4: return launch_ksplit<3, 2, 1, 1, 4, REG>(a_codes, a_scales, w_codes, w_scales, M, N, nbk, alpha, y, ldy, stream);   // 96 x 64
        case 6: return launch_ksplit<2, 1, 1, 1, 4, REG>(a_codes, a_scales, w_codes, w_scales, M, N, nbk, alpha, y, ldy, stream);   // 64 x 32
        default: return launch_ksplit<2, 4, 2, 1, 4, REG>(a_codes, a_scales, w_codes, w_scales, M, N, nbk, alpha, y, ldy, stream);  // 128 x 128
    }
}

}  // namespace

// 0: not served here; 6: 64 x 32 tiles; 1: 64 x 64; 4: 96 x 64; 2: 128 x 64; 3: 128 x 128 (k quarters inside the workgroup each)
int gemm_ksplit_variant(int64_t M, int64_t N, int64_t Kp) {
    const int64_t nbk = Kp >> 4;
    if (nbk < 32) return 0;                               // at least two stages
    if ((uint64_t)M * (uint64_t)nbk * 8 >= 0xFFFF0000ull || (uint64_t)N * (uint64_t)nbk * 8 >= 0xFFFF0000ull) return 0;
    // The smallest tile that still covers the problem with at most one workgroup per compute unit (256), as long as
    // it occupies more than half of them (measured at 4096 x 4352, 14336 x 4352 and 4096 x 14592 weights, M = 128 ..
    // 1024: against the 128 x 128 tiles with K' split across workgroups these run 64 x 64 tiles 1.2-1.8x, 128 x 64
    // tiles 1.1-1.5x and 128 x 128 tiles 1.05-1.2x faster; with fewer tiles the split across workgroups wins, with
    // more the larger tiles of gemm.hip do).
    const int64_t m64 = (M + 63) / 64, m96 = (M + 95) / 96, m128 = (M + 127) / 128, n64 = (N + 63) / 64, n128 = (N + 127) / 128;
    auto fits = [](int64_t tiles) { return tiles >= 144 && tiles <= 256; };
    // the smallest tile also with fewer workgroups, for more than 64 rows and a short reduction (a tile takes 10.7 us
    // over K' = 4352, 17.3 over 8448, 27 over 14592 whatever their number; the alternatives, the eight-row-tile
    // streaming kernel and 128 x 128 tiles with K' split across workgroups, take 15-17, 21-29 and 24-26 us there)
    const int64_t t6 = m64 * ((N + 31) / 32);
    if (fits(t6) || (M > 64 && nbk <= 544 && t6 >= 32 && t6 <= 256)) return 6;
    if (fits(m64 * n64)) return 1;
    if (fits(m96 * n64)) return 4;
    if (fits(m128 * n64)) return 2;
    if (fits(m128 * n128)) return 3;
    return 0;
}

arcq_status launch_gemm_ksplit(int variant, const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* w_codes,
                               const uint8_t* w_scales, int64_t M, int64_t N, int64_t Kp, float alpha, void* y, int y_dtype,
                               int64_t ldy, hipStream_t stream) {
    const int nbk = (int)(Kp >> 4);
    // direct-to-LDS copies need rows that start on 16-byte boundaries (K' a multiple of 64 covers the scale bytes too)
    const bool copies = (nbk & 3) == 0 &&
                        ((reinterpret_cast<uintptr_t>(a_codes) | reinterpret_cast<uintptr_t>(w_codes)) & 15) == 0 &&
                        ((reinterpret_cast<uintptr_t>(a_scales) | reinterpret_cast<uintptr_t>(w_scales)) & 3) == 0;
    if (y_dtype == ARCQ_DTYPE_F16)
        return copies ? launch_ksplit_typed<false>(variant, a_codes, a_scales, w_codes, w_scales, (int)M, (int)N, nbk, alpha,
                                                   static_cast<_Float16*>(y), ldy, stream)
                      : launch_ksplit_typed<true>(variant, a_codes, a_scales, w_codes, w_scales, (int)M, (int)N, nbk, alpha,
                                                  static_cast<_Float16*>(y), ldy, stream);
    return copies ? launch_ksplit_typed<false>(variant, a_codes, a_scales, w_codes, w_scales, (int)M, (int)N, nbk, alpha,
                                               static_cast<float*>(y), ldy, stream)
                  : launch_ksplit_typed<true>(variant, a_codes, a_scales, w_codes, w_scales, (int)M, (int)N, nbk, alpha,
                                              static_cast<float*>(y), ldy, stream);
}

}  // namespace arcq
