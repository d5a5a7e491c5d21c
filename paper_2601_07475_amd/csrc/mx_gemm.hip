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
#include "lds_dma.h"

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

// Staged kernel for K' % 128 == 0.  A stage is 128 k: per row 64 bytes of codes (four 16-byte pieces =
// four MX blocks) and 4 scale bytes; stages travel global -> LDS with global_load_lds through a ring of
// three buffers, one barrier per stage.  LDS layout of one stage: A codes [BM][64] | W codes [BN][64] |
// A scales [BM] dwords | W scales [BN] dwords (regions padded to whole workgroup-wide copies).  The four
// pieces of a row are stored XOR-swizzled with (row >> 1) & 3, applied by choosing which global piece a
// lane fetches (a wave-wide copy writes lane l to base + 16 l).
template <int WM, int WN, int GM, int GN>
struct MxCfg {
    static constexpr int BM = 32 * WM * GM, BN = 32 * WN * GN;
    static constexpr int NT = 64 * GM * GN;
    static constexpr int NA = (BM * 4 + NT - 1) / NT, NW = (BN * 4 + NT - 1) / NT;
    static constexpr int NAS = (BM + NT - 1) / NT, NWS = (BN + NT - 1) / NT;
    static constexpr int NDMA = NA + NW + NAS + NWS;
    static constexpr int A_CODES = 0;
    static constexpr int W_CODES = NA * NT * 16;
    static constexpr int A_SCALES = W_CODES + NW * NT * 16;
    static constexpr int W_SCALES = A_SCALES + NAS * NT * 4;
    static constexpr int STAGE_BYTES = W_SCALES + NWS * NT * 4;
    static constexpr int NSTAGE = 3;
    static constexpr int LDS_BYTES = NSTAGE * STAGE_BYTES;
};

template <int WM, int WN, int GM, int GN, typename OutT>
__global__ __launch_bounds__(64 * GM * GN) void mx_gemm_staged_kernel(
    const uint8_t* __restrict__ a_codes, const uint8_t* __restrict__ a_scales,
    const uint8_t* __restrict__ w_codes, const uint8_t* __restrict__ w_scales, int M, int N, int nstage,
    OutT* __restrict__ y, int64_t ldy, int tiles_m, int tiles_n) {
    using C = MxCfg<WM, WN, GM, GN>;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

    // workgroup -> tile: a contiguous run of the tile sequence per XCD, column-major groups of 8 tile rows
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

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane & 31, h = lane >> 5;
    const int wg_m0 = tile_m * C::BM, wg_n0 = tile_n * C::BN;
    const int wrow0 = (wave / GN) * (32 * WM), wcol0 = (wave % GN) * (32 * WN);

    // ---- copies: thread -> (row, piece) of a workgroup-wide copy
    const uint32_t cpitch = (uint32_t)nstage * 64u, spitch = (uint32_t)nstage * 4u;
    const uint32_t lp = (uint32_t)((tid & 3) ^ ((tid >> 3) & 3)) * 16u;      // global piece this lane fetches
    const int crow = tid >> 2;
    const uint32_t wave_slot = __builtin_amdgcn_readfirstlane((uint32_t)(tid & ~63));
    const uint32_t lds0 = lds_address(lds);
    auto issue_one = [&](int d, int stage, int buf) {
        const uint32_t base = lds0 + buf * C::STAGE_BYTES;
        constexpr int NA = C::NA, NW = C::NW, NAS = C::NAS, NT = C::NT;
        // rows past the edge of the operand re-read its last row (never stored)
        if (d < NA) {
            const uint32_t row = (uint32_t)min(wg_m0 + d * (NT / 4) + crow, M - 1);
            dma16(a_codes, row * cpitch + (uint32_t)stage * 64u + lp, base + C::A_CODES + 16u * (d * NT + wave_slot));
        } else if (d < NA + NW) {
            const int p = d - NA;
            const uint32_t row = (uint32_t)min(wg_n0 + p * (NT / 4) + crow, N - 1);
            dma16(w_codes, row * cpitch + (uint32_t)stage * 64u + lp, base + C::W_CODES + 16u * (p * NT + wave_slot));
        } else if (d < NA + NW + NAS) {
            const int p = d - NA - NW;
            const uint32_t row = (uint32_t)min(wg_m0 + p * NT + tid, M - 1);
            dma4(a_scales, row * spitch + (uint32_t)stage * 4u, base + C::A_SCALES + 4u * (p * NT + wave_slot));
        } else {
            const int p = d - NA - NW - NAS;
            const uint32_t row = (uint32_t)min(wg_n0 + p * NT + tid, N - 1);
            dma4(w_scales, row * spitch + (uint32_t)stage * 4u, base + C::W_SCALES + 4u * (p * NT + wave_slot));
        }
    };

    // ---- LDS read offsets of this lane: piece 2t + h of its rows, physical position XOR (row >> 1) & 3
    const uint32_t swz = (uint32_t)(r >> 1) & 3u;
    const uint32_t rd_a = C::A_CODES + (wrow0 + r) * 64, rd_w = C::W_CODES + (wcol0 + r) * 64;
    const uint32_t rd_as = C::A_SCALES + (wrow0 + r) * 4, rd_ws = C::W_SCALES + (wcol0 + r) * 4;
    const uint32_t pc[2] = {16u * ((uint32_t)h ^ swz), 16u * ((2u + (uint32_t)h) ^ swz)};

    float16v acc[WM][WN];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    uint4 fa[2][WM], fw[2][WN];             // fragments of k-step 0 and 1 of the current stage
    int sa[WM], sw[WN], sa_n[WM], sw_n[WN]; // scale registers (already shifted so that byte 2t is the lane's)
    auto read_codes = [&](int t, const uint8_t* st) {
#pragma unroll
        for (int i = 0; i < WM; ++i) fa[t][i] = *reinterpret_cast<const uint4*>(st + rd_a + i * 2048 + pc[t]);
#pragma unroll
        for (int j = 0; j < WN; ++j) fw[t][j] = *reinterpret_cast<const uint4*>(st + rd_w + j * 2048 + pc[t]);
    };
    auto read_scales = [&](const uint8_t* st, int (&da)[WM], int (&dw)[WN]) {
#pragma unroll
        for (int i = 0; i < WM; ++i) da[i] = (int)(*reinterpret_cast<const uint32_t*>(st + rd_as + i * 128) >> (8 * h));
#pragma unroll
        for (int j = 0; j < WN; ++j) dw[j] = (int)(*reinterpret_cast<const uint32_t*>(st + rd_ws + j * 128) >> (8 * h));
    };
    auto mfmas = [&](int t, int first, int count) {     // MFMAs first .. first+count-1 of k-step t (row-major over i, j)
#pragma unroll
        for (int q = first; q < first + count; ++q) {
            const int i = q / WN, j = q % WN;
            // weights as the row operand: see store_tile_swapped
            acc[i][j] = mfma_mx(fw[t][j], fa[t][i], acc[i][j], sw[j], sa[i], t);
        }
    };

    // ---- pipeline: the copies of stage s+2 are issued during stage s (its buffer was last read in stage
    // s-1, which every wave left before the barrier inside stage s-1); the barrier that opens stage s+1 and the
    // reads of its first fragments sit before the last half of the MFMAs of stage s.
    constexpr int HALF = (WM * WN) / 2;
    issue_one(0, 0, 0);
#pragma unroll
    for (int d = 1; d < C::NDMA; ++d) issue_one(d, 0, 0);
#pragma unroll
    for (int d = 0; d < C::NDMA; ++d) issue_one(d, min(1, nstage - 1), 1);
    wait_vmcnt<C::NDMA>();
    wg_barrier();
    read_codes(0, lds);
    read_scales(lds, sa, sw);
    int buf = 0;
    for (int s = 0; s < nstage; ++s) {
        const uint8_t* st = lds + buf * C::STAGE_BYTES;
        const int buf1 = buf == 2 ? 0 : buf + 1, buf2 = buf == 0 ? 2 : buf - 1;
        const int fetch = min(s + 2, nstage - 1);
        read_codes(1, st);
#pragma unroll
        for (int d = 0; d < C::NDMA / 2; ++d) issue_one(d, fetch, buf2);
        mfmas(0, 0, WM * WN);
#pragma unroll
        for (int d = C::NDMA / 2; d < C::NDMA; ++d) issue_one(d, fetch, buf2);
        mfmas(1, 0, HALF);
        // stage s+1 must have landed: this stage's own copies are younger
        wait_vmcnt<C::NDMA>();
        wg_barrier();
        read_codes(0, lds + buf1 * C::STAGE_BYTES);
        read_scales(lds + buf1 * C::STAGE_BYTES, sa_n, sw_n);
        mfmas(1, HALF, WM * WN - HALF);
#pragma unroll
        for (int i = 0; i < WM; ++i) sa[i] = sa_n[i];
#pragma unroll
        for (int j = 0; j < WN; ++j) sw[j] = sw_n[j];
        buf = buf1;
    }
    wait_vmcnt<0>();                            // no copy may still be in flight when the LDS is released

    const int m0 = wg_m0 + wrow0, n0 = wg_n0 + wcol0;
    const bool vec_ok = (ldy & 3) == 0 && (reinterpret_cast<uintptr_t>(y) & 15) == 0;
    store_tile_swapped<WM, WN>(acc, m0, n0, r, h, M, N, 1.0f, y, ldy, vec_ok);
}

// Fallback for any K' (multiple of 32) and any alignment the API admits: operands straight from global
// memory, one 64 x 64 tile per wave.  A k-step is two blocks; when the block count is odd the upper
// half of the lanes contributes zero codes in the last step.
template <typename OutT>
__global__ __launch_bounds__(256) void mx_gemm_direct_kernel(
    const uint8_t* __restrict__ a_codes, const uint8_t* __restrict__ a_scales,
    const uint8_t* __restrict__ w_codes, const uint8_t* __restrict__ w_scales, int M, int N, int nb,
    OutT* __restrict__ y, int64_t ldy) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
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

template <int WM, int WN, int GM, int GN, typename OutT>
arcq_status launch_mx_staged(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* w_codes,
                             const uint8_t* w_scales, int M, int N, int nstage, OutT* y, int64_t ldy, hipStream_t stream) {
    using C = MxCfg<WM, WN, GM, GN>;
    auto kern = mx_gemm_staged_kernel<WM, WN, GM, GN, OutT>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
    if (e != hipSuccess) return fail(ARCQ_HIP_ERROR, "hipFuncSetAttribute(LDS=%d): %s", C::LDS_BYTES, hipGetErrorString(e));
    const int tiles_m = (M + C::BM - 1) / C::BM, tiles_n = (N + C::BN - 1) / C::BN;
    hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(C::NT), C::LDS_BYTES, stream, a_codes, a_scales, w_codes,
                       w_scales, M, N, nstage, y, ldy, tiles_m, tiles_n);
    return check_launch("mx_gemm_staged_kernel");
}

template <typename OutT>
arcq_status launch_mx_typed(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* w_codes,
                            const uint8_t* w_scales, int64_t M, int64_t N, int64_t Kp, OutT* y, int64_t ldy,
                            hipStream_t stream) {
    const int nb = (int)(Kp >> 5);
    const bool offsets_fit = (uint64_t)M * (uint64_t)nb * 16 < 0xFFFF0000ull && (uint64_t)N * (uint64_t)nb * 16 < 0xFFFF0000ull;
    const bool aligned16 = ((reinterpret_cast<uintptr_t>(a_codes) | reinterpret_cast<uintptr_t>(w_codes)) & 15) == 0 &&
                           ((reinterpret_cast<uintptr_t>(a_scales) | reinterpret_cast<uintptr_t>(w_scales)) & 3) == 0;
    if ((nb & 3) == 0 && offsets_fit && aligned16) {
        const int nstage = nb >> 2;
        const int64_t t256 = ((M + 255) / 256) * ((N + 255) / 256);
        if (t256 >= 256)
            return launch_mx_staged<4, 4, 2, 2>(a_codes, a_scales, w_codes, w_scales, (int)M, (int)N, nstage, y, ldy, stream);
        const int64_t t128x256 = ((M + 127) / 128) * ((N + 255) / 256);
        if (t128x256 >= 192)
            return launch_mx_staged<2, 4, 2, 2>(a_codes, a_scales, w_codes, w_scales, (int)M, (int)N, nstage, y, ldy, stream);
        return launch_mx_staged<2, 2, 2, 2>(a_codes, a_scales, w_codes, w_scales, (int)M, (int)N, nstage, y, ldy, stream);
    }
    dim3 grid((unsigned)((N + 127) / 128), (unsigned)((M + 127) / 128));
    hipLaunchKernelGGL(mx_gemm_direct_kernel<OutT>, grid, dim3(256), 0, stream, a_codes, a_scales, w_codes, w_scales,
                       (int)M, (int)N, nb, y, ldy);
    return check_launch("mx_gemm_direct_kernel");
}

}  // namespace

arcq_status launch_mx_gemm(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* w_codes,
                           const uint8_t* w_scales, int64_t M, int64_t N, int64_t Kp, void* y, int y_dtype, int64_t ldy,
                           hipStream_t stream) {
    if (y_dtype == ARCQ_DTYPE_F16)
        return launch_mx_typed<_Float16>(a_codes, a_scales, w_codes, w_scales, M, N, Kp, static_cast<_Float16*>(y), ldy, stream);
    return launch_mx_typed<float>(a_codes, a_scales, w_codes, w_scales, M, N, Kp, static_cast<float*>(y), ldy, stream);
}

}  // namespace arcq
