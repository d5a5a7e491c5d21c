/*
 * arcq.h -- C ABI of libarcq: the ARCQuant hot path on AMD MI355X (gfx950).
 *
 * ARCQuant (arXiv 2601.07475) runs a W4A4 linear layer Y = X W^T in NVFP4 and
 * repairs the quantization error of the S largest-magnitude activation
 * channels by appending their quantized residual as S extra reduction columns,
 * so that one GEMM over K' = K + S computes
 *     Y ~= Q(X) Q(W)^T + Q(R_o) Q(W_o)^T                      (Section 3.2, eq. (2)).
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller.  The library
 *     never allocates, frees or synchronises; work is enqueued on `stream`
 *     (a hipStream_t passed as void*, NULL = the default stream) and results
 *     are valid in stream order.  Inputs are never modified.
 *   - Return value: ARCQ_OK or an error code; arcq_last_error() then holds a
 *     message.  Argument errors are detected before any HIP call is made.
 *   - NVFP4 (Appendix A, Table "formats"): elements are FP4 E2M1 (bias 1,
 *     magnitudes 0 .5 1 1.5 2 3 4 6), one FP8 E4M3 scale (bias 7, max 448,
 *     finite flavour) per block of 16 consecutive reordered channels, one
 *     FP32 scale per tensor.  Value = E2M1(code) * E4M3(scale byte) * tensor_scale.
 *   - Packed operand layout ("K' layout"), rows = M for activations, N for weights:
 *       codes  uint8 [rows, K'/2]   byte i of a row: element 2i in bits 0-3,
 *                                   element 2i+1 in bits 4-7; code = sign<<3 | index
 *       scales uint8 [rows, K'/16]  block b < K/16: primary block b;
 *                                   block K/16 + i: augmented block of primary
 *                                   block (K-S)/16 + i                 (Section 3.2 step (3))
 *     Rows are dense (pitch K'/2 and K'/16 bytes).
 *   - Shapes: K > 0, K % 16 == 0, 0 <= S <= K, S % 16 == 0, K <= ARCQ_MAX_K.
 *     rows may be 0 (nothing is launched).
 *   - Inputs must be finite; the result for NaN/Inf input is unspecified.
 */
#ifndef ARCQ_H
#define ARCQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int arcq_status;
#define ARCQ_OK                  0
#define ARCQ_INVALID_ARG         1   /* null pointer, tensor scale not finite / not in (2^-64, 2^64), bad dtype */
#define ARCQ_BAD_SHAPE           2   /* violates the shape rules above, or ld < row length */
#define ARCQ_BAD_ALIGN           3   /* pointer / leading dimension alignment, see each function */
#define ARCQ_HIP_ERROR           4   /* a launch failed; arcq_last_error() has the HIP message */
#define ARCQ_WORKSPACE_TOO_SMALL 5

#define ARCQ_MAX_K 65536             /* one fp16 row must fit the 160 KB LDS of a CU with room to spare */

#define ARCQ_DTYPE_F16 0
#define ARCQ_DTYPE_F32 1

/* flags of the *_ex entry points (0 = the behaviour of the plain entry points) */
#define ARCQ_LAYOUT_INTERLEAVED 1u   /* Appendix D "Interleaved Channel Layout" */
#define ARCQ_SCALE_ROUND_UP     2u   /* block scale never below max/q_max: alpha >= 1 of Section 3.4 */
#define ARCQ_RMSNORM_EXACT_SUM  4u   /* arcq_rmsnorm_quantize_act_ex only: see there */

/* Library version, major*10000 + minor*100 + patch. */
int arcq_version(void);

/* Message of the last error on the calling thread ("" if none).  The string is
 * thread-local storage of the library; do not free it. */
const char* arcq_last_error(void);

/* Bytes a caller must allocate for a packed operand of `rows` rows:
 *   *codes_bytes = rows*(K+S)/2, *scales_bytes = rows*(K+S)/16.   Host arithmetic only. */
arcq_status arcq_packed_sizes(int64_t rows, int64_t K, int64_t S,
                              size_t* codes_bytes, size_t* scales_bytes);

/*
 * Online activation quantizer, one fused pass (Section 3.2 "Online Activation
 * Quantization" steps (1)-(3); Section 3.3 fused kernel without the RMSNorm):
 *   (1) reorder: Xp[m, j] = x[m, perm[j]]; per block of 16: scale byte =
 *       E4M3(amax / (6 * tensor_scale)), codes = E2M1(Xp / s), s = E4M3 value * tensor_scale
 *       (Section 3.1 eq. (1), round-to-nearest-even, saturating);
 *   (2) on the last S reordered channels: r = Xp - s * Q, quantized the same way
 *       with the same tensor_scale;
 *   (3) output [Q_X | Q_R], [s_X | s_R] in the K' layout.
 * x       fp16 [M, K], row pitch ldx elements (ldx >= K); x 16-byte aligned, ldx % 8 == 0
 * perm    int32 [K], 16-byte aligned, a permutation of 0..K-1 (not checked; see arcq_check_perm):
 *         reordered position j takes source channel perm[j]; outliers are the LAST S positions.
 *         With entries outside 0..K-1 the output is unspecified; no global memory outside the
 *         arguments is touched.
 * codes   out, uint8 [M, (K+S)/2], 8-byte aligned;  scales out, uint8 [M, (K+S)/16]
 */
arcq_status arcq_quantize_act(const void* x, int64_t M, int64_t K, int64_t ldx,
                              const int32_t* perm, int64_t S, float tensor_scale,
                              uint8_t* codes, uint8_t* scales, void* stream);

/*
 * The same quantizer with RMSNorm in front, as one kernel (Section 3.3: the fused quantization
 * kernel integrates channel reordering, RMSNorm, primary and residual quantization).  The paper
 * gives no formula; this is y = x / sqrt(mean(x^2) + eps) * gamma with the roundings of the
 * reference layer: the mean of squares is defined with an EXACT sum of the squares (no summation order
 * enters the result), rounded once to fp64, divided by K in fp64 and rounded to fp32; rstd =
 * 1/sqrt(ms + eps) in fp32 (correctly rounded square root and division); x * rstd is rounded to fp32 and
 * then to fp16; times gamma, rounded once to fp16.  The result equals arcq_quantize_act applied to that
 * fp16 tensor.  tensor_scale refers to the NORMALISED activations.
 * gamma  fp16 [K], indexed by SOURCE channel (before the permutation), 16-byte aligned
 * eps    finite, >= 0
 */
arcq_status arcq_rmsnorm_quantize_act(const void* x, int64_t M, int64_t K, int64_t ldx,
                                      const void* gamma, float eps,
                                      const int32_t* perm, int64_t S, float tensor_scale,
                                      uint8_t* codes, uint8_t* scales, void* stream);

/*
 * Offline weight packer (Section 3.2 "Offline Weight Quantization"): reorder the
 * K axis of w with the same perm, quantize every block of 16 (plain
 * round-to-nearest), then append a verbatim copy of the codes and scale bytes of
 * the last S reordered channels: Q_Waug = [Q_W | Q_Wo].
 * w  fp16 [N, K] (nn.Linear layout, Y = X W^T), row pitch ldw; same alignment rules as x.
 */
arcq_status arcq_pack_weight(const void* w, int64_t N, int64_t K, int64_t ldw,
                             const int32_t* perm, int64_t S, float tensor_scale,
                             uint8_t* codes, uint8_t* scales, void* stream);

/*
 * Variants of the three calls above, selected by `flags` (an OR of the ARCQ_LAYOUT_ / ARCQ_SCALE_ bits;
 * any other bit is ARCQ_INVALID_ARG; flags = 0 is the plain call).  Everything else, sizes included, is
 * unchanged.  Both operands of a GEMM must be packed with the same flags.
 *
 * ARCQ_LAYOUT_INTERLEAVED (Appendix D "Interleaved Channel Layout"): the same blocks in another physical
 *   order along K'.  The (K-S)/16 blocks without compensation come first, in order; then every outlier
 *   block is immediately followed by its partner (its quantized residual for activations, its verbatim
 *   copy for weights): primary block (K-S)/16 + i sits at block position (K-S)/16 + 2i, its partner at
 *   (K-S)/16 + 2i + 1, for codes and scale bytes alike.  arcq_gemm reduces over K' in any order, so the
 *   product is the one of the plain layout up to the order of the fp32 sums.
 * ARCQ_SCALE_ROUND_UP (Section 3.4 takes the ratio alpha of the stored block scale to max/q_max in
 *   [1, 1.125]; Section 3.1 eq. (1) leaves the rounding open): the scale byte is the smallest E4M3 value
 *   not below amax / (6 * tensor_scale) instead of the nearest one, for primary and residual blocks, so no
 *   element saturates at 6; it still saturates at 448, and a nonzero quotient below the smallest subnormal
 *   2^-9 gets 2^-9 rather than 0.
 * ARCQ_RMSNORM_EXACT_SUM (arcq_rmsnorm_quantize_act_ex only; elsewhere ARCQ_INVALID_ARG): the kernel normally sums
 *   the squares of a row in fp64 and falls back to an exact integer sum for the rare row whose mean it cannot
 *   round with certainty; this bit sends EVERY row through the integer sum.  The output is identical by
 *   construction (that is what the bit lets a caller verify); the call is slower.
 */
arcq_status arcq_quantize_act_ex(const void* x, int64_t M, int64_t K, int64_t ldx,
                                 const int32_t* perm, int64_t S, float tensor_scale, uint32_t flags,
                                 uint8_t* codes, uint8_t* scales, void* stream);
arcq_status arcq_rmsnorm_quantize_act_ex(const void* x, int64_t M, int64_t K, int64_t ldx,
                                         const void* gamma, float eps,
                                         const int32_t* perm, int64_t S, float tensor_scale, uint32_t flags,
                                         uint8_t* codes, uint8_t* scales, void* stream);
arcq_status arcq_pack_weight_ex(const void* w, int64_t N, int64_t K, int64_t ldw,
                                const int32_t* perm, int64_t S, float tensor_scale, uint32_t flags,
                                uint8_t* codes, uint8_t* scales, void* stream);

/* Bytes of workspace arcq_gemm needs for this problem (may be 0).  Host arithmetic only. */
arcq_status arcq_gemm_workspace_size(int64_t M, int64_t N, int64_t Kp, size_t* bytes);

/*
 * The single GEMM over the extended reduction dimension (Section 3.2 "Unified
 * GEMM Execution", eq. (2)):
 *   y[m, n] = a_tensor_scale * w_tensor_scale *
 *             sum_{b < Kp/16} sa[m,b] * sw[n,b] * sum_{i<16} qa[m,16b+i] * qw[n,16b+i]
 * with fp32 accumulation.  Operands are decoded exactly (every code*scale
 * product fits fp16) and multiplied on the fp16 MFMA path.
 * a_*  packed activations [M, Kp] from arcq_quantize_act;  w_*  packed weights [N, Kp]
 *      from arcq_pack_weight; codes 8-byte aligned.  Kp % 16 == 0, Kp > 0.  Every such Kp and alignment runs
 *      on the tiled / weight-streaming kernels; Kp % 64 == 0 with 16-byte aligned codes and 4-byte aligned
 *      scales additionally lets the tiled kernels copy straight into LDS (up to 1.35x faster on large M).
 * y    out [M, N] row-major, pitch ldy elements (ldy >= N), y_dtype ARCQ_DTYPE_F16 / _F32,
 *      4-byte aligned (16-byte aligned with ldy % 8 == 0 lets the tiled kernels store whole lines).
 * workspace  device scratch of at least arcq_gemm_workspace_size bytes, 256-byte
 *      aligned (may be NULL when that size is 0); contents undefined afterwards.
 */
arcq_status arcq_gemm(const uint8_t* a_codes, const uint8_t* a_scales, float a_tensor_scale,
                      const uint8_t* w_codes, const uint8_t* w_scales, float w_tensor_scale,
                      int64_t M, int64_t N, int64_t Kp,
                      void* y, int y_dtype, int64_t ldy,
                      void* workspace, size_t workspace_bytes, void* stream);

/*
 * arcq_gemm for callers that cannot allocate device memory for a workspace (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): same arguments minus the workspace, same kernels, same
 * result bit for bit.  The fp32 partial results of a split reduction dimension go to a buffer of
 * ARCQ_NOALLOC_SCRATCH_BYTES that is part of the library image (every GPU the library runs on holds its own
 * copy until the process ends); the call allocates and frees nothing.
 *   - Shapes whose arcq_gemm_workspace_size exceeds ARCQ_NOALLOC_SCRATCH_BYTES are rejected with
 *     ARCQ_WORKSPACE_TOO_SMALL (use arcq_gemm with a workspace of the caller); checked before any HIP call.
 *   - The device of `stream` must be the calling thread's current device.  The first call on a device that needs
 *     scratch looks the buffer's address up once (hipGetSymbolAddress); make that call outside a graph capture.
 *   - All calls on one GPU share the buffer: calls that may overlap (different streams, or graphs replayed
 *     concurrently) race on it; order them.  Nothing in it has to start at zero (every partial result is written
 *     before it is read), and its contents are undefined afterwards.
 */
#define ARCQ_NOALLOC_SCRATCH_BYTES (8u << 20)
arcq_status arcq_gemm_noalloc(const uint8_t* a_codes, const uint8_t* a_scales, float a_tensor_scale,
                              const uint8_t* w_codes, const uint8_t* w_scales, float w_tensor_scale,
                              int64_t M, int64_t N, int64_t Kp,
                              void* y, int y_dtype, int64_t ldy, void* stream);

/*
 * Debug helper: checks on the device that perm[0..K-1] is a permutation of 0..K-1
 * (the calibration output of Section 3.2 "Adaptive Outlier Identification").
 * flags: device scratch, K bytes.  *result_host is written after the stream has been
 * synchronised by this call: 1 = valid, 0 = not a permutation.
 */
arcq_status arcq_check_perm(const int32_t* perm, int64_t K, uint8_t* flags,
                            int* result_host, void* stream);

/*
 * Offline calibration (Section 3.2 "Adaptive Outlier Identification"), two calls.
 *
 * arcq_calib_absmax folds one batch of calibration activations into the running per-channel
 * statistic: colmax[k] = max(colmax[k], max over rows of |x[m, k]|).  Batches may come in any order.
 * x       fp16 [M, K], row pitch ldx (same alignment rules as arcq_quantize_act); M may be 0
 * colmax  in/out, fp32 [K], 4-byte aligned; the caller fills it with zeros before the first batch;
 *         values stay >= 0.  Concurrent calls on the same colmax are safe (atomic maxima).
 *
 * arcq_calib_select turns the statistic into what the quantizer and the weight packer consume:
 *   perm  out, int32 [K]: channels in ascending order of colmax, equal values by ascending channel
 *         index, so the outliers are the last positions (the sorting strategy the paper adopts);
 *   info  out, int32 [4] on the device: {S, S_raw, bit pattern of the layer maximum (fp32),
 *         bit pattern of tau = 2^-3 * maximum}.  S_raw = number of channels with colmax > tau
 *         (a channel AT the threshold needs no compensation); S = S_raw rounded up to a multiple
 *         of 16, at most K (this library works on blocks of 16; the paper does not say).
 *   S_host  if not NULL the call synchronises the stream and stores S there; if NULL nothing is
 *         synchronised and the caller reads info in stream order.
 * colmax must hold finite values >= 0 (what arcq_calib_absmax produces); K as everywhere else.
 */
arcq_status arcq_calib_absmax(const void* x, int64_t M, int64_t K, int64_t ldx,
                              float* colmax, void* stream);
arcq_status arcq_calib_select(const float* colmax, int64_t K, int32_t* perm, int32_t* info,
                              int* S_host, void* stream);

/*
 * MXFP4 variant of the same path (the paper reports the method on MXFP4 as well: Section 4.3
 * "Generalizability" and the appendix table on INT4 and MXFP4).  Format (Section 3.1 "Block-scaled
 * Quantization", Appendix A): 32 E2M1 elements per block, one E8M0 scale byte per block (value
 * 2^(byte - 127)), no tensor scale.  Scale rule (the paper gives none; this is the rule of the OCP
 * Microscaling specification it cites): shared exponent = floor(log2(block maximum)) - 2; elements round
 * to nearest even on the E2M1 grid and saturate at 6; an all-zero block gets byte 127.  Residual channels,
 * their placement and the duplicated weight blocks are those of Section 3.2 with blocks of 32:
 *   codes  uint8 [rows, K'/2]  (element 2i in bits 0-3 of byte i), 16-byte aligned
 *   scales uint8 [rows, K'/32] block b < K/32 primary, block K/32 + i the augmented block of primary
 *                              block (K-S)/32 + i
 * Shapes: K % 32 == 0, S % 32 == 0, 0 <= S <= K <= ARCQ_MAX_K.  x / w, perm as in the NVFP4 calls, perm
 * 16-byte aligned.  This is the block format gfx950's scaled FP4 matrix instruction multiplies natively,
 * so arcq_mx_gemm needs no decode:
 *   y[m, n] = sum_b 2^(sa[m,b]-127) 2^(sw[n,b]-127) sum_{i<32} qa[m,32b+i] qw[n,32b+i],  fp32 accumulation
 * (Section 3.2 eq. (2)); Kp % 32 == 0; codes 4-byte aligned.  Every such shape runs on the tiled /
 * weight-streaming kernels; 16-byte aligned codes, 4-byte aligned scales and Kp % 128 == 0 additionally let
 * the tiled kernels copy straight into LDS (about 1.5x faster on large M); y as in arcq_gemm.  No workspace (see arcq_mx_gemm_ws below).
 */
arcq_status arcq_mx_packed_sizes(int64_t rows, int64_t K, int64_t S,
                                 size_t* codes_bytes, size_t* scales_bytes);
arcq_status arcq_mx_quantize_act(const void* x, int64_t M, int64_t K, int64_t ldx,
                                 const int32_t* perm, int64_t S,
                                 uint8_t* codes, uint8_t* scales, void* stream);
arcq_status arcq_mx_pack_weight(const void* w, int64_t N, int64_t K, int64_t ldw,
                                const int32_t* perm, int64_t S,
                                uint8_t* codes, uint8_t* scales, void* stream);
arcq_status arcq_mx_gemm(const uint8_t* a_codes, const uint8_t* a_scales,
                         const uint8_t* w_codes, const uint8_t* w_scales,
                         int64_t M, int64_t N, int64_t Kp,
                         void* y, int y_dtype, int64_t ldy, void* stream);
/*
 * arcq_mx_gemm with a workspace: problems with few output tiles and a long reduction dimension (a few hundred
 * rows against a down-projection) split K' into runs whose fp32 partial results go through the workspace and are
 * added in index order by a second kernel (same result up to the order of the fp32 additions).
 * arcq_mx_gemm_workspace_size: bytes needed for this shape (may be 0; host arithmetic only).
 * workspace  device scratch of at least that many bytes, 256-byte aligned; may be null when 0 bytes are needed.
 *            ARCQ_WORKSPACE_TOO_SMALL otherwise.  Calls that share a workspace must not overlap.
 */
arcq_status arcq_mx_gemm_workspace_size(int64_t M, int64_t N, int64_t Kp, size_t* bytes);
arcq_status arcq_mx_gemm_ws(const uint8_t* a_codes, const uint8_t* a_scales,
                            const uint8_t* w_codes, const uint8_t* w_scales,
                            int64_t M, int64_t N, int64_t Kp,
                            void* y, int y_dtype, int64_t ldy,
                            void* workspace, size_t workspace_bytes, void* stream);

/*
 * The same two variants for MXFP4 (flags as for arcq_quantize_act_ex, blocks of 32):
 * ARCQ_LAYOUT_INTERLEAVED puts primary block (K-S)/32 + i at block position (K-S)/32 + 2i and its partner
 * right behind it (Appendix D); ARCQ_SCALE_ROUND_UP takes the smallest power of two X with
 * block maximum <= 6 X (one step above the floor rule exactly when the maximum's significand exceeds 1.5),
 * so no element saturates (alpha >= 1, Section 3.4).
 */
arcq_status arcq_mx_quantize_act_ex(const void* x, int64_t M, int64_t K, int64_t ldx,
                                    const int32_t* perm, int64_t S, uint32_t flags,
                                    uint8_t* codes, uint8_t* scales, void* stream);
arcq_status arcq_mx_pack_weight_ex(const void* w, int64_t N, int64_t K, int64_t ldw,
                                   const int32_t* perm, int64_t S, uint32_t flags,
                                   uint8_t* codes, uint8_t* scales, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ARCQ_H */
