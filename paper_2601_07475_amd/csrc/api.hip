// C entry points of libarcq: argument validation (before any HIP call), then launch.
#include "internal.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>

namespace arcq {

namespace {
thread_local char g_err[512] = "";
}

arcq_status fail(arcq_status code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

void clear_error() { g_err[0] = '\0'; }

arcq_status check_launch(const char* what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(ARCQ_HIP_ERROR, "%s: %s", what, hipGetErrorString(e));
    return ARCQ_OK;
}

arcq_status raise_lds_limit(const void* kernel, std::atomic<uint64_t>& done) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(ARCQ_HIP_ERROR, "hipGetDevice: %s", hipGetErrorString(e));
    const uint64_t bit = 1ull << (dev & 63);
    if (done.load(std::memory_order_acquire) & bit) return ARCQ_OK;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes);
    if (e != hipSuccess) return fail(ARCQ_HIP_ERROR, "hipFuncSetAttribute(LDS=%d): %s", kMaxLdsBytes, hipGetErrorString(e));
    if (dev < 64) done.fetch_or(bit, std::memory_order_release);      // devices past 63 set it on every launch
    return ARCQ_OK;
}

int num_cu() {
    static std::atomic<int> cached[64];
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    if (dev >= 0 && dev < 64 && (n = cached[dev].load(std::memory_order_relaxed)) > 0) return n;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
    if (dev >= 0 && dev < 64) cached[dev].store(n, std::memory_order_relaxed);
    return n;
}

namespace {

bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

arcq_status check_scale(float s, const char* name) {
    if (!std::isfinite(s) || !(s > 0x1p-64f) || !(s < 0x1p64f))
        return fail(ARCQ_INVALID_ARG, "%s = %g: must be finite and within (2^-64, 2^64)", name, (double)s);
    return ARCQ_OK;
}

arcq_status check_flags(uint32_t flags, const char* who, uint32_t also_allowed = 0) {
    if (flags & ~(uint32_t)(ARCQ_LAYOUT_INTERLEAVED | ARCQ_SCALE_ROUND_UP | also_allowed))
        return fail(ARCQ_INVALID_ARG, "%s: unknown bits in flags = 0x%x", who, flags);
    return ARCQ_OK;
}

arcq_status check_KS(int64_t K, int64_t S) {
    if (K <= 0 || (K % 16) != 0) return fail(ARCQ_BAD_SHAPE, "K = %lld: must be > 0 and a multiple of 16", (long long)K);
    if (K > ARCQ_MAX_K) return fail(ARCQ_BAD_SHAPE, "K = %lld exceeds ARCQ_MAX_K = %d", (long long)K, ARCQ_MAX_K);
    if (S < 0 || S > K || (S % 16) != 0)
        return fail(ARCQ_BAD_SHAPE, "S = %lld: must satisfy 0 <= S <= K and S %% 16 == 0", (long long)S);
    return ARCQ_OK;
}

arcq_status quantize_entry(int mode, const char* who, const void* x, int64_t rows, int64_t K, int64_t ldx,
                           const int32_t* perm, int64_t S, float s_T, uint8_t* codes, uint8_t* scales,
                           void* stream, bool norm = false, const void* gamma = nullptr, float eps = 0.0f,
                           uint32_t flags = 0) {
    clear_error();
    if (arcq_status st = check_KS(K, S)) return st;
    if (arcq_status st = check_flags(flags, who, norm ? ARCQ_RMSNORM_EXACT_SUM : 0u)) return st;
    if (rows < 0 || rows > 0x7FFFFFFF) return fail(ARCQ_BAD_SHAPE, "%s: rows = %lld out of range", who, (long long)rows);
    if (ldx < K) return fail(ARCQ_BAD_SHAPE, "%s: leading dimension %lld < K = %lld", who, (long long)ldx, (long long)K);
    if (arcq_status st = check_scale(s_T, "tensor_scale")) return st;
    if (norm && (!std::isfinite(eps) || eps < 0.0f)) return fail(ARCQ_INVALID_ARG, "%s: eps = %g must be finite and >= 0", who, (double)eps);
    if (rows == 0) return ARCQ_OK;
    if (!x || !perm || !codes || !scales || (norm && !gamma)) return fail(ARCQ_INVALID_ARG, "%s: null pointer", who);
    if (norm && !aligned(gamma, 16)) return fail(ARCQ_BAD_ALIGN, "%s: gamma must be 16-byte aligned", who);
    if (!aligned(x, 16) || (ldx % 8) != 0)
        return fail(ARCQ_BAD_ALIGN, "%s: input must be 16-byte aligned with a leading dimension that is a multiple of 8", who);
    if (!aligned(codes, 8)) return fail(ARCQ_BAD_ALIGN, "%s: codes must be 8-byte aligned", who);
    if (!aligned(perm, 16)) return fail(ARCQ_BAD_ALIGN, "%s: perm must be 16-byte aligned", who);
    return launch_quantize(mode, x, rows, K, ldx, perm, S, s_T, codes, scales, norm ? gamma : nullptr, eps, flags,
                           static_cast<hipStream_t>(stream));
}

arcq_status check_KS_mx(int64_t K, int64_t S) {
    if (K <= 0 || (K % 32) != 0) return fail(ARCQ_BAD_SHAPE, "K = %lld: must be > 0 and a multiple of 32", (long long)K);
    if (K > ARCQ_MAX_K) return fail(ARCQ_BAD_SHAPE, "K = %lld exceeds ARCQ_MAX_K = %d", (long long)K, ARCQ_MAX_K);
    if (S < 0 || S > K || (S % 32) != 0)
        return fail(ARCQ_BAD_SHAPE, "S = %lld: must satisfy 0 <= S <= K and S %% 32 == 0", (long long)S);
    return ARCQ_OK;
}

arcq_status mx_quantize_entry(int mode, const char* who, const void* x, int64_t rows, int64_t K, int64_t ldx,
                              const int32_t* perm, int64_t S, uint8_t* codes, uint8_t* scales, void* stream,
                              uint32_t flags = 0) {
    clear_error();
    if (arcq_status st = check_KS_mx(K, S)) return st;
    if (arcq_status st = check_flags(flags, who)) return st;
    if (rows < 0 || rows > 0x7FFFFFFF) return fail(ARCQ_BAD_SHAPE, "%s: rows = %lld out of range", who, (long long)rows);
    if (ldx < K) return fail(ARCQ_BAD_SHAPE, "%s: leading dimension %lld < K = %lld", who, (long long)ldx, (long long)K);
    if (rows == 0) return ARCQ_OK;
    if (!x || !perm || !codes || !scales) return fail(ARCQ_INVALID_ARG, "%s: null pointer", who);
    if (!aligned(x, 16) || (ldx % 8) != 0)
        return fail(ARCQ_BAD_ALIGN, "%s: input must be 16-byte aligned with a leading dimension that is a multiple of 8", who);
    if (!aligned(codes, 16)) return fail(ARCQ_BAD_ALIGN, "%s: codes must be 16-byte aligned", who);
    if (!aligned(perm, 16)) return fail(ARCQ_BAD_ALIGN, "%s: perm must be 16-byte aligned", who);
    return launch_mx_quantize(mode, x, rows, K, ldx, perm, S, codes, scales, flags, static_cast<hipStream_t>(stream));
}

}  // namespace
}  // namespace arcq

using namespace arcq;

extern "C" {

int arcq_version(void) { return 100; }

const char* arcq_last_error(void) { return g_err; }

arcq_status arcq_packed_sizes(int64_t rows, int64_t K, int64_t S, size_t* codes_bytes, size_t* scales_bytes) {
    clear_error();
    if (arcq_status st = check_KS(K, S)) return st;
    if (rows < 0) return fail(ARCQ_BAD_SHAPE, "rows = %lld < 0", (long long)rows);
    if (!codes_bytes || !scales_bytes) return fail(ARCQ_INVALID_ARG, "null output pointer");
    *codes_bytes = (size_t)rows * (size_t)(K + S) / 2;
    *scales_bytes = (size_t)rows * (size_t)(K + S) / 16;
    return ARCQ_OK;
}

arcq_status arcq_quantize_act(const void* x, int64_t M, int64_t K, int64_t ldx, const int32_t* perm, int64_t S,
                              float tensor_scale, uint8_t* codes, uint8_t* scales, void* stream) {
    return quantize_entry(0, "arcq_quantize_act", x, M, K, ldx, perm, S, tensor_scale, codes, scales, stream);
}

arcq_status arcq_rmsnorm_quantize_act(const void* x, int64_t M, int64_t K, int64_t ldx, const void* gamma, float eps,
                                      const int32_t* perm, int64_t S, float tensor_scale, uint8_t* codes,
                                      uint8_t* scales, void* stream) {
    return quantize_entry(0, "arcq_rmsnorm_quantize_act", x, M, K, ldx, perm, S, tensor_scale, codes, scales, stream,
                          true, gamma, eps);
}

arcq_status arcq_pack_weight(const void* w, int64_t N, int64_t K, int64_t ldw, const int32_t* perm, int64_t S,
                             float tensor_scale, uint8_t* codes, uint8_t* scales, void* stream) {
    return quantize_entry(1, "arcq_pack_weight", w, N, K, ldw, perm, S, tensor_scale, codes, scales, stream);
}

arcq_status arcq_quantize_act_ex(const void* x, int64_t M, int64_t K, int64_t ldx, const int32_t* perm, int64_t S,
                                 float tensor_scale, uint32_t flags, uint8_t* codes, uint8_t* scales, void* stream) {
    return quantize_entry(0, "arcq_quantize_act_ex", x, M, K, ldx, perm, S, tensor_scale, codes, scales, stream,
                          false, nullptr, 0.0f, flags);
}

arcq_status arcq_rmsnorm_quantize_act_ex(const void* x, int64_t M, int64_t K, int64_t ldx, const void* gamma, float eps,
                                         const int32_t* perm, int64_t S, float tensor_scale, uint32_t flags,
                                         uint8_t* codes, uint8_t* scales, void* stream) {
    return quantize_entry(0, "arcq_rmsnorm_quantize_act_ex", x, M, K, ldx, perm, S, tensor_scale, codes, scales, stream,
                          true, gamma, eps, flags);
}

arcq_status arcq_pack_weight_ex(const void* w, int64_t N, int64_t K, int64_t ldw, const int32_t* perm, int64_t S,
                                float tensor_scale, uint32_t flags, uint8_t* codes, uint8_t* scales, void* stream) {
    return quantize_entry(1, "arcq_pack_weight_ex", w, N, K, ldw, perm, S, tensor_scale, codes, scales, stream,
                          false, nullptr, 0.0f, flags);
}

static arcq_status check_gemm_shape(int64_t M, int64_t N, int64_t Kp) {
    if (M < 0 || N < 0 || M > 0x7FFFFFFF || N > 0x7FFFFFFF)
        return fail(ARCQ_BAD_SHAPE, "M = %lld, N = %lld out of range", (long long)M, (long long)N);
    if (Kp <= 0 || (Kp % 16) != 0 || Kp > 2 * (int64_t)ARCQ_MAX_K)
        return fail(ARCQ_BAD_SHAPE, "K' = %lld: must be a positive multiple of 16, at most %d", (long long)Kp, 2 * ARCQ_MAX_K);
    return ARCQ_OK;
}

arcq_status arcq_gemm_workspace_size(int64_t M, int64_t N, int64_t Kp, size_t* bytes) {
    clear_error();
    if (arcq_status st = check_gemm_shape(M, N, Kp)) return st;
    if (!bytes) return fail(ARCQ_INVALID_ARG, "null output pointer");
    *bytes = gemm_workspace_bytes(M, N, Kp);
    return ARCQ_OK;
}

// Validation shared by arcq_gemm and arcq_gemm_noalloc; *run = false when there is nothing to launch.
static arcq_status check_gemm_args(const char* who, const uint8_t* a_codes, const uint8_t* a_scales, float a_tensor_scale,
                                   const uint8_t* w_codes, const uint8_t* w_scales, float w_tensor_scale,
                                   int64_t M, int64_t N, int64_t Kp, void* y, int y_dtype, int64_t ldy, bool* run) {
    *run = false;
    if (arcq_status st = check_gemm_shape(M, N, Kp)) return st;
    if (y_dtype != ARCQ_DTYPE_F16 && y_dtype != ARCQ_DTYPE_F32) return fail(ARCQ_INVALID_ARG, "y_dtype = %d", y_dtype);
    if (ldy < N) return fail(ARCQ_BAD_SHAPE, "ldy = %lld < N = %lld", (long long)ldy, (long long)N);
    if (arcq_status st = check_scale(a_tensor_scale, "a_tensor_scale")) return st;
    if (arcq_status st = check_scale(w_tensor_scale, "w_tensor_scale")) return st;
    if (M == 0 || N == 0) return ARCQ_OK;
    if (!a_codes || !a_scales || !w_codes || !w_scales || !y) return fail(ARCQ_INVALID_ARG, "%s: null pointer", who);
    if (!aligned(a_codes, 8) || !aligned(w_codes, 8)) return fail(ARCQ_BAD_ALIGN, "%s: codes must be 8-byte aligned", who);
    if (!aligned(y, 4)) return fail(ARCQ_BAD_ALIGN, "%s: y must be 4-byte aligned", who);
    *run = true;
    return ARCQ_OK;
}

arcq_status arcq_gemm(const uint8_t* a_codes, const uint8_t* a_scales, float a_tensor_scale,
                      const uint8_t* w_codes, const uint8_t* w_scales, float w_tensor_scale,
                      int64_t M, int64_t N, int64_t Kp, void* y, int y_dtype, int64_t ldy,
                      void* workspace, size_t workspace_bytes, void* stream) {
    clear_error();
    bool run = false;
    if (arcq_status st = check_gemm_args("arcq_gemm", a_codes, a_scales, a_tensor_scale, w_codes, w_scales, w_tensor_scale,
                                         M, N, Kp, y, y_dtype, ldy, &run)) return st;
    if (!run) return ARCQ_OK;
    const size_t need = gemm_workspace_bytes(M, N, Kp);
    if (need > 0) {
        if (!workspace || workspace_bytes < need)
            return fail(ARCQ_WORKSPACE_TOO_SMALL, "arcq_gemm: workspace of %zu bytes needed, %zu given", need, workspace_bytes);
        if (!aligned(workspace, 256)) return fail(ARCQ_BAD_ALIGN, "arcq_gemm: workspace must be 256-byte aligned");
    }
    // alpha in fp32: one rounding of the product of the two tensor scales
    const float alpha = a_tensor_scale * w_tensor_scale;
    return launch_gemm(a_codes, a_scales, w_codes, w_scales, M, N, Kp, alpha, y, y_dtype, ldy, workspace,
                       workspace_bytes, static_cast<hipStream_t>(stream));
}

arcq_status arcq_gemm_noalloc(const uint8_t* a_codes, const uint8_t* a_scales, float a_tensor_scale,
                              const uint8_t* w_codes, const uint8_t* w_scales, float w_tensor_scale,
                              int64_t M, int64_t N, int64_t Kp, void* y, int y_dtype, int64_t ldy, void* stream) {
    clear_error();
    bool run = false;
    if (arcq_status st = check_gemm_args("arcq_gemm_noalloc", a_codes, a_scales, a_tensor_scale, w_codes, w_scales,
                                         w_tensor_scale, M, N, Kp, y, y_dtype, ldy, &run)) return st;
    const size_t need = (M == 0 || N == 0) ? 0 : gemm_workspace_bytes(M, N, Kp);
    if (need > (size_t)ARCQ_NOALLOC_SCRATCH_BYTES)
        return fail(ARCQ_WORKSPACE_TOO_SMALL,
                    "arcq_gemm_noalloc: this shape needs %zu bytes of scratch, the built-in buffer holds %zu; "
                    "call arcq_gemm with a workspace of the caller", need, (size_t)ARCQ_NOALLOC_SCRATCH_BYTES);
    if (!run) return ARCQ_OK;
    void* ws = nullptr;
    if (need > 0)
        if (arcq_status st = gemm_scratch_pointer(&ws)) return st;
    const float alpha = a_tensor_scale * w_tensor_scale;
    return launch_gemm(a_codes, a_scales, w_codes, w_scales, M, N, Kp, alpha, y, y_dtype, ldy, ws, need,
                       static_cast<hipStream_t>(stream));
}

arcq_status arcq_check_perm(const int32_t* perm, int64_t K, uint8_t* flags, int* result_host, void* stream) {
    clear_error();
    if (K <= 0 || K > ARCQ_MAX_K) return fail(ARCQ_BAD_SHAPE, "K = %lld out of range", (long long)K);
    if (!perm || !flags || !result_host) return fail(ARCQ_INVALID_ARG, "arcq_check_perm: null pointer");
    return launch_check_perm(perm, K, flags, result_host, static_cast<hipStream_t>(stream));
}

arcq_status arcq_probe_mfma_f16(int iters, float* sink, double* flop_host, void* stream) {
    clear_error();
    if (iters < 1 || iters > (1 << 20)) return fail(ARCQ_INVALID_ARG, "arcq_probe_mfma_f16: iters = %d out of range", iters);
    if (!sink || !flop_host) return fail(ARCQ_INVALID_ARG, "arcq_probe_mfma_f16: null pointer");
    if (!aligned(sink, 4)) return fail(ARCQ_BAD_ALIGN, "arcq_probe_mfma_f16: sink must be 4-byte aligned");
    return launch_probe_mfma_f16(iters, sink, flop_host, static_cast<hipStream_t>(stream));
}

arcq_status arcq_probe_mfma_fp4(int iters, float* sink, double* flop_host, void* stream) {
    clear_error();
    if (iters < 1 || iters > (1 << 20)) return fail(ARCQ_INVALID_ARG, "arcq_probe_mfma_fp4: iters = %d out of range", iters);
    if (!sink || !flop_host) return fail(ARCQ_INVALID_ARG, "arcq_probe_mfma_fp4: null pointer");
    if (!aligned(sink, 4)) return fail(ARCQ_BAD_ALIGN, "arcq_probe_mfma_fp4: sink must be 4-byte aligned");
    return launch_probe_mfma_fp4(iters, sink, flop_host, static_cast<hipStream_t>(stream));
}

arcq_status arcq_ref_gemm_bf16(const void* x, const void* w, int64_t M, int64_t N, int64_t K, void* y, int64_t ldy,
                               void* stream) {
    clear_error();
    if (M < 0 || N <= 0 || K <= 0 || K > ARCQ_MAX_K || (K & 31) != 0) return fail(ARCQ_BAD_SHAPE, "arcq_ref_gemm_bf16: M = %lld, N = %lld, K = %lld (K %% 32 == 0)", (long long)M, (long long)N, (long long)K);
    if (ldy < N) return fail(ARCQ_BAD_SHAPE, "arcq_ref_gemm_bf16: ldy = %lld < N", (long long)ldy);
    if ((uint64_t)M * (uint64_t)K * 2 >= 0xFFFF0000ull || (uint64_t)N * (uint64_t)K * 2 >= 0xFFFF0000ull)
        return fail(ARCQ_BAD_SHAPE, "arcq_ref_gemm_bf16: an operand of 4 GiB or more");
    if (M == 0) return ARCQ_OK;
    if (!x || !w || !y) return fail(ARCQ_INVALID_ARG, "arcq_ref_gemm_bf16: null pointer");
    if (!aligned(x, 16) || !aligned(w, 16)) return fail(ARCQ_BAD_ALIGN, "arcq_ref_gemm_bf16: operands must be 16-byte aligned");
    if (!aligned(y, 2)) return fail(ARCQ_BAD_ALIGN, "arcq_ref_gemm_bf16: y must be 2-byte aligned");
    return launch_ref_gemm_bf16(x, w, M, N, K, static_cast<_Float16*>(y), ldy, static_cast<hipStream_t>(stream));
}

arcq_status arcq_calib_absmax(const void* x, int64_t M, int64_t K, int64_t ldx, float* colmax, void* stream) {
    clear_error();
    if (arcq_status st = check_KS(K, 0)) return st;
    if (M < 0 || M > 0x7FFFFFFF) return fail(ARCQ_BAD_SHAPE, "arcq_calib_absmax: M = %lld out of range", (long long)M);
    if (ldx < K) return fail(ARCQ_BAD_SHAPE, "arcq_calib_absmax: leading dimension %lld < K = %lld", (long long)ldx, (long long)K);
    if (M == 0) return ARCQ_OK;
    if (!x || !colmax) return fail(ARCQ_INVALID_ARG, "arcq_calib_absmax: null pointer");
    if (!aligned(x, 16) || (ldx % 8) != 0)
        return fail(ARCQ_BAD_ALIGN, "arcq_calib_absmax: input must be 16-byte aligned with a leading dimension that is a multiple of 8");
    if (!aligned(colmax, 4)) return fail(ARCQ_BAD_ALIGN, "arcq_calib_absmax: colmax must be 4-byte aligned");
    return launch_calib_absmax(x, M, K, ldx, colmax, static_cast<hipStream_t>(stream));
}

arcq_status arcq_calib_select(const float* colmax, int64_t K, int32_t* perm, int32_t* info, int* S_host, void* stream) {
    clear_error();
    if (arcq_status st = check_KS(K, 0)) return st;
    if (!colmax || !perm || !info) return fail(ARCQ_INVALID_ARG, "arcq_calib_select: null pointer");
    if (!aligned(colmax, 4) || !aligned(perm, 4) || !aligned(info, 4))
        return fail(ARCQ_BAD_ALIGN, "arcq_calib_select: pointers must be 4-byte aligned");
    return launch_calib_select(colmax, K, perm, info, S_host, static_cast<hipStream_t>(stream));
}

arcq_status arcq_mx_packed_sizes(int64_t rows, int64_t K, int64_t S, size_t* codes_bytes, size_t* scales_bytes) {
    clear_error();
    if (arcq_status st = check_KS_mx(K, S)) return st;
    if (rows < 0) return fail(ARCQ_BAD_SHAPE, "rows = %lld < 0", (long long)rows);
    if (!codes_bytes || !scales_bytes) return fail(ARCQ_INVALID_ARG, "null output pointer");
    *codes_bytes = (size_t)rows * (size_t)(K + S) / 2;
    *scales_bytes = (size_t)rows * (size_t)(K + S) / 32;
    return ARCQ_OK;
}

arcq_status arcq_mx_quantize_act(const void* x, int64_t M, int64_t K, int64_t ldx, const int32_t* perm, int64_t S,
                                 uint8_t* codes, uint8_t* scales, void* stream) {
    return mx_quantize_entry(0, "arcq_mx_quantize_act", x, M, K, ldx, perm, S, codes, scales, stream);
}

arcq_status arcq_mx_pack_weight(const void* w, int64_t N, int64_t K, int64_t ldw, const int32_t* perm, int64_t S,
                                uint8_t* codes, uint8_t* scales, void* stream) {
    return mx_quantize_entry(1, "arcq_mx_pack_weight", w, N, K, ldw, perm, S, codes, scales, stream);
}

arcq_status arcq_mx_quantize_act_ex(const void* x, int64_t M, int64_t K, int64_t ldx, const int32_t* perm, int64_t S,
                                    uint32_t flags, uint8_t* codes, uint8_t* scales, void* stream) {
    return mx_quantize_entry(0, "arcq_mx_quantize_act_ex", x, M, K, ldx, perm, S, codes, scales, stream, flags);
}

arcq_status arcq_mx_pack_weight_ex(const void* w, int64_t N, int64_t K, int64_t ldw, const int32_t* perm, int64_t S,
                                   uint32_t flags, uint8_t* codes, uint8_t* scales, void* stream) {
    return mx_quantize_entry(1, "arcq_mx_pack_weight_ex", w, N, K, ldw, perm, S, codes, scales, stream, flags);
}

static arcq_status mx_gemm_entry(const char* name, const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* w_codes,
                                 const uint8_t* w_scales, int64_t M, int64_t N, int64_t Kp, void* y, int y_dtype, int64_t ldy,
                                 bool with_workspace, void* workspace, size_t workspace_bytes, void* stream) {
    clear_error();
    if (M < 0 || N < 0 || M > 0x7FFFFFFF || N > 0x7FFFFFFF)
        return fail(ARCQ_BAD_SHAPE, "M = %lld, N = %lld out of range", (long long)M, (long long)N);
    if (Kp <= 0 || (Kp % 32) != 0 || Kp > 2 * (int64_t)ARCQ_MAX_K)
        return fail(ARCQ_BAD_SHAPE, "K' = %lld: must be a positive multiple of 32, at most %d", (long long)Kp, 2 * ARCQ_MAX_K);
    if (y_dtype != ARCQ_DTYPE_F16 && y_dtype != ARCQ_DTYPE_F32) return fail(ARCQ_INVALID_ARG, "y_dtype = %d", y_dtype);
    if (ldy < N) return fail(ARCQ_BAD_SHAPE, "ldy = %lld < N = %lld", (long long)ldy, (long long)N);
    if (M == 0 || N == 0) return ARCQ_OK;
    if (!a_codes || !a_scales || !w_codes || !w_scales || !y) return fail(ARCQ_INVALID_ARG, "%s: null pointer", name);
    if (!aligned(a_codes, 4) || !aligned(w_codes, 4)) return fail(ARCQ_BAD_ALIGN, "%s: codes must be 4-byte aligned", name);
    if (!aligned(y, 4)) return fail(ARCQ_BAD_ALIGN, "%s: y must be 4-byte aligned", name);
    void* ws = nullptr;
    if (with_workspace) {
        const size_t need = mx_gemm_workspace_bytes(M, N, Kp);
        if (need > 0) {
            if (!workspace || workspace_bytes < need)
                return fail(ARCQ_WORKSPACE_TOO_SMALL, "%s: workspace of %zu bytes needed, %zu given", name, need, workspace_bytes);
            if (!aligned(workspace, 256)) return fail(ARCQ_BAD_ALIGN, "%s: workspace must be 256-byte aligned", name);
            ws = workspace;
        }
    }
    return launch_mx_gemm(a_codes, a_scales, w_codes, w_scales, M, N, Kp, y, y_dtype, ldy, ws, static_cast<hipStream_t>(stream));
}

arcq_status arcq_mx_gemm(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* w_codes, const uint8_t* w_scales,
                         int64_t M, int64_t N, int64_t Kp, void* y, int y_dtype, int64_t ldy, void* stream) {
    return mx_gemm_entry("arcq_mx_gemm", a_codes, a_scales, w_codes, w_scales, M, N, Kp, y, y_dtype, ldy, false, nullptr, 0, stream);
}

arcq_status arcq_mx_gemm_workspace_size(int64_t M, int64_t N, int64_t Kp, size_t* bytes) {
    clear_error();
    if (M < 0 || N < 0 || M > 0x7FFFFFFF || N > 0x7FFFFFFF)
        return fail(ARCQ_BAD_SHAPE, "M = %lld, N = %lld out of range", (long long)M, (long long)N);
    if (Kp <= 0 || (Kp % 32) != 0 || Kp > 2 * (int64_t)ARCQ_MAX_K)
        return fail(ARCQ_BAD_SHAPE, "K' = %lld: must be a positive multiple of 32, at most %d", (long long)Kp, 2 * ARCQ_MAX_K);
    if (!bytes) return fail(ARCQ_INVALID_ARG, "null output pointer");
    *bytes = (M == 0 || N == 0) ? 0 : mx_gemm_workspace_bytes(M, N, Kp);
    return ARCQ_OK;
}

arcq_status arcq_mx_gemm_ws(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* w_codes, const uint8_t* w_scales,
                            int64_t M, int64_t N, int64_t Kp, void* y, int y_dtype, int64_t ldy,
                            void* workspace, size_t workspace_bytes, void* stream) {
    return mx_gemm_entry("arcq_mx_gemm_ws", a_codes, a_scales, w_codes, w_scales, M, N, Kp, y, y_dtype, ldy, true, workspace,
                         workspace_bytes, stream);
}

}  // extern "C"
