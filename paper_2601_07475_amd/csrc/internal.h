// Internal declarations shared by the translation units of libarcq (host side only).
#pragma once
#include <hip/hip_runtime.h>

#include <atomic>
#include <stddef.h>
#include <stdint.h>

#include "../../include/arcq.h"
#include "../../include/arcq_bench.h"

namespace arcq {

// Records a message for arcq_last_error() and returns `code`.
arcq_status fail(arcq_status code, const char* fmt, ...);
void clear_error();

// After a kernel launch: turns a pending HIP launch error into ARCQ_HIP_ERROR.
arcq_status check_launch(const char* what);

// Kernels with more than 48 KB of dynamic LDS need their limit raised once per device.  `done` is a bit mask
// over device indices, one static per kernel instantiation; the limit is raised to the whole 160 KB of a
// compute unit, so one call serves every launch shape of that kernel.
constexpr int kMaxLdsBytes = 160 * 1024;
arcq_status raise_lds_limit(const void* kernel, std::atomic<uint64_t>& done);
// Compute units of the current device (cached per device).
int num_cu();

// mode 0: activations (residual blocks appended); mode 1: weights (outlier blocks duplicated).
// gamma != nullptr (mode 0 only): RMSNorm with that weight and eps in front of the quantizer.
arcq_status launch_quantize(int mode, const void* x, int64_t rows, int64_t K, int64_t ldx,
                            const int32_t* perm, int64_t S, float s_T,
                            uint8_t* codes, uint8_t* scales, const void* gamma, float eps, uint32_t flags,
                            hipStream_t stream);

size_t gemm_workspace_bytes(int64_t M, int64_t N, int64_t Kp);
// device address, on the current device, of the library's built-in scratch (ARCQ_NOALLOC_SCRATCH_BYTES)
arcq_status gemm_scratch_pointer(void** out);
arcq_status launch_gemm(const uint8_t* a_codes, const uint8_t* a_scales,
                        const uint8_t* w_codes, const uint8_t* w_scales,
                        int64_t M, int64_t N, int64_t Kp, float alpha,
                        void* y, int y_dtype, int64_t ldy,
                        void* workspace, size_t workspace_bytes, hipStream_t stream);

// Tiled kernel whose waves split every stage along k inside the workgroup (gemm_ksplit.hip): which of its tile
// shapes serves this problem (0: none), and its launch.
int gemm_ksplit_variant(int64_t M, int64_t N, int64_t Kp);
arcq_status launch_gemm_ksplit(int variant, const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* w_codes,
                               const uint8_t* w_scales, int64_t M, int64_t N, int64_t Kp, float alpha, void* y, int y_dtype,
                               int64_t ldy, hipStream_t stream);

arcq_status launch_probe_mfma_f16(int iters, float* sink, double* flop_host, hipStream_t stream);
arcq_status launch_probe_mfma_fp4(int iters, float* sink, double* flop_host, hipStream_t stream);
arcq_status launch_ref_gemm_bf16(const void* x, const void* w, int64_t M, int64_t N, int64_t K, _Float16* y, int64_t ldy,
                                 hipStream_t stream);
arcq_status launch_check_perm(const int32_t* perm, int64_t K, uint8_t* flags,
                              int* result_host, hipStream_t stream);

arcq_status launch_calib_absmax(const void* x, int64_t M, int64_t K, int64_t ldx, float* colmax, hipStream_t stream);
arcq_status launch_calib_select(const float* colmax, int64_t K, int32_t* perm, int32_t* info, int* S_host,
                                hipStream_t stream);

// MXFP4 variant (blocks of 32, E8M0 scales, no tensor scale)
arcq_status launch_mx_quantize(int mode, const void* x, int64_t rows, int64_t K, int64_t ldx, const int32_t* perm,
                               int64_t S, uint8_t* codes, uint8_t* scales, uint32_t flags, hipStream_t stream);
// workspace: fp32 partial results of a split reduction dimension, or null (never splits)
arcq_status launch_mx_gemm(const uint8_t* a_codes, const uint8_t* a_scales, const uint8_t* w_codes,
                           const uint8_t* w_scales, int64_t M, int64_t N, int64_t Kp, void* y, int y_dtype, int64_t ldy,
                           void* workspace, hipStream_t stream);
size_t mx_gemm_workspace_bytes(int64_t M, int64_t N, int64_t Kp);
// y = alpha * (partial[0] + partial[1] + ... in index order), partial results fp32 [splits][M][N]
arcq_status launch_splitk_reduce(const float* partial, int splits, int M, int N, float alpha, void* y, int y_dtype,
                                 int64_t ldy, hipStream_t stream);

}  // namespace arcq
