/*
 * arcq_bench.h -- measurement aids of libarcq (no part of the ARCQuant method; see arcq.h for the method's calls):
 * the matrix-rate probes that give the ceiling a GEMM's roofline fraction is read against on a given machine, and
 * the hand-written bf16 GEMM the quantized linear layer is timed against.  Same conventions as arcq.h: device
 * pointers owned by the caller, work enqueued on `stream`, status codes, arcq_last_error().
 */
#ifndef ARCQ_BENCH_H
#define ARCQ_BENCH_H

#include "arcq.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Diagnostic for measurements (no part of the method): enqueues a kernel in which 4096 waves (four per
 * SIMD on 256 CUs) each issue 4 * iters fp16 32x32x16 matrix instructions on register operands, the
 * instruction arcq_gemm is built on, with no memory traffic in the loop.  Timing the launch gives the
 * matrix rate this machine sustains, the ceiling to read arcq_gemm's roofline fraction against.
 * iters   1 .. 2^20
 * sink    device, ARCQ_PROBE_SINK_FLOATS floats, written (keeps the loop alive), 4-byte aligned
 * flop_host  host pointer: receives the floating-point operations of one launch
 */
#define ARCQ_PROBE_SINK_FLOATS 262144
arcq_status arcq_probe_mfma_f16(int iters, float* sink, double* flop_host, void* stream);
/* The same for the instruction arcq_mx_gemm is built on: 4 * iters scaled FP4 32x32x64 matrix instructions
 * per wave (both operands E2M1, unit block scales); same arguments, same sink size. */
arcq_status arcq_probe_mfma_fp4(int iters, float* sink, double* flop_host, void* stream);

/*
 * Comparison kernel for measurements (no part of the method): the unquantized linear layer y = x w^T on bf16
 * operands, written on the same tiled skeleton as arcq_mx_gemm (operand rows travel global -> LDS in 128-byte
 * units, v_mfma_f32_32x32x16_bf16, fp32 accumulation), the 16-bit baseline the quantized path is timed against.
 * x  device, bf16 [M, K] row-major, pitch K, 16-byte aligned     w  device, bf16 [N, K] row-major, 16-byte aligned
 * y  device, fp16 [M, N], pitch ldy >= N                         K % 32 == 0, operands below 4 GiB each
 */
arcq_status arcq_ref_gemm_bf16(const void* x, const void* w, int64_t M, int64_t N, int64_t K, void* y, int64_t ldy,
                               void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ARCQ_BENCH_H */
