// Debug helper: device-side check that perm is a permutation of 0..K-1.
#include "internal.h"

namespace arcq {

namespace {

__global__ void perm_clear_kernel(uint8_t* flags, int K) {
    for (int j = blockIdx.x * blockDim.x + threadIdx.x; j < K; j += gridDim.x * blockDim.x) flags[j] = 0;
}

__global__ void perm_mark_kernel(const int32_t* perm, uint8_t* flags, int K) {
    for (int j = blockIdx.x * blockDim.x + threadIdx.x; j < K; j += gridDim.x * blockDim.x) {
        const int p = perm[j];
        if (p >= 0 && p < K) flags[p] = 1;      // same value from every writer
    }
}

// one workgroup: all K flags set <=> every value in range and no value twice
__global__ __launch_bounds__(1024) void perm_reduce_kernel(uint8_t* flags, int K) {
    int ok = 1;
    for (int j = threadIdx.x; j < K; j += blockDim.x) ok &= (flags[j] == 1);
    ok = __syncthreads_and(ok);
    if (threadIdx.x == 0) flags[0] = (uint8_t)ok;
}

}  // namespace

arcq_status launch_check_perm(const int32_t* perm, int64_t K, uint8_t* flags, int* result_host,
                              hipStream_t stream) {
    const int k = (int)K;
    const int grid = (k + 255) / 256;
    hipLaunchKernelGGL(perm_clear_kernel, dim3(grid), dim3(256), 0, stream, flags, k);
    hipLaunchKernelGGL(perm_mark_kernel, dim3(grid), dim3(256), 0, stream, perm, flags, k);
    hipLaunchKernelGGL(perm_reduce_kernel, dim3(1), dim3(1024), 0, stream, flags, k);
    if (arcq_status st = check_launch("perm_check kernels")) return st;
    uint8_t r = 0;
    hipError_t e = hipMemcpyAsync(&r, flags, 1, hipMemcpyDeviceToHost, stream);
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    if (e != hipSuccess) return fail(ARCQ_HIP_ERROR, "arcq_check_perm: %s", hipGetErrorString(e));
    *result_host = r;
    return ARCQ_OK;
}

}  // namespace arcq
