// Offline calibration (Section 3.2 "Adaptive Outlier Identification"): per-channel absolute maximum
// over calibration activations, then the channel order and the outlier count S.
//
// Statistics are fp32 values >= 0 held as their bit patterns, which order like unsigned integers:
// the running maximum is an integer atomic maximum and the sort key is the pattern itself.
#include "internal.h"

#include <hip/hip_fp16.h>

namespace arcq {

namespace {

typedef uint16_t u16x2 __attribute__((ext_vector_type(2)));

// |a|, |b| as fp16 bit patterns, element-wise maximum (patterns of non-negative halves order like integers)
__device__ __forceinline__ uint32_t absmax2(uint32_t acc, uint32_t v) {
    const u16x2 a = __builtin_bit_cast(u16x2, acc), b = __builtin_bit_cast(u16x2, v & 0x7FFF7FFFu);
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(a, b));
}

// Four waves per workgroup: lane l of every wave owns the 8 channels 8 (64 blockIdx.x + l) .. + 7; wave w
// scans rows w, w + 4, ... of strip blockIdx.y with 16-byte loads (a wave instruction reads 1 KB of one
// row), eight rows in flight; the four waves combine through LDS and one of them merges the eight
// maxima into the running statistic with integer atomic maxima (atomics on one address serialise in
// the L2, so there are few strips and one atomic per channel and strip).
// HBM-bound: 2 bytes per element read once.
constexpr int ABSMAX_UNROLL = 8;
__global__ __launch_bounds__(256) void absmax_kernel(const uint16_t* __restrict__ x, int64_t ldx, int M, int K,
                                                     int rows_per_strip, uint32_t* __restrict__ colmax) {
    __shared__ uint4 part[3][64];
    const int c8 = min((int)(blockIdx.x * 64 + threadIdx.x), (K >> 3) - 1);     // surplus lanes repeat the last group
    const int m0 = blockIdx.y * rows_per_strip + threadIdx.y, m1 = min(M, (int)(blockIdx.y + 1) * rows_per_strip);
    const uint4* src = reinterpret_cast<const uint4*>(x + 8 * (int64_t)c8);
    const int64_t pitch16 = ldx >> 3;                       // row pitch in 16-byte units
    uint4 mx[ABSMAX_UNROLL];
#pragma unroll
    for (int u = 0; u < ABSMAX_UNROLL; ++u) mx[u] = make_uint4(0, 0, 0, 0);
    int m = m0;
    for (; m + 4 * (ABSMAX_UNROLL - 1) < m1; m += 4 * ABSMAX_UNROLL) {
        uint4 v[ABSMAX_UNROLL];
#pragma unroll
        for (int u = 0; u < ABSMAX_UNROLL; ++u) v[u] = src[(int64_t)(m + 4 * u) * pitch16];
#pragma unroll
        for (int u = 0; u < ABSMAX_UNROLL; ++u) {
            mx[u].x = absmax2(mx[u].x, v[u].x);
            mx[u].y = absmax2(mx[u].y, v[u].y);
            mx[u].z = absmax2(mx[u].z, v[u].z);
            mx[u].w = absmax2(mx[u].w, v[u].w);
        }
    }
    for (; m < m1; m += 4) {
        const uint4 v = src[(int64_t)m * pitch16];
        mx[0].x = absmax2(mx[0].x, v.x);
        mx[0].y = absmax2(mx[0].y, v.y);
        mx[0].z = absmax2(mx[0].z, v.z);
        mx[0].w = absmax2(mx[0].w, v.w);
    }
#pragma unroll
    for (int u = 1; u < ABSMAX_UNROLL; ++u) {
        mx[0].x = absmax2(mx[0].x, mx[u].x);
        mx[0].y = absmax2(mx[0].y, mx[u].y);
        mx[0].z = absmax2(mx[0].z, mx[u].z);
        mx[0].w = absmax2(mx[0].w, mx[u].w);
    }
    if (threadIdx.y > 0) part[threadIdx.y - 1][threadIdx.x] = mx[0];
    __syncthreads();
    if (threadIdx.y > 0) return;
#pragma unroll
    for (int w = 0; w < 3; ++w) {
        const uint4 o = part[w][threadIdx.x];
        mx[0].x = absmax2(mx[0].x, o.x);
        mx[0].y = absmax2(mx[0].y, o.y);
        mx[0].z = absmax2(mx[0].z, o.z);
        mx[0].w = absmax2(mx[0].w, o.w);
    }
    const uint32_t r[4] = {mx[0].x, mx[0].y, mx[0].z, mx[0].w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float lo = __half2float(__ushort_as_half((unsigned short)(r[e] & 0xFFFFu)));
        const float hi = __half2float(__ushort_as_half((unsigned short)(r[e] >> 16)));
        atomicMax(colmax + 8 * c8 + 2 * e, __float_as_uint(lo));
        atomicMax(colmax + 8 * c8 + 2 * e + 1, __float_as_uint(hi));
    }
}

// One workgroup: layer maximum, tau = 2^-3 max (exact), number of channels above tau, S rounded up to
// a block of 16.  info = {S, S_raw, bits(max), bits(tau)}.
__global__ __launch_bounds__(1024) void calib_stats_kernel(const uint32_t* __restrict__ colmax, int K,
                                                           int32_t* __restrict__ info) {
    __shared__ uint32_t part[16];
    __shared__ uint32_t total;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t mx = 0;
    for (int k = tid; k < K; k += 1024) mx = max(mx, colmax[k]);
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) mx = max(mx, (uint32_t)__shfl_xor((int)mx, m, 64));
    if (lane == 0) part[wave] = mx;
    __syncthreads();
    if (tid == 0) {
        uint32_t t = 0;
        for (int w = 0; w < 16; ++w) t = max(t, part[w]);
        total = t;
    }
    __syncthreads();
    const float layer_max = __uint_as_float(total);
    const float tau = layer_max * 0.125f;
    int cnt = 0;
    for (int k = tid; k < K; k += 1024) cnt += __uint_as_float(colmax[k]) > tau ? 1 : 0;
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) cnt += __shfl_xor(cnt, m, 64);
    __syncthreads();
    if (lane == 0) part[wave] = (uint32_t)cnt;
    __syncthreads();
    if (tid == 0) {
        int s_raw = 0;
        for (int w = 0; w < 16; ++w) s_raw += (int)part[w];
        const int s = min(K, (s_raw + 15) / 16 * 16);
        info[0] = s;
        info[1] = s_raw;
        info[2] = (int32_t)total;
        info[3] = (int32_t)__float_as_uint(tau);
    }
}

// Stable ascending order by counting: the position of channel k is the number of channels that come
// before it (smaller statistic, or equal statistic and smaller index).  Every position is hit exactly
// once whatever the values, so the output is always a permutation.  K^2 comparisons, tiles of the
// keys staged in LDS; K <= 65536 keeps this well under a millisecond, and it runs once per layer.
constexpr int RANK_TILE = 2048;
__global__ __launch_bounds__(256) void calib_rank_kernel(const uint32_t* __restrict__ colmax, int K,
                                                         int32_t* __restrict__ perm) {
    __shared__ uint32_t keys[RANK_TILE];
    const int k = blockIdx.x * 256 + threadIdx.x;
    const uint32_t mine = k < K ? colmax[k] : 0u;
    int before = 0;
    for (int j0 = 0; j0 < K; j0 += RANK_TILE) {
        const int n = min(RANK_TILE, K - j0);
        __syncthreads();
        for (int j = threadIdx.x; j < n; j += 256) keys[j] = colmax[j0 + j];
        __syncthreads();
        // tiles wholly below / above k need only one of the two comparisons
        if (j0 + n <= k) {
            for (int j = 0; j < n; ++j) before += keys[j] <= mine ? 1 : 0;
        } else if (j0 > k) {
            for (int j = 0; j < n; ++j) before += keys[j] < mine ? 1 : 0;
        } else {
            for (int j = 0; j < n; ++j) before += (keys[j] < mine || (keys[j] == mine && j0 + j < k)) ? 1 : 0;
        }
    }
    if (k < K) perm[before] = k;
}

}  // namespace

arcq_status launch_calib_absmax(const void* x, int64_t M, int64_t K, int64_t ldx, float* colmax, hipStream_t stream) {
    const int colblocks = (int)((K / 8 + 63) / 64);
    // about 1024 workgroups (4 per CU, 128 KB in flight per CU), strips of at least 32 rows
    int64_t rows_per_strip = (M * colblocks + 1023) / 1024;
    if (rows_per_strip < 32) rows_per_strip = 32;
    const int64_t strips = (M + rows_per_strip - 1) / rows_per_strip;
    hipLaunchKernelGGL(absmax_kernel, dim3(colblocks, (unsigned)strips), dim3(64, 4), 0, stream,
                       static_cast<const uint16_t*>(x), ldx, (int)M, (int)K, (int)rows_per_strip,
                       reinterpret_cast<uint32_t*>(colmax));
    return check_launch("absmax_kernel");
}

arcq_status launch_calib_select(const float* colmax, int64_t K, int32_t* perm, int32_t* info, int* S_host,
                                hipStream_t stream) {
    const uint32_t* keys = reinterpret_cast<const uint32_t*>(colmax);
    hipLaunchKernelGGL(calib_stats_kernel, dim3(1), dim3(1024), 0, stream, keys, (int)K, info);
    hipLaunchKernelGGL(calib_rank_kernel, dim3((unsigned)((K + 255) / 256)), dim3(256), 0, stream, keys, (int)K, perm);
    if (arcq_status st = check_launch("calibration kernels")) return st;
    if (S_host) {
        int32_t s = 0;
        hipError_t e = hipMemcpyAsync(&s, info, sizeof(s), hipMemcpyDeviceToHost, stream);
        if (e == hipSuccess) e = hipStreamSynchronize(stream);
        if (e != hipSuccess) return fail(ARCQ_HIP_ERROR, "arcq_calib_select: %s", hipGetErrorString(e));
        *S_host = s;
    }
    return ARCQ_OK;
}

}  // namespace arcq
