// Helpers of the padded-filter-count route: layers whose filter count K is not a multiple of 8
// (the 3 / 12 / 15 / 60-channel heads of a region proposal network) run on the MFMA kernels as
// layers with K rounded up to Kp, with zero filters (forward) or zero gradient channels (data
// and weight gradient) in the extra positions.  The tensors that get padded are the small ones:
// the filter, and the K-channel activation or gradient tensor; the C-channel tensor is used in
// place.
#include "common.h"

namespace sdconv {

// dst[row][0..Kp) = src[row][0..K), zeros behind: rows = pixels (dy) ; one thread per element of dst
__global__ __launch_bounds__(256) void pad_channels_kernel(const __half* __restrict__ src, __half* __restrict__ dst,
                                                           long total, int K, int Kp)
{
    for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
        const long row = i / Kp;
        const int k = (int)(i - row * Kp);
        dst[i] = k < K ? src[row * K + k] : __float2half_rn(0.f);
    }
}

// dst[0..n) = src[0..n), dst[n..total) = 0: a [K][R][S][C] filter becomes [Kp][R][S][C]
__global__ __launch_bounds__(256) void pad_rows_kernel(const __half* __restrict__ src, __half* __restrict__ dst,
                                                       long n, long total)
{
    for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x)
        dst[i] = i < n ? src[i] : __float2half_rn(0.f);
}

// y[row][0..K) = tail(yp[row][0..K)): drops the padding channels of a forward result and applies
// the elementwise tail, if any, on the way
__global__ __launch_bounds__(256) void unpad_channels_kernel(const __half* __restrict__ yp, __half* __restrict__ y,
                                                             long total, int K, int Kp, Epilogue E)
{
    for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
        const long row = i / K;
        const int k = (int)(i - row * K);
        float v = __half2float(yp[row * Kp + k]);
        y[i] = __float2half_rn(epilogue_apply(E, v, k, i));
    }
}

__global__ __launch_bounds__(256) void copy_f32_kernel(const float* __restrict__ src, float* __restrict__ dst, long n)
{
    for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (long)gridDim.x * blockDim.x) dst[i] = src[i];
}

static unsigned grid_for(long total)
{
    long b = (total + 255) / 256;
    return (unsigned)(b < 1 ? 1 : (b > 65536 ? 65536 : b));
}

hipError_t launch_pad_channels(const __half* src, __half* dst, long rows, int K, int Kp, hipStream_t st)
{
    const long total = rows * Kp;
    hipLaunchKernelGGL(pad_channels_kernel, dim3(grid_for(total)), dim3(256), 0, st, src, dst, total, K, Kp);
    return hipGetLastError();
}

hipError_t launch_pad_rows(const __half* src, __half* dst, long n, long total, hipStream_t st)
{
    hipLaunchKernelGGL(pad_rows_kernel, dim3(grid_for(total)), dim3(256), 0, st, src, dst, n, total);
    return hipGetLastError();
}

hipError_t launch_unpad_channels(const __half* yp, __half* y, long rows, int K, int Kp, const Epilogue& ep, hipStream_t st)
{
    const long total = rows * K;
    hipLaunchKernelGGL(unpad_channels_kernel, dim3(grid_for(total)), dim3(256), 0, st, yp, y, total, K, Kp, ep);
    return hipGetLastError();
}

hipError_t launch_copy_f32(const float* src, float* dst, long n, hipStream_t st)
{
    hipLaunchKernelGGL(copy_f32_kernel, dim3(grid_for(n)), dim3(256), 0, st, src, dst, n);
    return hipGetLastError();
}

}  // namespace sdconv
