// Loss-scale removal with overflow detection over a flat fp32 gradient buffer.
// HBM-bound: 4 bytes read + 4 bytes written per element, nothing else.
//   grad[i] <- grad[i] * inv_scale   (one fp32 multiply, no contraction partner)
//   flag    <- any input with all-ones exponent (+-inf, NaN)
// Every element is written even when the flag trips.  Each wave reduces its lanes'
// findings with a ballot; only waves that saw a non-finite value touch the flag.
#include "common.h"

namespace sdconv {

constexpr int kUnscaleThreads = 256;
constexpr int kUnscaleVecPerThread = 4;   // float4 loads in flight per thread

__device__ __forceinline__ unsigned nonfinite_bits(float v)
{
    return ((__float_as_uint(v) & 0x7f800000u) == 0x7f800000u) ? 1u : 0u;
}

__global__ void clear_flag_kernel(int32_t* flag) { *flag = 0; }

// scale_on_device: nullptr, or the current loss scale in device memory: inv_scale is then
// 1/scale, one correctly rounded binary32 division.
__global__ __launch_bounds__(kUnscaleThreads) void unscale_check_kernel(
    float* __restrict__ grad, size_t n, size_t head, size_t nvec, float inv_scale,
    const float* __restrict__ scale_on_device, int32_t* __restrict__ flag)
{
    typedef float float4v __attribute__((ext_vector_type(4)));
    if (scale_on_device) inv_scale = __fdiv_rn(1.0f, *scale_on_device);
    unsigned bad = 0;
    float4v* body = reinterpret_cast<float4v*>(grad + head);
    size_t base = (size_t)blockIdx.x * (kUnscaleThreads * kUnscaleVecPerThread) + threadIdx.x;
    float4v v[kUnscaleVecPerThread];
#pragma unroll
    for (int j = 0; j < kUnscaleVecPerThread; ++j) {
        size_t i = base + (size_t)j * kUnscaleThreads;
        if (i < nvec) v[j] = __builtin_nontemporal_load(body + i);
    }
#pragma unroll
    for (int j = 0; j < kUnscaleVecPerThread; ++j) {
        size_t i = base + (size_t)j * kUnscaleThreads;
        if (i < nvec) {
            bad |= nonfinite_bits(v[j].x) | nonfinite_bits(v[j].y) | nonfinite_bits(v[j].z) |
                   nonfinite_bits(v[j].w);
            float4v o;
            o.x = __fmul_rn(v[j].x, inv_scale);
            o.y = __fmul_rn(v[j].y, inv_scale);
            o.z = __fmul_rn(v[j].z, inv_scale);
            o.w = __fmul_rn(v[j].w, inv_scale);
            __builtin_nontemporal_store(o, body + i);
        }
    }
    // Unaligned head (< 4 elements) and ragged tail (< 4 elements): block 0, first lanes.
    if (blockIdx.x == 0) {
        size_t tail_start = head + nvec * 4;
        size_t ntail = n - tail_start;
        size_t t = threadIdx.x;
        if (t < head) {
            float g = grad[t];
            bad |= nonfinite_bits(g);
            grad[t] = __fmul_rn(g, inv_scale);
        } else if (t >= 8 && t - 8 < ntail) {
            float g = grad[tail_start + (t - 8)];
            bad |= nonfinite_bits(g);
            grad[tail_start + (t - 8)] = __fmul_rn(g, inv_scale);
        }
    }
    unsigned long long any = __ballot(bad != 0);
    if (any != 0ull && (threadIdx.x & 63) == 0) atomicOr(flag, 1);
}

hipError_t launch_unscale_check(float* grad, size_t n, float inv_scale, const float* scale_on_device,
                                int32_t* flag, hipStream_t st)
{
    hipLaunchKernelGGL(clear_flag_kernel, dim3(1), dim3(1), 0, st, flag);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || n == 0) return e;
    size_t mis = (reinterpret_cast<uintptr_t>(grad) >> 2) & 3u;     // floats past a 16-byte line
    size_t head = mis ? (4 - mis) : 0;
    if (head > n) head = n;
    size_t nvec = (n - head) / 4;
    size_t per_block = (size_t)kUnscaleThreads * kUnscaleVecPerThread;
    size_t blocks = (nvec + per_block - 1) / per_block;
    if (blocks == 0) blocks = 1;
    hipLaunchKernelGGL(unscale_check_kernel, dim3((unsigned)blocks), dim3(kUnscaleThreads), 0, st,
                       grad, n, head, nvec, inv_scale, scale_on_device, flag);
    return hipGetLastError();
}

}  // namespace sdconv
