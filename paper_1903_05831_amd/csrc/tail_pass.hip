// The elementwise tail as a pass of its own over an NHWC binary16 tensor, in place: what a
// framework runs after a convolution when the tail is not fused into it.  It exists to be
// timed against conv2d_fwd_fused / conv2d_dgrad_fused (it reads and writes the whole
// activation once more); its result differs from theirs by the extra rounding to binary16
// between convolution and tail.  One lane handles 8 consecutive channels of a pixel.
#include "common.h"

namespace sdconv {

typedef _Float16 tp_half8 __attribute__((ext_vector_type(8)));
typedef float tp_float4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void tail_pass_kernel(_Float16* __restrict__ t, long chunks, int C, Epilogue E)
{
    for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < chunks; i += (long)gridDim.x * blockDim.x) {
        const long e0 = i * 8;
        const int c = (int)(e0 % C);
        tp_half8 v = __builtin_nontemporal_load(reinterpret_cast<const tp_half8*>(t + e0));
        float f[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) f[e] = (float)v[e];
        if (E.scale) {
            tp_float4 a = *reinterpret_cast<const tp_float4*>(E.scale + c), b = *reinterpret_cast<const tp_float4*>(E.scale + c + 4);
#pragma unroll
            for (int e = 0; e < 4; ++e) { f[e] *= a[e]; f[4 + e] *= b[e]; }
        }
        if (E.bias) {
            tp_float4 a = *reinterpret_cast<const tp_float4*>(E.bias + c), b = *reinterpret_cast<const tp_float4*>(E.bias + c + 4);
#pragma unroll
            for (int e = 0; e < 4; ++e) { f[e] += a[e]; f[4 + e] += b[e]; }
        }
        if (E.residual) {
            tp_half8 r = __builtin_nontemporal_load(reinterpret_cast<const tp_half8*>(reinterpret_cast<const _Float16*>(E.residual) + e0));
#pragma unroll
            for (int e = 0; e < 8; ++e) f[e] += (float)r[e];
        }
        if (E.relu) {
#pragma unroll
            for (int e = 0; e < 8; ++e) f[e] = f[e] > 0.f ? f[e] : 0.f;
        }
        if (E.mask) {
            tp_half8 m = __builtin_nontemporal_load(reinterpret_cast<const tp_half8*>(reinterpret_cast<const _Float16*>(E.mask) + e0));
#pragma unroll
            for (int e = 0; e < 8; ++e) f[e] = (float)m[e] > 0.f ? f[e] : 0.f;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = (_Float16)f[e];
        __builtin_nontemporal_store(v, reinterpret_cast<tp_half8*>(t + e0));
    }
}

hipError_t launch_tail_pass(__half* t, long pixels, int C, const Epilogue& ep, hipStream_t st)
{
    const long chunks = pixels * C / 8;
    if (chunks == 0) return hipSuccess;
    long blocks = (chunks + 255) / 256;
    if (blocks > 256 * 16) blocks = 256 * 16;
    hipLaunchKernelGGL(tail_pass_kernel, dim3((unsigned)blocks), dim3(256), 0, st, reinterpret_cast<_Float16*>(t), chunks, C, ep);
    return hipGetLastError();
}

}  // namespace sdconv
