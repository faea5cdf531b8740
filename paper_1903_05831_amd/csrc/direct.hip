// Direct (one result per thread / per block) convolution kernels.  They accept every
// valid descriptor and are the route for channel counts the MFMA kernels do not tile
// (C or K not a multiple of 8).  fp16 inputs, fp32 accumulation, the optional elementwise
// tail in fp32, one rounding on store.  The same kernels on fp32 tensors (T = float: fp32
// products and sums, no tail) serve the descriptors the fp32 matrix kernels do not take.
#include "common.h"

namespace sdconv {

__device__ __forceinline__ float to_f32(__half v) { return __half2float(v); }
__device__ __forceinline__ float to_f32(float v) { return v; }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ __half from_f32<__half>(float v) { return __float2half_rn(v); }
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }

template <typename T>
__global__ __launch_bounds__(256) void direct_fwd_kernel(Geom g, const T* __restrict__ x,
                                                         const T* __restrict__ w,
                                                         T* __restrict__ y, long total, Epilogue E)
{
    long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    int k = (int)(i % g.K);
    long t = i / g.K;
    int wo = (int)(t % g.Wo); t /= g.Wo;
    int ho = (int)(t % g.Ho);
    int n = (int)(t / g.Ho);
    float acc = 0.f;
    for (int r = 0; r < g.R; ++r) {
        int h = ho * g.sh - g.ph + r * g.dh;
        if (h < 0 || h >= g.H) continue;
        for (int s = 0; s < g.S; ++s) {
            int wi = wo * g.sw - g.pw + s * g.dw;
            if (wi < 0 || wi >= g.W) continue;
            const T* xp = x + (((long)n * g.H + h) * g.W + wi) * g.C;
            const T* wp = w + (((long)k * g.R + r) * g.S + s) * g.C;
            for (int c = 0; c < g.C; ++c) acc += to_f32(xp[c]) * to_f32(wp[c]);
        }
    }
    y[i] = from_f32<T>(epilogue_apply(E, acc, k, i));
}

template <typename T>
__global__ __launch_bounds__(256) void direct_dgrad_kernel(Geom g, const T* __restrict__ dy,
                                                           const T* __restrict__ w,
                                                           T* __restrict__ dx, long total, Epilogue E)
{
    long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total) return;
    int c = (int)(i % g.C);
    long t = i / g.C;
    int wi = (int)(t % g.W); t /= g.W;
    int h = (int)(t % g.H);
    int n = (int)(t / g.H);
    float acc = 0.f;
    for (int r = 0; r < g.R; ++r) {
        int th = h + g.ph - r * g.dh;
        if (th < 0 || th % g.sh) continue;
        int ho = th / g.sh;
        if (ho >= g.Ho) continue;
        for (int s = 0; s < g.S; ++s) {
            int tw = wi + g.pw - s * g.dw;
            if (tw < 0 || tw % g.sw) continue;
            int wo = tw / g.sw;
            if (wo >= g.Wo) continue;
            const T* gp = dy + (((long)n * g.Ho + ho) * g.Wo + wo) * g.K;
            const T* wp = w + ((long)r * g.S + s) * g.C + c;
            long wstride = (long)g.R * g.S * g.C;
            for (int k = 0; k < g.K; ++k) acc += to_f32(gp[k]) * to_f32(wp[k * wstride]);
        }
    }
    dx[i] = from_f32<T>(epilogue_apply(E, acc, c, i));
}

// One workgroup per dw element: threads stride over output pixels, then a fixed-order
// tree reduction (deterministic).
template <typename T>
__global__ __launch_bounds__(256) void direct_wgrad_kernel(Geom g, const T* __restrict__ x,
                                                           const T* __restrict__ dy,
                                                           float* __restrict__ dw)
{
    __shared__ float red[256];
    long e = blockIdx.x;
    int c = (int)(e % g.C);
    long t = e / g.C;
    int s = (int)(t % g.S); t /= g.S;
    int r = (int)(t % g.R);
    int k = (int)(t / g.R);
    long pixels = (long)g.N * g.Ho * g.Wo;
    float acc = 0.f;
    for (long p = threadIdx.x; p < pixels; p += 256) {
        int wo = (int)(p % g.Wo);
        long q = p / g.Wo;
        int ho = (int)(q % g.Ho);
        int n = (int)(q / g.Ho);
        int h = ho * g.sh - g.ph + r * g.dh;
        int wi = wo * g.sw - g.pw + s * g.dw;
        if (h < 0 || h >= g.H || wi < 0 || wi >= g.W) continue;
        acc += to_f32(dy[p * g.K + k]) * to_f32(x[(((long)n * g.H + h) * g.W + wi) * g.C + c]);
    }
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) dw[e] = red[0];
}

static inline unsigned blocks_for(long total) { return (unsigned)((total + 255) / 256); }

hipError_t launch_direct_fwd(const Geom& g, const __half* x, const __half* w, __half* y, hipStream_t st,
                             const Epilogue& ep)
{
    long total = (long)g.N * g.Ho * g.Wo * g.K;
    hipLaunchKernelGGL(direct_fwd_kernel<__half>, dim3(blocks_for(total)), dim3(256), 0, st, g, x, w, y, total, ep);
    return hipGetLastError();
}

hipError_t launch_direct_dgrad(const Geom& g, const __half* dy, const __half* w, __half* dx, hipStream_t st,
                               const Epilogue& ep)
{
    long total = (long)g.N * g.H * g.W * g.C;
    hipLaunchKernelGGL(direct_dgrad_kernel<__half>, dim3(blocks_for(total)), dim3(256), 0, st, g, dy, w, dx, total, ep);
    return hipGetLastError();
}

hipError_t launch_direct_wgrad(const Geom& g, const __half* x, const __half* dy, float* dw, hipStream_t st)
{
    long total = (long)g.K * g.R * g.S * g.C;
    hipLaunchKernelGGL(direct_wgrad_kernel<__half>, dim3((unsigned)total), dim3(256), 0, st, g, x, dy, dw);
    return hipGetLastError();
}

// The single-precision companion path on descriptors its matrix kernels do not take (channel or
// filter counts that are not a multiple of 4, more than 64 taps, more than 16 stride classes).
hipError_t launch_direct_fwd_f32(const Geom& g, const float* x, const float* w, float* y, hipStream_t st)
{
    long total = (long)g.N * g.Ho * g.Wo * g.K;
    hipLaunchKernelGGL(direct_fwd_kernel<float>, dim3(blocks_for(total)), dim3(256), 0, st, g, x, w, y, total,
                       no_epilogue());
    return hipGetLastError();
}

hipError_t launch_direct_dgrad_f32(const Geom& g, const float* dy, const float* w, float* dx, hipStream_t st)
{
    long total = (long)g.N * g.H * g.W * g.C;
    hipLaunchKernelGGL(direct_dgrad_kernel<float>, dim3(blocks_for(total)), dim3(256), 0, st, g, dy, w, dx, total,
                       no_epilogue());
    return hipGetLastError();
}

hipError_t launch_direct_wgrad_f32(const Geom& g, const float* x, const float* dy, float* dw, hipStream_t st)
{
    long total = (long)g.K * g.R * g.S * g.C;
    hipLaunchKernelGGL(direct_wgrad_kernel<float>, dim3((unsigned)total), dim3(256), 0, st, g, x, dy, dw);
    return hipGetLastError();
}

}  // namespace sdconv
