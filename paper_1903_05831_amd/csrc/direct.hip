// Direct (one result per thread / per block) convolution kernels.  They accept every
// valid descriptor and are the route for channel counts the MFMA kernels do not tile
// (C or K not a multiple of 8).  fp16 inputs, fp32 accumulation, the optional elementwise
// tail in fp32, one rounding on store.
#include "common.h"

namespace sdconv {

__global__ __launch_bounds__(256) void direct_fwd_kernel(Geom g, const __half* __restrict__ x,
                                                         const __half* __restrict__ w,
                                                         __half* __restrict__ y, long total, Epilogue E)
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
            const __half* xp = x + (((long)n * g.H + h) * g.W + wi) * g.C;
            const __half* wp = w + (((long)k * g.R + r) * g.S + s) * g.C;
            for (int c = 0; c < g.C; ++c) acc += __half2float(xp[c]) * __half2float(wp[c]);
        }
    }
    y[i] = __float2half_rn(epilogue_apply(E, acc, k, i));
}

__global__ __launch_bounds__(256) void direct_dgrad_kernel(Geom g, const __half* __restrict__ dy,
                                                           const __half* __restrict__ w,
                                                           __half* __restrict__ dx, long total, Epilogue E)
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
            const __half* gp = dy + (((long)n * g.Ho + ho) * g.Wo + wo) * g.K;
            const __half* wp = w + ((long)r * g.S + s) * g.C + c;
            long wstride = (long)g.R * g.S * g.C;
            for (int k = 0; k < g.K; ++k) acc += __half2float(gp[k]) * __half2float(wp[k * wstride]);
        }
    }
    dx[i] = __float2half_rn(epilogue_apply(E, acc, c, i));
}

// One workgroup per dw element: threads stride over output pixels, then a fixed-order
// tree reduction (deterministic).
__global__ __launch_bounds__(256) void direct_wgrad_kernel(Geom g, const __half* __restrict__ x,
                                                           const __half* __restrict__ dy,
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
        acc += __half2float(dy[p * g.K + k]) *
               __half2float(x[(((long)n * g.H + h) * g.W + wi) * g.C + c]);
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
    hipLaunchKernelGGL(direct_fwd_kernel, dim3(blocks_for(total)), dim3(256), 0, st, g, x, w, y, total, ep);
    return hipGetLastError();
}

hipError_t launch_direct_dgrad(const Geom& g, const __half* dy, const __half* w, __half* dx, hipStream_t st,
                               const Epilogue& ep)
{
    long total = (long)g.N * g.H * g.W * g.C;
    hipLaunchKernelGGL(direct_dgrad_kernel, dim3(blocks_for(total)), dim3(256), 0, st, g, dy, w, dx, total, ep);
    return hipGetLastError();
}

hipError_t launch_direct_wgrad(const Geom& g, const __half* x, const __half* dy, float* dw, hipStream_t st)
{
    long total = (long)g.K * g.R * g.S * g.C;
    hipLaunchKernelGGL(direct_wgrad_kernel, dim3((unsigned)total), dim3(256), 0, st, g, x, dy, dw);
    return hipGetLastError();
}

}  // namespace sdconv
