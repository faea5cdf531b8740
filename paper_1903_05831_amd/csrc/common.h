// Internal declarations shared by the HIP translation units of libsdconv.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>
#include <atomic>
#include "sdconv.h"

namespace sdconv {

// Problem geometry handed to kernels by value.
struct Geom {
    int N, H, W, C;
    int K, R, S;
    int sh, sw, ph, pw, dh, dw;
    int Ho, Wo;
};

inline Geom make_geom(const conv2d_desc& d, int Ho, int Wo)
{
    Geom g;
    g.N = d.N; g.H = d.H; g.W = d.W; g.C = d.C;
    g.K = d.K; g.R = d.R; g.S = d.S;
    g.sh = d.stride_h; g.sw = d.stride_w; g.ph = d.pad_h; g.pw = d.pad_w;
    g.dh = d.dil_h; g.dw = d.dil_w; g.Ho = Ho; g.Wo = Wo;
    return g;
}

// Elementwise tail applied to the fp32 result of a forward or data-gradient pass before its one
// rounding to binary16 (a frozen batch normalisation is the affine part, section 2.3 of the
// paper; shortcut and ReLU are what follows it in a residual block).  c is the destination
// channel, i the flat NHWC index of the destination element:
//   v = acc;  v *= scale[c];  v += bias[c];  v += residual[i];  relu: v = v > 0 ? v : 0;
//   mask: v = mask[i] > 0 ? v : 0          (null pointers / relu == 0 leave a step out)
struct Epilogue {
    const float* scale;
    const float* bias;
    const __half* residual;
    const __half* mask;
    int relu;
    __host__ __device__ bool any() const { return scale || bias || residual || mask || relu; }
};
inline Epilogue no_epilogue() { return Epilogue{nullptr, nullptr, nullptr, nullptr, 0}; }

__device__ __forceinline__ float epilogue_apply(const Epilogue& E, float v, int c, long i)
{
    if (E.scale) v *= E.scale[c];
    if (E.bias) v += E.bias[c];
    if (E.residual) v += __half2float(E.residual[i]);
    if (E.relu) v = v > 0.f ? v : 0.f;
    if (E.mask) v = __half2float(E.mask[i]) > 0.f ? v : 0.f;
    return v;
}

// What the dispatcher decided for one (geometry, pass).
enum Route { ROUTE_DIRECT = 0, ROUTE_IGEMM = 1, ROUTE_THIN = 2, ROUTE_PADK = 3 };
struct Plan {
    Route route;
    int variant;             // tile variant index within the route
    int splits;              // wgrad: number of pixel-range partial sums
    size_t workspace_bytes;  // device scratch the pass needs
    const char* name;        // kernel variant name, static string
    int steps_per_split = 0; // wgrad: 64-pixel steps each pixel range covers
};
Plan plan_fwd(const Geom& g);
Plan plan_dgrad(const Geom& g);
Plan plan_wgrad(const Geom& g);
hipError_t run_fwd(const Geom& g, const Plan& p, const __half* x, const __half* w, __half* y, void* ws, hipStream_t st,
                   const Epilogue& ep = no_epilogue());
hipError_t run_dgrad(const Geom& g, const Plan& p, const __half* dy, const __half* w, __half* dx, void* ws, hipStream_t st,
                     const Epilogue& ep = no_epilogue());
hipError_t run_wgrad(const Geom& g, const Plan& p, const __half* x, const __half* dy, float* dw, void* ws, hipStream_t st);

// Single-precision companion path (conv_f32.hip): matrix kernels for channel and filter counts in
// multiples of 4 (f32_supported), the direct kernels for everything else.
bool f32_supported(const Geom& g);
size_t f32_workspace_bytes(const Geom& g, int pass);
hipError_t run_fwd_f32(const Geom& g, const float* x, const float* w, float* y, hipStream_t st);
hipError_t run_dgrad_f32(const Geom& g, const float* dy, const float* w, float* dx, void* ws, hipStream_t st);
hipError_t run_wgrad_f32(const Geom& g, const float* x, const float* dy, float* dw, void* ws, hipStream_t st);

// Launchers return hipGetLastError() of their launches.  All work goes to `st`.
hipError_t launch_direct_fwd(const Geom& g, const __half* x, const __half* w, __half* y, hipStream_t st,
                             const Epilogue& ep = no_epilogue());
hipError_t launch_direct_dgrad(const Geom& g, const __half* dy, const __half* w, __half* dx, hipStream_t st,
                               const Epilogue& ep = no_epilogue());
hipError_t launch_direct_wgrad(const Geom& g, const __half* x, const __half* dy, float* dw, hipStream_t st);
hipError_t launch_direct_fwd_f32(const Geom& g, const float* x, const float* w, float* y, hipStream_t st);
hipError_t launch_direct_dgrad_f32(const Geom& g, const float* dy, const float* w, float* dx, hipStream_t st);
hipError_t launch_direct_wgrad_f32(const Geom& g, const float* x, const float* dy, float* dw, hipStream_t st);
hipError_t launch_pad_channels(const __half* src, __half* dst, long rows, int K, int Kp, hipStream_t st);
hipError_t launch_pad_rows(const __half* src, __half* dst, long n, long total, hipStream_t st);
hipError_t launch_unpad_channels(const __half* yp, __half* y, long rows, int K, int Kp, const Epilogue& ep, hipStream_t st);
hipError_t launch_copy_f32(const float* src, float* dst, long n, hipStream_t st);
hipError_t launch_tail_pass(__half* t, long pixels, int C, const Epilogue& ep, hipStream_t st);
hipError_t launch_unscale_check(float* grad, size_t n, float inv_scale, const float* scale_on_device,
                                int32_t* flag, hipStream_t st);
hipError_t launch_sgd_momentum(float* w, float* mom, const float* g, void* w16, size_t n, float lr, float mu,
                               float wd, const int32_t* flag, void* state, float growth, float backoff,
                               int32_t interval, hipStream_t st);

}  // namespace sdconv
