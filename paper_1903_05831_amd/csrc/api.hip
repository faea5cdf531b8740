// C-ABI entry points of libsdconv: argument validation, kernel selection, launches.
#include "common.h"
#include "sdconv_bench.h"
#include <math.h>

using namespace sdconv;

static thread_local int g_last_hip_error = 0;

static int hip_status(hipError_t e)
{
    if (e == hipSuccess) return SDCONV_OK;
    g_last_hip_error = (int)e;
    return SDCONV_EHIP;
}

static bool desc_shape(const conv2d_desc* d, int* Ho, int* Wo)
{
    if (!d) return false;
    if (d->N < 1 || d->H < 1 || d->W < 1 || d->C < 1 || d->K < 1 || d->R < 1 || d->S < 1) return false;
    if (d->stride_h < 1 || d->stride_w < 1 || d->dil_h < 1 || d->dil_w < 1) return false;
    if (d->pad_h < 0 || d->pad_w < 0) return false;
    long eh = (long)d->H + 2L * d->pad_h - (long)d->dil_h * (d->R - 1) - 1;
    long ew = (long)d->W + 2L * d->pad_w - (long)d->dil_w * (d->S - 1) - 1;
    if (eh < 0 || ew < 0) return false;
    long ho = eh / d->stride_h + 1, wo = ew / d->stride_w + 1;
    const long lim = 0x7fffffffL;
    long nx = (long)d->N * d->H;
    if (nx > lim || (nx *= d->W) > lim || (nx *= d->C) > lim) return false;
    long ny = (long)d->N * ho;
    if (ny > lim || (ny *= wo) > lim || (ny *= d->K) > lim) return false;
    long nw = (long)d->K * d->R;
    if (nw > lim || (nw *= d->S) > lim || (nw *= d->C) > lim) return false;
    *Ho = (int)ho;
    *Wo = (int)wo;
    return true;
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

extern "C" __attribute__((visibility("default"))) int conv2d_out_shape(const conv2d_desc* desc, int32_t* Ho, int32_t* Wo)
{
    int ho, wo;
    if (!Ho || !Wo || !desc_shape(desc, &ho, &wo)) return SDCONV_EINVAL;
    *Ho = ho;
    *Wo = wo;
    return SDCONV_OK;
}

extern "C" __attribute__((visibility("default"))) size_t conv2d_workspace_bytes(const conv2d_desc* desc, int pass)
{
    int ho, wo;
    if (!desc_shape(desc, &ho, &wo)) return 0;
    Geom g = make_geom(*desc, ho, wo);
    switch (pass) {
        case SDCONV_FWD: return plan_fwd(g).workspace_bytes;
        case SDCONV_DGRAD: return plan_dgrad(g).workspace_bytes;
        case SDCONV_WGRAD: return plan_wgrad(g).workspace_bytes;
        default: return 0;
    }
}

static int check_common(const conv2d_desc* desc, const void* a, const void* b, const void* out,
                        void* ws, size_t ws_bytes, size_t need, int* Ho, int* Wo)
{
    if (!desc_shape(desc, Ho, Wo)) return SDCONV_EINVAL;
    if (!a || !b || !out) return SDCONV_EINVAL;
    if (!aligned16(a) || !aligned16(b) || !aligned16(out)) return SDCONV_EINVAL;
    if (need) {
        if (!ws || ws_bytes < need) return SDCONV_EWORKSPACE;
        if (reinterpret_cast<uintptr_t>(ws) & 255u) return SDCONV_EINVAL;
    }
    return SDCONV_OK;
}

extern "C" __attribute__((visibility("default"))) int conv2d_fwd(const conv2d_desc* desc, const void* x, const void* w, void* y,
                          void* workspace, size_t workspace_bytes, void* hip_stream)
{
    int Ho, Wo;
    if (!desc_shape(desc, &Ho, &Wo)) return SDCONV_EINVAL;
    Geom g = make_geom(*desc, Ho, Wo);
    Plan p = plan_fwd(g);
    int rc = check_common(desc, x, w, y, workspace, workspace_bytes, p.workspace_bytes, &Ho, &Wo);
    if (rc) return rc;
    return hip_status(run_fwd(g, p, (const __half*)x, (const __half*)w, (__half*)y, workspace,
                              (hipStream_t)hip_stream));
}

extern "C" __attribute__((visibility("default"))) int conv2d_dgrad(const conv2d_desc* desc, const void* dy, const void* w, void* dx,
                            void* workspace, size_t workspace_bytes, void* hip_stream)
{
    int Ho, Wo;
    if (!desc_shape(desc, &Ho, &Wo)) return SDCONV_EINVAL;
    Geom g = make_geom(*desc, Ho, Wo);
    Plan p = plan_dgrad(g);
    int rc = check_common(desc, dy, w, dx, workspace, workspace_bytes, p.workspace_bytes, &Ho, &Wo);
    if (rc) return rc;
    return hip_status(run_dgrad(g, p, (const __half*)dy, (const __half*)w, (__half*)dx, workspace,
                                (hipStream_t)hip_stream));
}

extern "C" __attribute__((visibility("default"))) int conv2d_fwd_fused(const conv2d_desc* desc, const void* x, const void* w,
                                                                       const conv2d_fwd_epilogue* ep, void* y,
                                                                       void* workspace, size_t workspace_bytes,
                                                                       void* hip_stream)
{
    int Ho, Wo;
    if (!desc_shape(desc, &Ho, &Wo) || !ep) return SDCONV_EINVAL;
    if (!aligned16(ep->scale) || !aligned16(ep->bias) || !aligned16(ep->residual)) return SDCONV_EINVAL;
    Geom g = make_geom(*desc, Ho, Wo);
    Plan p = plan_fwd(g);
    int rc = check_common(desc, x, w, y, workspace, workspace_bytes, p.workspace_bytes, &Ho, &Wo);
    if (rc) return rc;
    Epilogue E{ep->scale, ep->bias, static_cast<const __half*>(ep->residual), nullptr, ep->relu ? 1 : 0};
    return hip_status(run_fwd(g, p, (const __half*)x, (const __half*)w, (__half*)y, workspace,
                              (hipStream_t)hip_stream, E));
}

extern "C" __attribute__((visibility("default"))) int conv2d_dgrad_fused(const conv2d_desc* desc, const void* dy, const void* w,
                                                                         const conv2d_dgrad_epilogue* ep, void* dx,
                                                                         void* workspace, size_t workspace_bytes,
                                                                         void* hip_stream)
{
    int Ho, Wo;
    if (!desc_shape(desc, &Ho, &Wo) || !ep) return SDCONV_EINVAL;
    if (!aligned16(ep->scale) || !aligned16(ep->relu_mask)) return SDCONV_EINVAL;
    Geom g = make_geom(*desc, Ho, Wo);
    Plan p = plan_dgrad(g);
    int rc = check_common(desc, dy, w, dx, workspace, workspace_bytes, p.workspace_bytes, &Ho, &Wo);
    if (rc) return rc;
    Epilogue E{ep->scale, nullptr, nullptr, static_cast<const __half*>(ep->relu_mask), 0};
    return hip_status(run_dgrad(g, p, (const __half*)dy, (const __half*)w, (__half*)dx, workspace,
                                (hipStream_t)hip_stream, E));
}

extern "C" __attribute__((visibility("default"))) int conv2d_wgrad(const conv2d_desc* desc, const void* x, const void* dy, float* dw,
                            void* workspace, size_t workspace_bytes, void* hip_stream)
{
    int Ho, Wo;
    if (!desc_shape(desc, &Ho, &Wo)) return SDCONV_EINVAL;
    Geom g = make_geom(*desc, Ho, Wo);
    Plan p = plan_wgrad(g);
    int rc = check_common(desc, x, dy, dw, workspace, workspace_bytes, p.workspace_bytes, &Ho, &Wo);
    if (rc) return rc;
    return hip_status(run_wgrad(g, p, (const __half*)x, (const __half*)dy, dw, workspace,
                                (hipStream_t)hip_stream));
}

namespace sdconv {
int wgrad_static_scratch(const Geom& g, const Plan& p, const __half* x, const __half* dy, float* dw, hipStream_t st,
                         hipError_t* hip_error);
}

extern "C" __attribute__((visibility("default"))) int conv2d_wgrad_static_scratch(const conv2d_desc* desc, const void* x,
                                                                                  const void* dy, float* dw,
                                                                                  void* hip_stream)
{
    int Ho, Wo;
    if (!desc_shape(desc, &Ho, &Wo)) return SDCONV_EINVAL;
    Geom g = make_geom(*desc, Ho, Wo);
    Plan p = plan_wgrad(g);
    int rc = check_common(desc, x, dy, dw, nullptr, 0, 0, &Ho, &Wo);
    if (rc) return rc;
    hipError_t e = hipSuccess;
    rc = wgrad_static_scratch(g, p, (const __half*)x, (const __half*)dy, dw, (hipStream_t)hip_stream, &e);
    if (rc == SDCONV_EHIP) g_last_hip_error = (int)e;
    return rc;
}

extern "C" __attribute__((visibility("default"))) size_t conv2d_workspace_bytes_f32(const conv2d_desc* desc, int pass)
{
    int Ho, Wo;
    if (!desc_shape(desc, &Ho, &Wo)) return 0;
    return f32_workspace_bytes(make_geom(*desc, Ho, Wo), pass);
}

static int f32_call(const conv2d_desc* desc, int pass, const float* a, const float* b, float* out, void* workspace,
                    size_t workspace_bytes, void* hip_stream)
{
    int Ho, Wo;
    if (!desc_shape(desc, &Ho, &Wo)) return SDCONV_EINVAL;
    Geom g = make_geom(*desc, Ho, Wo);
    // 32-bit element offsets inside the kernels
    const size_t lim = (size_t)1 << 31;
    if ((size_t)g.N * g.H * g.W * g.C >= lim || (size_t)g.N * Ho * Wo * g.K >= lim) return SDCONV_EINVAL;
    int rc = check_common(desc, a, b, out, workspace, workspace_bytes, f32_workspace_bytes(g, pass), &Ho, &Wo);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)hip_stream;
    if (pass == SDCONV_FWD) return hip_status(run_fwd_f32(g, a, b, out, st));
    if (pass == SDCONV_DGRAD) return hip_status(run_dgrad_f32(g, a, b, out, workspace, st));
    return hip_status(run_wgrad_f32(g, a, b, out, workspace, st));
}

extern "C" __attribute__((visibility("default"))) int conv2d_fwd_f32(const conv2d_desc* desc, const float* x, const float* w,
                                                                     float* y, void* workspace, size_t workspace_bytes,
                                                                     void* hip_stream)
{
    return f32_call(desc, SDCONV_FWD, x, w, y, workspace, workspace_bytes, hip_stream);
}

extern "C" __attribute__((visibility("default"))) int conv2d_dgrad_f32(const conv2d_desc* desc, const float* dy,
                                                                       const float* w, float* dx, void* workspace,
                                                                       size_t workspace_bytes, void* hip_stream)
{
    return f32_call(desc, SDCONV_DGRAD, dy, w, dx, workspace, workspace_bytes, hip_stream);
}

extern "C" __attribute__((visibility("default"))) int conv2d_wgrad_f32(const conv2d_desc* desc, const float* x,
                                                                       const float* dy, float* dw, void* workspace,
                                                                       size_t workspace_bytes, void* hip_stream)
{
    return f32_call(desc, SDCONV_WGRAD, x, dy, dw, workspace, workspace_bytes, hip_stream);
}

extern "C" __attribute__((visibility("default"))) int grad_unscale_check(float* grad, size_t n, float inv_scale, int32_t* found_nonfinite,
                                  void* hip_stream)
{
    if (!found_nonfinite) return SDCONV_EINVAL;
    if (n > 0 && !grad) return SDCONV_EINVAL;
    if (reinterpret_cast<uintptr_t>(grad) & 3u) return SDCONV_EINVAL;
    if (reinterpret_cast<uintptr_t>(found_nonfinite) & 3u) return SDCONV_EINVAL;
    if (!isfinite(inv_scale) || !(inv_scale > 0.f)) return SDCONV_EINVAL;
    if (n >= ((size_t)1 << 40)) return SDCONV_EINVAL;
    return hip_status(launch_unscale_check(grad, n, inv_scale, nullptr, found_nonfinite, (hipStream_t)hip_stream));
}

extern "C" __attribute__((visibility("default"))) int grad_unscale_check_dynamic(float* grad, size_t n,
                                                                                 const loss_scale_state* state,
                                                                                 int32_t* found_nonfinite,
                                                                                 void* hip_stream)
{
    if (!found_nonfinite || !state) return SDCONV_EINVAL;
    if (n > 0 && !grad) return SDCONV_EINVAL;
    if (reinterpret_cast<uintptr_t>(grad) & 3u) return SDCONV_EINVAL;
    if ((reinterpret_cast<uintptr_t>(found_nonfinite) & 3u) || (reinterpret_cast<uintptr_t>(state) & 3u))
        return SDCONV_EINVAL;
    if (n >= ((size_t)1 << 40)) return SDCONV_EINVAL;
    return hip_status(launch_unscale_check(grad, n, 1.0f, &state->scale, found_nonfinite, (hipStream_t)hip_stream));
}

extern "C" __attribute__((visibility("default"))) int sgd_momentum_update(
    float* master_w, float* momentum_buf, const float* grad, void* w_half, size_t n, float lr, float momentum,
    float weight_decay, const int32_t* found_nonfinite, loss_scale_state* state, float growth, float backoff,
    int32_t interval, void* hip_stream)
{
    if (!found_nonfinite || !state) return SDCONV_EINVAL;
    if (n > 0 && (!master_w || !momentum_buf || !grad || !w_half)) return SDCONV_EINVAL;
    if ((reinterpret_cast<uintptr_t>(master_w) | reinterpret_cast<uintptr_t>(momentum_buf) |
         reinterpret_cast<uintptr_t>(grad)) & 15u)
        return SDCONV_EINVAL;
    if (reinterpret_cast<uintptr_t>(w_half) & 7u) return SDCONV_EINVAL;
    if ((reinterpret_cast<uintptr_t>(found_nonfinite) & 3u) || (reinterpret_cast<uintptr_t>(state) & 3u))
        return SDCONV_EINVAL;
    if (!isfinite(lr) || !isfinite(momentum) || !isfinite(weight_decay)) return SDCONV_EINVAL;
    if (!isfinite(growth) || !isfinite(backoff) || !(growth > 0.f) || !(backoff > 0.f) || interval < 1)
        return SDCONV_EINVAL;
    if (n >= ((size_t)1 << 40)) return SDCONV_EINVAL;
    return hip_status(launch_sgd_momentum(master_w, momentum_buf, grad, w_half, n, lr, momentum, weight_decay,
                                          found_nonfinite, state, growth, backoff, interval,
                                          (hipStream_t)hip_stream));
}

extern "C" __attribute__((visibility("default"))) const char* sdconv_status_string(int status)
{
    switch (status) {
        case SDCONV_OK: return "ok";
        case SDCONV_EINVAL: return "invalid argument";
        case SDCONV_EUNSUPPORTED: return "unsupported configuration";
        case SDCONV_EWORKSPACE: return "workspace missing or too small";
        case SDCONV_EHIP: return "HIP runtime error";
        default: return "unknown status";
    }
}

extern "C" __attribute__((visibility("default"))) int sdconv_last_hip_error(void) { return g_last_hip_error; }

extern "C" __attribute__((visibility("default"))) const char* sdconv_kernel_name(const conv2d_desc* desc, int pass)
{
    int ho, wo;
    if (!desc_shape(desc, &ho, &wo)) return "invalid";
    Geom g = make_geom(*desc, ho, wo);
    switch (pass) {
        case SDCONV_FWD: return plan_fwd(g).name;
        case SDCONV_DGRAD: return plan_dgrad(g).name;
        case SDCONV_WGRAD: return plan_wgrad(g).name;
        default: return "invalid";
    }
}

namespace sdconv { hipError_t launch_mfma_ceiling(float* out, int blocks, int iters, hipStream_t st); }

extern "C" __attribute__((visibility("default"))) int sdconv_tail_pass(void* t, size_t pixels, int32_t channels,
                                                                       const float* scale, const float* bias,
                                                                       const void* residual, const void* relu_mask,
                                                                       int32_t relu, void* hip_stream)
{
    if (!t || channels <= 0 || channels % 8 || pixels == 0 || pixels * (size_t)channels >= ((size_t)1 << 31))
        return SDCONV_EINVAL;
    if (!aligned16(t) || !aligned16(scale) || !aligned16(bias) || !aligned16(residual) || !aligned16(relu_mask))
        return SDCONV_EINVAL;
    Epilogue E{scale, bias, static_cast<const __half*>(residual), static_cast<const __half*>(relu_mask), relu ? 1 : 0};
    return hip_status(launch_tail_pass(static_cast<__half*>(t), (long)pixels, channels, E, (hipStream_t)hip_stream));
}

extern "C" __attribute__((visibility("default"))) int sdconv_mfma_ceiling(float* scratch, int blocks, int iters,
                                                                          void* hip_stream)
{
    if (!scratch || blocks <= 0 || iters <= 0) return SDCONV_EINVAL;
    hipError_t e = sdconv::launch_mfma_ceiling(scratch, blocks, iters, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) { g_last_hip_error = (int)e; return SDCONV_EHIP; }
    return SDCONV_OK;
}
