/*
 * sdconv -- mixed-precision 2-D convolution for detector training on MI355X (gfx950).
 *
 * C ABI of the hot path behind the paper's mixed-precision training feature
 * (section 2.2, "Mixed Precision Training": half-precision compute with the loss
 * scaling of Micikevicius et al.; Figure 1(b) measures it on a Faster R-CNN with a
 * ResNet-50-C4 backbone).  The library holds hand-written HIP kernels only; callers
 * bring device memory and a HIP stream.
 *
 * Common conventions
 *   - Every data pointer is a DEVICE pointer to a dense, contiguous tensor, aligned to
 *     16 bytes, owned by the caller.  The library never allocates, frees or keeps device
 *     memory.  Inputs and outputs must not overlap.
 *   - Layouts (last index fastest):  x, dx [N][H][W][C]   y, dy [N][Ho][Wo][K]
 *     w, dw [K][R][S][C].  x, w, y, dy, dx are IEEE binary16; dw is binary32.
 *     Ho = floor((H + 2*pad_h - dil_h*(R-1) - 1) / stride_h) + 1, likewise Wo.
 *   - Cross-correlation (no kernel flip), zero padding, groups = 1, no bias.
 *   - Products are binary16 x binary16 accumulated in binary32 (MFMA); y and dx are
 *     rounded once (nearest even) from the binary32 sum; dw stays binary32.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).  All
 *     device work is enqueued on it and the call returns without waiting.
 *   - `workspace` is caller-owned device scratch of at least conv2d_workspace_bytes()
 *     bytes (may be NULL when that is 0), 256-byte aligned.  Its contents are undefined
 *     after the call.  Calls that share a workspace must be ordered on one stream.
 *   - Outputs are overwritten in full (beta = 0); dx positions that no filter tap
 *     reaches are written as +0.
 *   - Return value: SDCONV_OK or a negative SDCONV_E* code.  SDCONV_EINVAL, SDCONV_EUNSUPPORTED
 *     and SDCONV_EWORKSPACE are found before anything is enqueued.  SDCONV_EHIP reports a HIP
 *     call that failed; a pass that takes several launches (a filter copy or padding kernel in
 *     front of the main kernel, a reduction behind it) may then have enqueued the earlier ones,
 *     and the output is undefined.  No exception crosses this boundary.
 *   - Every tensor must hold fewer than 2^31 elements (kernels use 32-bit offsets).
 *   - Thread safety: calls from several host threads are safe.  The library's own state is a
 *     per-thread record of the last HIP error, once-only kernel attribute settings, and small
 *     device-side records that overlapping grad_unscale_check* calls take turns on (up to 1024
 *     such calls may be in flight on one device at a time).
 *   - Environment: none is read, unless SDCONV_TUNE=1 was set before the first call: then the
 *     SDCONV_* variables of the tuner and of the variant tests override the kernel choice.
 */
#ifndef SDCONV_H
#define SDCONV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int32_t N, H, W, C;          /* input tensor, NHWC                       */
    int32_t K, R, S;             /* filter bank KRSC, K = output channels    */
    int32_t stride_h, stride_w;  /* >= 1                                     */
    int32_t pad_h, pad_w;        /* >= 0, zeros on both sides                */
    int32_t dil_h, dil_w;        /* >= 1                                     */
} conv2d_desc;

enum {
    SDCONV_OK = 0,
    SDCONV_EINVAL = -1,       /* null pointer, non-positive size, empty output, bad scale, misalignment */
    SDCONV_EUNSUPPORTED = -2, /* reserved: every valid descriptor is served                             */
    SDCONV_EWORKSPACE = -3,   /* workspace missing or smaller than conv2d_workspace_bytes()             */
    SDCONV_EHIP = -4          /* a HIP call failed; see sdconv_last_hip_error()                         */
};

enum { SDCONV_FWD = 0, SDCONV_DGRAD = 1, SDCONV_WGRAD = 2 };

/* Output extent of the convolution `desc` describes.  Host-only, touches no device.
 * Returns SDCONV_EINVAL for an invalid descriptor or an empty output. */
int conv2d_out_shape(const conv2d_desc *desc, int32_t *Ho, int32_t *Wo);

/* Device scratch the given pass needs for `desc` (0 for an invalid descriptor or pass).
 * Host-only.  wgrad uses it for split-K partial sums, dgrad for a re-laid-out filter. */
size_t conv2d_workspace_bytes(const conv2d_desc *desc, int pass);

/* Forward: y[n,ho,wo,k] = sum_{r,s,c} x[n, ho*stride_h - pad_h + r*dil_h,
 *                                         wo*stride_w - pad_w + s*dil_w, c] * w[k,r,s,c],
 * reads outside the image are zero.  (Half-precision forward compute of section 2.2.) */
int conv2d_fwd(const conv2d_desc *desc, const void *x, const void *w, void *y,
               void *workspace, size_t workspace_bytes, void *hip_stream);

/* Data gradient (adjoint of conv2d_fwd in x):
 * dx[n,h,w,c] = sum over (k,r,s) with ho*stride_h - pad_h + r*dil_h == h and
 *               wo*stride_w - pad_w + s*dil_w == w of dy[n,ho,wo,k] * w[k,r,s,c].
 * (Half-precision backward compute of section 2.2; dy carries the loss scale.) */
int conv2d_dgrad(const conv2d_desc *desc, const void *dy, const void *w, void *dx,
                 void *workspace, size_t workspace_bytes, void *hip_stream);

/* Weight gradient (adjoint of conv2d_fwd in w), binary32 result:
 * dw[k,r,s,c] = sum_{n,ho,wo} dy[n,ho,wo,k] * x[n, ho*stride_h - pad_h + r*dil_h,
 *                                                 wo*stride_w - pad_w + s*dil_w, c].
 * The reduction over pixels is split across workgroups; partial sums are combined in a
 * fixed order, so results are bit-identical from run to run.  (fp32 master gradients of
 * the mixed-precision recipe section 2.2 adopts.) */
int conv2d_wgrad(const conv2d_desc *desc, const void *x, const void *dy, float *dw,
                 void *workspace, size_t workspace_bytes, void *hip_stream);

/* Loss-scale removal and overflow check (the loss scaling section 2.2 adopts):
 * grad[i] <- grad[i] * inv_scale (one binary32 rounding) for i < n, in place, every
 * element written; *found_nonfinite (device int32) <- 1 if any grad[i] was +inf, -inf or
 * NaN BEFORE scaling, else 0.  The flag is cleared on the stream by this call.
 * n = 0 is legal (flag becomes 0, grad may be NULL).  inv_scale must be finite and > 0. */
int grad_unscale_check(float *grad, size_t n, float inv_scale, int32_t *found_nonfinite,
                       void *hip_stream);

/* ---- optimizer tail (the step right after the overflow check) ------------------------------
 * Section 2.2 of the paper adopts the loss scaling of its cited mixed-precision recipe; the
 * scale schedule and the optimizer are not spelled out there.  Taken here: the dynamic
 * schedule of that recipe and SGD with momentum on fp32 master weights in the formulation of
 * the framework the paper builds on. */

/* Loss-scale state in DEVICE memory (4-byte aligned), owned by the caller. */
typedef struct {
    float scale;         /* current loss scale S */
    int32_t good_steps;  /* steps without overflow since the scale last changed */
} loss_scale_state;

/* grad_unscale_check with inv_scale = 1 / state->scale read on the device (one correctly
 * rounded binary32 division), so that the scale never has to visit the host.  state is only
 * read.  Same alignment, ownership and error rules as grad_unscale_check. */
int grad_unscale_check_dynamic(float *grad, size_t n, const loss_scale_state *state,
                               int32_t *found_nonfinite, void *hip_stream);

/* One optimizer step over n elements of flat device buffers, then one loss-scale transition.
 *   if *found_nonfinite == 0, for every i (each operation a separate binary32 operation):
 *       momentum_buf[i] <- momentum*momentum_buf[i] - lr*(grad[i] + weight_decay*master_w[i])
 *       master_w[i]     <- master_w[i] + momentum_buf[i]
 *   else master_w and momentum_buf are left untouched (the step is skipped);
 *   always: w_half[i] <- binary16(master_w[i]), round to nearest even (n halves, 8-byte aligned);
 *   then:   flag set -> state->scale *= backoff, good_steps = 0;
 *           else ++good_steps, and when it reaches interval: scale *= growth, good_steps = 0.
 * grad is the UNSCALED gradient (after grad_unscale_check*), read only.  master_w,
 * momentum_buf and grad are 16-byte aligned fp32; found_nonfinite and state are device
 * pointers, the flag is only read.  Asynchronous on hip_stream; no host synchronisation.
 * SDCONV_EINVAL: null pointers (with n > 0), misalignment, non-finite lr / momentum /
 * weight_decay, growth or backoff not finite and > 0, interval < 1.  n = 0 only advances the
 * state. */
int sgd_momentum_update(float *master_w, float *momentum_buf, const float *grad, void *w_half,
                        size_t n, float lr, float momentum, float weight_decay,
                        const int32_t *found_nonfinite, loss_scale_state *state, float growth,
                        float backoff, int32_t interval, void *hip_stream);

/* ---- fused epilogues ------------------------------------------------------------------------
 * Section 2.3 of the paper recalls that detectors are trained with the batch-normalisation
 * parameters frozen: such a layer is a fixed per-channel affine map of the convolution output,
 * followed in a residual block by the shortcut addition and the ReLU.  These two calls apply
 * that elementwise tail to the binary32 result of the pass, before its one rounding to
 * binary16, instead of a separate pass over the activation tensor. */

/* Tail of the forward pass.  Device pointers, each optional (NULL leaves the step out):
 *   scale, bias  binary32 [K], 16-byte aligned (frozen BN: scale = gamma / sqrt(var + eps),
 *                bias = beta - mean * scale);
 *   residual     binary16 [N][Ho][Wo][K] (the shortcut branch), 16-byte aligned, read only;
 *   relu         nonzero: v <- v > 0 ? v : +0  (a NaN becomes +0). */
typedef struct {
    const float *scale;
    const float *bias;
    const void *residual;
    int32_t relu;
} conv2d_fwd_epilogue;

/* y[n,ho,wo,k] = act( scale[k] * conv2d_fwd(x, w)[n,ho,wo,k] + bias[k] + residual[n,ho,wo,k] ),
 * every operation in binary32 on the binary32 accumulator, one rounding to binary16 at the end.
 * (Exception: with a filter count K that is not a multiple of 8 and C that is, the convolution
 * result is rounded to binary16 first and the tail is applied to that value: two roundings.)
 * `ep` itself is a HOST pointer and must not be NULL (all members NULL / 0 gives conv2d_fwd).
 * Workspace, alignment, ownership and error rules as conv2d_fwd; y must not overlap residual. */
int conv2d_fwd_fused(const conv2d_desc *desc, const void *x, const void *w,
                     const conv2d_fwd_epilogue *ep, void *y, void *workspace,
                     size_t workspace_bytes, void *hip_stream);

/* Tail of the data gradient: the chain rule through a = relu(scale * z + bias), the activation
 * that feeds this convolution (dx is then dL/dz of the layer before).  Device pointers, each
 * optional:
 *   scale      binary32 [C], 16-byte aligned (the affine map's factor; bias does not enter);
 *   relu_mask  binary16 [N][H][W][C], 16-byte aligned: the activation a itself (the x of the
 *              forward pass); the gradient passes where relu_mask > 0, strictly. */
typedef struct {
    const float *scale;
    const void *relu_mask;
} conv2d_dgrad_epilogue;

/* dx[n,h,w,c] = relu_mask[n,h,w,c] > 0 ? scale[c] * conv2d_dgrad(dy, w)[n,h,w,c] : +0,
 * in binary32 on the binary32 accumulator, one rounding to binary16.  `ep` is a HOST pointer,
 * not NULL.  Otherwise as conv2d_dgrad; dx must not overlap relu_mask. */
int conv2d_dgrad_fused(const conv2d_desc *desc, const void *dy, const void *w,
                       const conv2d_dgrad_epilogue *ep, void *dx, void *workspace,
                       size_t workspace_bytes, void *hip_stream);

/* ---- callers that cannot allocate device memory ---------------------------------------------
 * For code under HIP graph capture, tight serving loops and harnesses that forbid hipMalloc:
 * conv2d_wgrad without a workspace argument.  The scratch conv2d_wgrad would take from its
 * workspace (split-K partial sums, padded copies) lives in a device array of
 * SDCONV_STATIC_SCRATCH_BYTES bytes inside the library, one copy per GPU, held until the process
 * ends.  The call allocates and frees nothing and calls no allocating routine; its first call
 * on a device looks the array's address up once (do that call outside a capture).
 * Same arguments, results (bit for bit), alignment, ownership and asynchrony as conv2d_wgrad.
 * SDCONV_EWORKSPACE when conv2d_workspace_bytes(desc, SDCONV_WGRAD) exceeds
 * SDCONV_STATIC_SCRATCH_BYTES (nothing is enqueued); the other codes as conv2d_wgrad.
 * All calls on one GPU share that GPU's array: calls that may overlap in time (different
 * streams without an ordering between them, several host threads) race on it and give wrong
 * results; order them on one stream or with events. */
#define SDCONV_STATIC_SCRATCH_BYTES 67108864 /* 64 MiB */
int conv2d_wgrad_static_scratch(const conv2d_desc *desc, const void *x, const void *dy, float *dw,
                                void *hip_stream);

/* ---- single-precision companion path ----------------------------------------------------------
 * Section 2.2 and Figure 1(b) of the paper compare mixed-precision training with full-precision
 * (FP32) training.  These calls run the same three passes on binary32 tensors (binary32
 * products and accumulation on the fp32 matrix instructions, results binary32), so that the
 * comparison can be made on this hardware; they are a measurement companion, not a tuned path.
 * Layouts, conventions, alignment, ownership, asynchrony and error rules are those of the
 * half-precision calls with every tensor binary32.  C and K multiples of 4 with at most 64 filter
 * taps and stride_h * stride_w <= 16 run on the matrix instructions; every other valid
 * descriptor is served by one-thread-per-output kernels. */
size_t conv2d_workspace_bytes_f32(const conv2d_desc *desc, int pass);
int conv2d_fwd_f32(const conv2d_desc *desc, const float *x, const float *w, float *y,
                   void *workspace, size_t workspace_bytes, void *hip_stream);
int conv2d_dgrad_f32(const conv2d_desc *desc, const float *dy, const float *w, float *dx,
                     void *workspace, size_t workspace_bytes, void *hip_stream);
int conv2d_wgrad_f32(const conv2d_desc *desc, const float *x, const float *dy, float *dw,
                     void *workspace, size_t workspace_bytes, void *hip_stream);

/* Static, human-readable text for a status code. */
const char *sdconv_status_string(int status);

/* hipError_t (as int) of the last SDCONV_EHIP returned on the calling thread, else 0. */
int sdconv_last_hip_error(void);

/* Name of the kernel variant the dispatcher picks for (desc, pass), e.g. for profiles.
 * Static string; "invalid" for a bad descriptor. */
const char *sdconv_kernel_name(const conv2d_desc *desc, int pass);

#ifdef __cplusplus
}
#endif
#endif /* SDCONV_H */
