/*
 * CPU oracle for the mixed-precision convolution path (test infrastructure only).
 *
 * This file is a checker, not a product: it may be called from tests, from the
 * smoke check and from the benchmark's CPU-baseline leg, and from nowhere else.
 * It shares no code, header, table or helper with the HIP library.
 *
 * What it computes: the textbook definitions of a 2-D cross-correlation and of
 * its two adjoints, evaluated in fp64 on inputs that are given as IEEE binary16
 * bit patterns (the half-precision compute of the paper's "Mixed Precision
 * Training" subsection, section 2.2), and the loss-scale removal with overflow
 * detection that the loss-scaling recipe adopted in that subsection needs.
 * The *_f32 entry points evaluate the same sums on binary32 inputs (the full-precision
 * training that subsection compares against).
 * Nothing is blocked, fused or reordered: every output element is one plain
 * nested sum, so the code can be compared with the formulas by eye.
 *
 * Layouts (dense, row-major, last index fastest):
 *   x, dx : [N][H][W][C]         y, dy : [N][Ho][Wo][K]        w, dw : [K][R][S][C]
 *   Ho = floor((H + 2*pad_h - dil_h*(R-1) - 1) / stride_h) + 1   (same for Wo)
 *
 * Parity pins (see tests): brute-force im2col + library matmul, 1x1 = matmul,
 * adjoint identities with one-hot probes, delta-kernel shift, all-ones border
 * counts (hand-written fixture), stride and dilation invariants, and an
 * independent library convolution in float64.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t N, H, W, C;
    int32_t K, R, S;
    int32_t stride_h, stride_w, pad_h, pad_w, dil_h, dil_w;
} oracle_conv_desc;

/* ---- binary16 -> double, exact ------------------------------------------------ */

static double half_bits_to_double(uint16_t b)
{
    int sign = (b >> 15) & 1;
    int expo = (b >> 10) & 0x1f;
    int frac = b & 0x3ff;
    double v;
    if (expo == 0) {
        v = ldexp((double)frac, -24);               /* zero and subnormals */
    } else if (expo == 31) {
        v = frac ? NAN : INFINITY;
    } else {
        v = ldexp((double)(frac | 0x400), expo - 25);
    }
    return sign ? -v : v;
}

/* Whole tensors are widened once per call so the sums below read doubles. */
static double *widen(const uint16_t *src, size_t n)
{
    double *dst = (double *)malloc((n ? n : 1) * sizeof(double));
    if (!dst) return NULL;
    /* independent elements: the loop is shared among the threads, nothing else changes */
#pragma omp parallel for schedule(static)
    for (long long i = 0; i < (long long)n; ++i) dst[i] = half_bits_to_double(src[i]);
    return dst;
}

/* binary32 -> double is exact as well (the single-precision companion path) */
static double *widen_f32(const float *src, size_t n)
{
    double *dst = (double *)malloc((n ? n : 1) * sizeof(double));
    if (!dst) return NULL;
#pragma omp parallel for schedule(static)
    for (long long i = 0; i < (long long)n; ++i) dst[i] = (double)src[i];
    return dst;
}

static int out_extent(int in, int pad, int dil, int ksz, int stride)
{
    int span = in + 2 * pad - dil * (ksz - 1) - 1;
    if (span < 0) return 0;
    return span / stride + 1;
}

int oracle_conv2d_out_shape(const oracle_conv_desc *d, int32_t *Ho, int32_t *Wo)
{
    if (!d || d->N < 1 || d->H < 1 || d->W < 1 || d->C < 1 || d->K < 1 || d->R < 1 ||
        d->S < 1 || d->stride_h < 1 || d->stride_w < 1 || d->pad_h < 0 || d->pad_w < 0 ||
        d->dil_h < 1 || d->dil_w < 1)
        return -1;
    int ho = out_extent(d->H, d->pad_h, d->dil_h, d->R, d->stride_h);
    int wo = out_extent(d->W, d->pad_w, d->dil_w, d->S, d->stride_w);
    if (ho < 1 || wo < 1) return -1;
    *Ho = ho;
    *Wo = wo;
    return 0;
}

/* ---- one output element of each pass, straight from its definition ------------- */

/* y[n,ho,wo,k] = sum_{r,s,c} x[n, ho*sh - ph + r*dh, wo*sw - pw + s*dw, c] * w[k,r,s,c],
 * taps outside the image contribute zero. */
static double fwd_element(const oracle_conv_desc *d, const double *x, const double *w,
                          int n, int ho, int wo, int k)
{
    double acc = 0.0;
    for (int r = 0; r < d->R; ++r) {
        int h = ho * d->stride_h - d->pad_h + r * d->dil_h;
        if (h < 0 || h >= d->H) continue;
        for (int s = 0; s < d->S; ++s) {
            int wi = wo * d->stride_w - d->pad_w + s * d->dil_w;
            if (wi < 0 || wi >= d->W) continue;
            const double *xp = x + (((size_t)n * d->H + h) * d->W + wi) * d->C;
            const double *wp = w + (((size_t)k * d->R + r) * d->S + s) * d->C;
            for (int c = 0; c < d->C; ++c) acc += xp[c] * wp[c];
        }
    }
    return acc;
}

/* dx[n,h,w,c] = sum over (k,r,s) of dy[n,ho,wo,k] * w[k,r,s,c] for exactly those taps
 * whose forward read position equals (h,w): ho*sh - ph + r*dh == h and likewise for w.
 * Written as a gather over taps; a position that no tap reaches gets the empty sum. */
static double dgrad_element(const oracle_conv_desc *d, const double *dy, const double *w,
                            int Ho, int Wo, int n, int h, int wi, int c)
{
    double acc = 0.0;
    for (int r = 0; r < d->R; ++r) {
        int th = h + d->pad_h - r * d->dil_h;
        if (th < 0 || th % d->stride_h != 0) continue;
        int ho = th / d->stride_h;
        if (ho >= Ho) continue;
        for (int s = 0; s < d->S; ++s) {
            int tw = wi + d->pad_w - s * d->dil_w;
            if (tw < 0 || tw % d->stride_w != 0) continue;
            int wo = tw / d->stride_w;
            if (wo >= Wo) continue;
            const double *gp = dy + (((size_t)n * Ho + ho) * Wo + wo) * d->K;
            for (int k = 0; k < d->K; ++k)
                acc += gp[k] * w[(((size_t)k * d->R + r) * d->S + s) * d->C + c];
        }
    }
    return acc;
}

/* dw[k,r,s,c] = sum_{n,ho,wo} dy[n,ho,wo,k] * x[n, ho*sh - ph + r*dh, wo*sw - pw + s*dw, c],
 * out-of-image reads are zero. */
static double wgrad_element(const oracle_conv_desc *d, const double *x, const double *dy,
                            int Ho, int Wo, int k, int r, int s, int c)
{
    double acc = 0.0;
    for (int n = 0; n < d->N; ++n) {
        for (int ho = 0; ho < Ho; ++ho) {
            int h = ho * d->stride_h - d->pad_h + r * d->dil_h;
            if (h < 0 || h >= d->H) continue;
            for (int wo = 0; wo < Wo; ++wo) {
                int wi = wo * d->stride_w - d->pad_w + s * d->dil_w;
                if (wi < 0 || wi >= d->W) continue;
                acc += dy[(((size_t)n * Ho + ho) * Wo + wo) * d->K + k] *
                       x[(((size_t)n * d->H + h) * d->W + wi) * d->C + c];
            }
        }
    }
    return acc;
}

/* ---- whole tensors and sampled elements ----------------------------------------- */
/* `idx == NULL`: compute every output element, out has the full output size.
 * `idx != NULL`: compute only the `nidx` flat output indices listed, out[i] <-> idx[i]. */

static size_t numel_x(const oracle_conv_desc *d) { return (size_t)d->N * d->H * d->W * d->C; }
static size_t numel_w(const oracle_conv_desc *d) { return (size_t)d->K * d->R * d->S * d->C; }

/* The three passes on widened (fp64) copies of the inputs; x, w, dy are freed here. */
static int fwd_widened(const oracle_conv_desc *d, double *x, double *w, const int64_t *idx, int64_t nidx,
                       double *out)
{
    int32_t Ho, Wo;
    if (oracle_conv2d_out_shape(d, &Ho, &Wo)) { free(x); free(w); return -1; }
    if (!x || !w) { free(x); free(w); return -2; }
    int64_t total = (int64_t)d->N * Ho * Wo * d->K;
    int64_t count = idx ? nidx : total;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) {
        int64_t f = idx ? idx[i] : i;
        int k = (int)(f % d->K);
        int64_t t = f / d->K;
        int wo = (int)(t % Wo); t /= Wo;
        int ho = (int)(t % Ho);
        int n = (int)(t / Ho);
        out[i] = fwd_element(d, x, w, n, ho, wo, k);
    }
    free(x); free(w);
    return 0;
}

int oracle_conv2d_fwd(const oracle_conv_desc *d, const uint16_t *x16, const uint16_t *w16,
                      const int64_t *idx, int64_t nidx, double *out)
{
    int32_t Ho, Wo;
    if (oracle_conv2d_out_shape(d, &Ho, &Wo) || !x16 || !w16 || !out) return -1;
    return fwd_widened(d, widen(x16, numel_x(d)), widen(w16, numel_w(d)), idx, nidx, out);
}

int oracle_conv2d_fwd_f32(const oracle_conv_desc *d, const float *x32, const float *w32,
                          const int64_t *idx, int64_t nidx, double *out)
{
    int32_t Ho, Wo;
    if (oracle_conv2d_out_shape(d, &Ho, &Wo) || !x32 || !w32 || !out) return -1;
    return fwd_widened(d, widen_f32(x32, numel_x(d)), widen_f32(w32, numel_w(d)), idx, nidx, out);
}

static int dgrad_widened(const oracle_conv_desc *d, double *dy, double *w, const int64_t *idx, int64_t nidx,
                         double *out)
{
    int32_t Ho, Wo;
    if (oracle_conv2d_out_shape(d, &Ho, &Wo)) { free(dy); free(w); return -1; }
    if (!dy || !w) { free(dy); free(w); return -2; }
    int64_t total = (int64_t)numel_x(d);
    int64_t count = idx ? nidx : total;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) {
        int64_t f = idx ? idx[i] : i;
        int c = (int)(f % d->C);
        int64_t t = f / d->C;
        int wi = (int)(t % d->W); t /= d->W;
        int h = (int)(t % d->H);
        int n = (int)(t / d->H);
        out[i] = dgrad_element(d, dy, w, Ho, Wo, n, h, wi, c);
    }
    free(dy); free(w);
    return 0;
}

int oracle_conv2d_dgrad(const oracle_conv_desc *d, const uint16_t *dy16, const uint16_t *w16,
                        const int64_t *idx, int64_t nidx, double *out)
{
    int32_t Ho, Wo;
    if (oracle_conv2d_out_shape(d, &Ho, &Wo) || !dy16 || !w16 || !out) return -1;
    return dgrad_widened(d, widen(dy16, (size_t)d->N * Ho * Wo * d->K), widen(w16, numel_w(d)), idx, nidx, out);
}

int oracle_conv2d_dgrad_f32(const oracle_conv_desc *d, const float *dy32, const float *w32,
                            const int64_t *idx, int64_t nidx, double *out)
{
    int32_t Ho, Wo;
    if (oracle_conv2d_out_shape(d, &Ho, &Wo) || !dy32 || !w32 || !out) return -1;
    return dgrad_widened(d, widen_f32(dy32, (size_t)d->N * Ho * Wo * d->K), widen_f32(w32, numel_w(d)), idx, nidx,
                         out);
}

static int wgrad_widened(const oracle_conv_desc *d, double *x, double *dy, const int64_t *idx, int64_t nidx,
                         double *out)
{
    int32_t Ho, Wo;
    if (oracle_conv2d_out_shape(d, &Ho, &Wo)) { free(x); free(dy); return -1; }
    if (!x || !dy) { free(x); free(dy); return -2; }
    int64_t total = (int64_t)numel_w(d);
    int64_t count = idx ? nidx : total;
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t i = 0; i < count; ++i) {
        int64_t f = idx ? idx[i] : i;
        int c = (int)(f % d->C);
        int64_t t = f / d->C;
        int s = (int)(t % d->S); t /= d->S;
        int r = (int)(t % d->R);
        int k = (int)(t / d->R);
        out[i] = wgrad_element(d, x, dy, Ho, Wo, k, r, s, c);
    }
    free(x); free(dy);
    return 0;
}

int oracle_conv2d_wgrad(const oracle_conv_desc *d, const uint16_t *x16, const uint16_t *dy16,
                        const int64_t *idx, int64_t nidx, double *out)
{
    int32_t Ho, Wo;
    if (oracle_conv2d_out_shape(d, &Ho, &Wo) || !x16 || !dy16 || !out) return -1;
    return wgrad_widened(d, widen(x16, numel_x(d)), widen(dy16, (size_t)d->N * Ho * Wo * d->K), idx, nidx, out);
}

int oracle_conv2d_wgrad_f32(const oracle_conv_desc *d, const float *x32, const float *dy32,
                            const int64_t *idx, int64_t nidx, double *out)
{
    int32_t Ho, Wo;
    if (oracle_conv2d_out_shape(d, &Ho, &Wo) || !x32 || !dy32 || !out) return -1;
    return wgrad_widened(d, widen_f32(x32, numel_x(d)), widen_f32(dy32, (size_t)d->N * Ho * Wo * d->K), idx, nidx,
                         out);
}

/* ---- loss-scale removal and overflow detection ---------------------------------- */
/* out[i] = fp32(g[i] * inv_scale). The fp64 product of two fp32 values is exact, so the
 * single rounding to fp32 is the correctly rounded fp32 product. The flag looks at the
 * values that come in: 1 if any of them is +inf, -inf or NaN, else 0. */
int oracle_unscale_check(const float *g, int64_t n, float inv_scale, float *out, int32_t *flag)
{
    if (n < 0 || !flag || (n > 0 && (!g || !out))) return -1;
    int32_t bad = 0;
    for (int64_t i = 0; i < n; ++i) {
        if (!isfinite(g[i])) bad = 1;
        out[i] = (float)((double)g[i] * (double)inv_scale);
    }
    *flag = bad;
    return 0;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
