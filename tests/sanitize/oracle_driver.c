/*
 * Runs the CPU oracle (oracle/oracle_conv.c, compiled into this program with
 * -fsanitize=address,undefined) over small cases that reach every branch of it: padding on all
 * sides, stride larger than the filter, dilation, sampled and whole outputs, binary16 subnormals
 * and signed zeros, the binary32 entry points, empty and non-finite gradient buffers, invalid
 * descriptors.  Any report of the sanitizers ends the program with a non-zero status; the results
 * are written to the file named on the command line so that the caller can compare them with the
 * ordinary build of the oracle.  Test infrastructure only.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t N, H, W, C;
    int32_t K, R, S;
    int32_t stride_h, stride_w, pad_h, pad_w, dil_h, dil_w;
} oracle_conv_desc;

int oracle_conv2d_out_shape(const oracle_conv_desc *, int32_t *, int32_t *);
int oracle_conv2d_fwd(const oracle_conv_desc *, const uint16_t *, const uint16_t *, const int64_t *, int64_t, double *);
int oracle_conv2d_dgrad(const oracle_conv_desc *, const uint16_t *, const uint16_t *, const int64_t *, int64_t, double *);
int oracle_conv2d_wgrad(const oracle_conv_desc *, const uint16_t *, const uint16_t *, const int64_t *, int64_t, double *);
int oracle_conv2d_fwd_f32(const oracle_conv_desc *, const float *, const float *, const int64_t *, int64_t, double *);
int oracle_conv2d_dgrad_f32(const oracle_conv_desc *, const float *, const float *, const int64_t *, int64_t, double *);
int oracle_conv2d_wgrad_f32(const oracle_conv_desc *, const float *, const float *, const int64_t *, int64_t, double *);
int oracle_unscale_check(const float *, int64_t, float, float *, int32_t *);

static uint64_t lcg_state;
static uint64_t lcg(void)
{
    lcg_state = lcg_state * 6364136223846793005ull + 1442695040888963407ull;
    return lcg_state;
}
/* any finite binary16 pattern: zeros of both signs, subnormals, normals up to 65504 */
static uint16_t next_half(void)
{
    uint16_t b = (uint16_t)(lcg() >> 40);
    if ((b & 0x7c00) == 0x7c00) b ^= 0x4000;
    return b;
}
/* small finite floats k / 8, k in -512 .. 511 */
static float next_float(void) { return (float)((int)((lcg() >> 40) & 1023) - 512) / 8.0f; }

static FILE *out;
static void dump(const double *v, int64_t n) { fwrite(v, sizeof(double), (size_t)n, out); }

static const oracle_conv_desc kCases[] = {
    {1, 5, 6, 3, 4, 3, 3, 1, 1, 1, 1, 1, 1},
    {2, 7, 5, 4, 2, 3, 2, 2, 2, 1, 0, 1, 1},
    {1, 6, 6, 2, 3, 1, 1, 3, 3, 0, 0, 1, 1},   /* stride > filter: dx positions without a tap */
    {1, 9, 8, 2, 2, 3, 3, 1, 2, 2, 2, 2, 2},   /* dilation 2, pad 2 */
    {2, 4, 4, 5, 1, 2, 2, 1, 1, 0, 1, 1, 1},
    {1, 1, 1, 1, 1, 1, 1, 1, 1, 0, 0, 1, 1},
};

static int run_case(const oracle_conv_desc *d, int ci)
{
    int32_t Ho, Wo;
    if (oracle_conv2d_out_shape(d, &Ho, &Wo)) return 1;
    int64_t nx = (int64_t)d->N * d->H * d->W * d->C, ny = (int64_t)d->N * Ho * Wo * d->K,
            nw = (int64_t)d->K * d->R * d->S * d->C;
    uint16_t *x = malloc(nx * 2), *w = malloc(nw * 2), *g = malloc(ny * 2);
    float *xf = malloc(nx * 4), *wf = malloc(nw * 4), *gf = malloc(ny * 4);
    lcg_state = 1000 + ci;
    for (int64_t i = 0; i < nx; ++i) { x[i] = next_half(); xf[i] = next_float(); }
    for (int64_t i = 0; i < nw; ++i) { w[i] = next_half(); wf[i] = next_float(); }
    for (int64_t i = 0; i < ny; ++i) { g[i] = next_half(); gf[i] = next_float(); }
    double *oy = malloc(ny * 8), *ox = malloc(nx * 8), *ow = malloc(nw * 8);
    int rc = 0;
    rc |= oracle_conv2d_fwd(d, x, w, NULL, 0, oy); dump(oy, ny);
    rc |= oracle_conv2d_dgrad(d, g, w, NULL, 0, ox); dump(ox, nx);
    rc |= oracle_conv2d_wgrad(d, x, g, NULL, 0, ow); dump(ow, nw);
    rc |= oracle_conv2d_fwd_f32(d, xf, wf, NULL, 0, oy); dump(oy, ny);
    rc |= oracle_conv2d_dgrad_f32(d, gf, wf, NULL, 0, ox); dump(ox, nx);
    rc |= oracle_conv2d_wgrad_f32(d, xf, gf, NULL, 0, ow); dump(ow, nw);
    /* sampled outputs: first, last and one in the middle, in this (unsorted) order */
    int64_t iy[3] = {ny - 1, 0, ny / 2}, ix[3] = {nx - 1, 0, nx / 2}, iw[3] = {nw - 1, 0, nw / 2};
    double s[3];
    rc |= oracle_conv2d_fwd(d, x, w, iy, 3, s); dump(s, 3);
    rc |= oracle_conv2d_dgrad(d, g, w, ix, 3, s); dump(s, 3);
    rc |= oracle_conv2d_wgrad(d, x, g, iw, 3, s); dump(s, 3);
    rc |= oracle_conv2d_fwd(d, x, w, iy, 0, s);          /* an empty sample list */
    free(x); free(w); free(g); free(xf); free(wf); free(gf); free(oy); free(ox); free(ow);
    return rc;
}

int main(int argc, char **argv)
{
    if (argc < 2) return 2;
    out = fopen(argv[1], "wb");
    if (!out) return 2;
    int rc = 0;
    for (size_t c = 0; c < sizeof(kCases) / sizeof(kCases[0]); ++c) rc |= run_case(&kCases[c], (int)c);

    /* invalid descriptors are refused, nothing is touched */
    oracle_conv_desc bad = kCases[0];
    int32_t ho, wo;
    bad.H = 2; bad.pad_h = 0; bad.R = 5;
    if (oracle_conv2d_out_shape(&bad, &ho, &wo) == 0) rc |= 4;
    bad = kCases[0]; bad.stride_w = 0;
    if (oracle_conv2d_fwd(&bad, NULL, NULL, NULL, 0, NULL) == 0) rc |= 4;
    if (oracle_conv2d_out_shape(NULL, &ho, &wo) == 0) rc |= 4;

    /* loss-scale removal: empty buffer, one element, a buffer with every class of value */
    int32_t flag = -1;
    rc |= oracle_unscale_check(NULL, 0, 0.5f, NULL, &flag);
    if (flag != 0) rc |= 8;
    float one = 3.0f, res;
    rc |= oracle_unscale_check(&one, 1, 0.25f, &res, &flag);
    if (res != 0.75f || flag != 0) rc |= 8;
    enum { NG = 1000 };
    float *gbuf = malloc(NG * 4), *gout = malloc(NG * 4);
    lcg_state = 77;
    for (int i = 0; i < NG; ++i) gbuf[i] = next_float() * 1e30f;      /* some overflow to inf when scaled up */
    uint32_t inf_bits = 0x7f800000u, nan_bits = 0x7fc00001u, den_bits = 0x00000003u;
    memcpy(&gbuf[10], &den_bits, 4);
    rc |= oracle_unscale_check(gbuf, NG, 1.0f / 1024.0f, gout, &flag);
    if (flag != 0) rc |= 8;
    memcpy(&gbuf[NG - 1], &inf_bits, 4);
    rc |= oracle_unscale_check(gbuf, NG, 1.0f / 1024.0f, gout, &flag);
    if (flag != 1) rc |= 8;
    memcpy(&gbuf[NG - 1], &nan_bits, 4);
    rc |= oracle_unscale_check(gbuf, NG, 1.0f / 1024.0f, gout, &flag);
    if (flag != 1) rc |= 8;
    if (oracle_unscale_check(gbuf, -1, 1.0f, gout, &flag) == 0) rc |= 8;
    free(gbuf); free(gout);
    fclose(out);
    printf("oracle_driver status %d\n", rc);
    return rc;
}
