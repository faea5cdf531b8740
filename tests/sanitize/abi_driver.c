/*
 * Drives the host side of libsdconv's C ABI (argument validation, output shapes, workspace
 * queries, kernel selection) through valid, extreme and invalid arguments.  It is linked against
 * a build of the library whose ABI layer (api.hip, dispatch.hip, static_scratch.hip) was compiled
 * with -fsanitize=address,undefined on the host side; no call here reaches a GPU: every compute
 * call is made with arguments that must be refused before anything is enqueued.  A sanitizer
 * report or a wrong status ends the program with a non-zero status.  Test infrastructure only.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>
#include "sdconv.h"
#include "sdconv_bench.h"

static int failures;
#define EXPECT(cond) do { if (!(cond)) { ++failures; printf("line %d: %s\n", __LINE__, #cond); } } while (0)

static conv2d_desc base(void)
{
    conv2d_desc d = {1, 8, 8, 8, 8, 3, 3, 1, 1, 1, 1, 1, 1};
    return d;
}

int main(void)
{
    int32_t ho, wo;
    void *ok = (void *)(uintptr_t)0x10000, *odd = (void *)(uintptr_t)0x10004;   /* never dereferenced */
    long swept = 0;

    /* a sweep of descriptors: shapes, workspace sizes and kernel names are host-only */
    static const int Ns[] = {1, 2, 512}, HW[] = {1, 7, 14, 50, 200, 4096}, CK[] = {1, 3, 8, 60, 64, 256, 2048},
                     Rs[] = {1, 3, 7}, St[] = {1, 2, 3, 5}, Pd[] = {0, 1, 3}, Dl[] = {1, 2};
    for (unsigned a = 0; a < 3; ++a) for (unsigned b = 0; b < 6; ++b) for (unsigned c = 0; c < 7; ++c)
    for (unsigned e = 0; e < 7; ++e) for (unsigned f = 0; f < 3; ++f) for (unsigned g = 0; g < 4; ++g)
    for (unsigned h = 0; h < 3; ++h) for (unsigned i = 0; i < 2; ++i) {
        conv2d_desc d = {Ns[a], HW[b], HW[(b + 1) % 6], CK[c], CK[e], Rs[f], Rs[(f + 1) % 3], St[g], St[(g + 1) % 4],
                         Pd[h], Pd[(h + 1) % 3], Dl[i], Dl[(i + 1) % 2]};
        int rc = conv2d_out_shape(&d, &ho, &wo);
        EXPECT(rc == SDCONV_OK || rc == SDCONV_EINVAL);
        for (int pass = 0; pass < 3; ++pass) {
            size_t ws = conv2d_workspace_bytes(&d, pass), ws32 = conv2d_workspace_bytes_f32(&d, pass);
            const char *name = sdconv_kernel_name(&d, pass);
            EXPECT(name && strlen(name) > 0);
            if (rc != SDCONV_OK) EXPECT(ws == 0 && ws32 == 0 && strcmp(name, "invalid") == 0);
            else EXPECT(ws % 256 == 0 && strcmp(name, "invalid") != 0);
        }
        ++swept;
    }
    EXPECT(conv2d_workspace_bytes(NULL, 0) == 0 && conv2d_workspace_bytes_f32(NULL, 0) == 0);
    conv2d_desc d = base();
    EXPECT(conv2d_workspace_bytes(&d, 7) == 0 && strcmp(sdconv_kernel_name(&d, -1), "invalid") == 0);
    EXPECT(conv2d_out_shape(&d, NULL, &wo) == SDCONV_EINVAL && conv2d_out_shape(NULL, &ho, &wo) == SDCONV_EINVAL);

    /* extreme and invalid field values */
    const int32_t extremes[] = {INT32_MIN, -1, 0, INT32_MAX};
    for (unsigned field = 0; field < 13; ++field)
        for (unsigned v = 0; v < 4; ++v) {
            d = base();
            ((int32_t *)&d)[field] = extremes[v];
            int rc = conv2d_out_shape(&d, &ho, &wo);
            EXPECT(rc == SDCONV_OK || rc == SDCONV_EINVAL);
            if (rc == SDCONV_EINVAL) {
                EXPECT(conv2d_fwd(&d, ok, ok, ok, NULL, 0, NULL) == SDCONV_EINVAL);
                EXPECT(conv2d_dgrad(&d, ok, ok, ok, NULL, 0, NULL) == SDCONV_EINVAL);
                EXPECT(conv2d_wgrad(&d, ok, ok, (float *)ok, NULL, 0, NULL) == SDCONV_EINVAL);
                EXPECT(conv2d_wgrad_static_scratch(&d, ok, ok, (float *)ok, NULL) == SDCONV_EINVAL);
                EXPECT(conv2d_fwd_f32(&d, (float *)ok, (float *)ok, (float *)ok, NULL, 0, NULL) == SDCONV_EINVAL);
            }
            (void)conv2d_workspace_bytes(&d, SDCONV_WGRAD);
            (void)sdconv_kernel_name(&d, SDCONV_DGRAD);
        }
    conv2d_desc big = {70000, 256, 256, 64, 8, 1, 1, 1, 1, 0, 0, 1, 1};          /* 2^31 elements and more */
    EXPECT(conv2d_out_shape(&big, &ho, &wo) == SDCONV_EINVAL);

    /* pointers: null, misaligned; workspace: missing, too small, misaligned */
    d = base();
    EXPECT(conv2d_fwd(&d, NULL, ok, ok, NULL, 0, NULL) == SDCONV_EINVAL);
    EXPECT(conv2d_fwd(&d, ok, odd, ok, NULL, 0, NULL) == SDCONV_EINVAL);
    EXPECT(conv2d_dgrad(&d, ok, ok, NULL, NULL, 0, NULL) == SDCONV_EINVAL);
    EXPECT(conv2d_wgrad(&d, ok, ok, NULL, NULL, 0, NULL) == SDCONV_EINVAL);
    conv2d_desc r4 = {2, 50, 84, 256, 256, 3, 3, 1, 1, 1, 1, 1, 1};
    size_t need = conv2d_workspace_bytes(&r4, SDCONV_WGRAD);
    EXPECT(need > 0);
    EXPECT(conv2d_wgrad(&r4, ok, ok, (float *)ok, NULL, 0, NULL) == SDCONV_EWORKSPACE);
    EXPECT(conv2d_wgrad(&r4, ok, ok, (float *)ok, ok, need - 1, NULL) == SDCONV_EWORKSPACE);
    EXPECT(conv2d_wgrad(&r4, ok, ok, (float *)ok, (void *)(uintptr_t)0x10010, need, NULL) == SDCONV_EINVAL);
    conv2d_desc huge = {8, 56, 56, 1024, 1024, 3, 3, 1, 1, 1, 1, 1, 1};
    EXPECT(conv2d_workspace_bytes(&huge, SDCONV_WGRAD) > SDCONV_STATIC_SCRATCH_BYTES);
    EXPECT(conv2d_wgrad_static_scratch(&huge, ok, ok, (float *)ok, NULL) == SDCONV_EWORKSPACE);
    EXPECT(conv2d_fwd_fused(&d, ok, ok, NULL, ok, NULL, 0, NULL) == SDCONV_EINVAL);
    conv2d_fwd_epilogue fe = {(const float *)odd, NULL, NULL, 1};
    EXPECT(conv2d_fwd_fused(&d, ok, ok, &fe, ok, NULL, 0, NULL) == SDCONV_EINVAL);
    conv2d_dgrad_epilogue de = {NULL, odd};
    EXPECT(conv2d_dgrad_fused(&d, ok, ok, &de, ok, NULL, 0, NULL) == SDCONV_EINVAL);
    EXPECT(conv2d_dgrad_f32(&r4, (float *)ok, (float *)ok, (float *)ok, NULL, 0, NULL) == SDCONV_EWORKSPACE);

    /* loss-scale removal and optimizer arguments */
    EXPECT(grad_unscale_check((float *)ok, 8, 1.0f, NULL, NULL) == SDCONV_EINVAL);
    EXPECT(grad_unscale_check(NULL, 8, 1.0f, (int32_t *)ok, NULL) == SDCONV_EINVAL);
    EXPECT(grad_unscale_check((float *)ok, 8, 0.0f, (int32_t *)ok, NULL) == SDCONV_EINVAL);
    EXPECT(grad_unscale_check((float *)ok, 8, -1.0f, (int32_t *)ok, NULL) == SDCONV_EINVAL);
    EXPECT(grad_unscale_check((float *)ok, 8, NAN, (int32_t *)ok, NULL) == SDCONV_EINVAL);
    EXPECT(grad_unscale_check((float *)ok, 8, INFINITY, (int32_t *)ok, NULL) == SDCONV_EINVAL);
    EXPECT(grad_unscale_check((float *)(uintptr_t)0x10001, 8, 1.0f, (int32_t *)ok, NULL) == SDCONV_EINVAL);
    EXPECT(grad_unscale_check((float *)ok, (size_t)1 << 41, 1.0f, (int32_t *)ok, NULL) == SDCONV_EINVAL);
    EXPECT(grad_unscale_check_dynamic((float *)ok, 8, NULL, (int32_t *)ok, NULL) == SDCONV_EINVAL);
    loss_scale_state *st = (loss_scale_state *)ok;
    EXPECT(sgd_momentum_update(NULL, (float *)ok, (float *)ok, ok, 8, 0.1f, 0.9f, 0.f, (int32_t *)ok, st, 2.f, .5f, 10, NULL) == SDCONV_EINVAL);
    EXPECT(sgd_momentum_update((float *)ok, (float *)ok, (float *)ok, ok, 8, NAN, 0.9f, 0.f, (int32_t *)ok, st, 2.f, .5f, 10, NULL) == SDCONV_EINVAL);
    EXPECT(sgd_momentum_update((float *)ok, (float *)ok, (float *)ok, ok, 8, 0.1f, 0.9f, 0.f, (int32_t *)ok, st, 0.f, .5f, 10, NULL) == SDCONV_EINVAL);
    EXPECT(sgd_momentum_update((float *)ok, (float *)ok, (float *)ok, ok, 8, 0.1f, 0.9f, 0.f, (int32_t *)ok, st, 2.f, .5f, 0, NULL) == SDCONV_EINVAL);
    EXPECT(sgd_momentum_update((float *)ok, (float *)odd, (float *)ok, ok, 8, 0.1f, 0.9f, 0.f, (int32_t *)ok, st, 2.f, .5f, 10, NULL) == SDCONV_EINVAL);
    EXPECT(sdconv_tail_pass(NULL, 8, 8, NULL, NULL, NULL, NULL, 0, NULL) == SDCONV_EINVAL);
    EXPECT(sdconv_tail_pass(ok, 8, 7, NULL, NULL, NULL, NULL, 0, NULL) == SDCONV_EINVAL);
    EXPECT(sdconv_mfma_ceiling(NULL, 1, 1, NULL) == SDCONV_EINVAL);
    for (int s = -6; s <= 1; ++s) EXPECT(strlen(sdconv_status_string(s)) > 0);
    EXPECT(sdconv_last_hip_error() == 0);

    printf("abi_driver: %ld descriptors swept, %d failures\n", swept, failures);
    return failures ? 1 : 0;
}
