/*
 * sdconv_bench.h -- measurement aids of libsdconv.  Not part of the convolution path: bench.py
 * uses them to report what the device sustains and what a fused epilogue replaces.  Same
 * conventions as sdconv.h (device pointers, asynchronous on the caller's HIP stream, return codes).
 */
#ifndef SDCONV_BENCH_H
#define SDCONV_BENCH_H

#include "sdconv.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Measurement aid, not part of the convolution path: launches `blocks` workgroups of 8 waves
 * that each issue iters * 16 v_mfma_f32_32x32x16_f16 on registers only (32768 FLOP per
 * instruction and wave), i.e. blocks * 8 * iters * 16 * 32768 FLOP in total.  Timed by the
 * caller, it gives the fp16 matrix rate the device sustains (the clock under matrix load is
 * below the spec-sheet clock).  scratch: device buffer of at least blocks * 512 floats,
 * overwritten.  Asynchronous on hip_stream.  SDCONV_EINVAL for a null buffer or non-positive
 * counts. */
int sdconv_mfma_ceiling(float *scratch, int blocks, int iters, void *hip_stream);

/* Measurement aid: the elementwise tail of conv2d_fwd_fused / conv2d_dgrad_fused as a separate
 * in-place pass over t, a binary16 [pixels][channels] tensor (what runs after a convolution
 * when the tail is not fused; it reads and writes the whole activation once more, and rounds
 * to binary16 twice where the fused calls round once):
 *   v = t[p][c]; v *= scale[c]; v += bias[c]; v += residual[p][c]; relu: v = max(v, 0);
 *   relu_mask: v = relu_mask[p][c] > 0 ? v : 0;  t[p][c] = binary16(v)
 * with binary32 arithmetic; NULL pointers / relu == 0 leave a step out.  All pointers are
 * device pointers, 16-byte aligned; channels must be a multiple of 8.  Asynchronous on
 * hip_stream.  SDCONV_EINVAL for a null t, bad sizes or misalignment. */
int sdconv_tail_pass(void *t, size_t pixels, int32_t channels, const float *scale, const float *bias,
                     const void *residual, const void *relu_mask, int32_t relu, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* SDCONV_BENCH_H */
