// MFMA-only loop: what the matrix pipes sustain on this device when nothing else limits them.
// The benchmark reports it next to the spec-sheet peak, because the clock under sustained matrix
// load is lower than the peak engine clock the spec figure assumes.
#include "common.h"

namespace sdconv {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));

// 8 waves per workgroup (two per SIMD), 8 independent accumulators per wave, `iters` rounds of
// 16 v_mfma_f32_32x32x16_f16 each.
__global__ __launch_bounds__(512) void mfma_ceiling_kernel(float* out, int iters)
{
    const int lane = threadIdx.x & 63;
    float16v acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
    half8 a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        a[e] = (_Float16)(0.001f * (float)(lane + e));
        b[e] = (_Float16)(0.002f * (float)(lane ^ e));
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc[i], 0, 0, 0);
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(b, a, acc[i], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) s += acc[i][e];
    out[(size_t)blockIdx.x * 512 + threadIdx.x] = s;
}

hipError_t launch_mfma_ceiling(float* out, int blocks, int iters, hipStream_t st)
{
    hipLaunchKernelGGL(mfma_ceiling_kernel, dim3((unsigned)blocks), dim3(512), 0, st, out, iters);
    return hipGetLastError();
}

}  // namespace sdconv
