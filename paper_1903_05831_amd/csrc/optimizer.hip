// Optimizer tail of a mixed-precision step, on flat fp32 buffers, consuming the device-side
// overflow flag of the loss-scale check without a host round trip:
//   - SGD with momentum and weight decay on fp32 master weights,
//       mom <- mu*mom - lr*(g + wd*w);  w <- w + mom        (skipped when the flag is set)
//     every operation a separate binary32 operation (no fused multiply-add), then
//       w16 <- binary16(w), round to nearest even           (always written);
//   - one transition of the dynamic loss-scale state machine (one thread):
//       flag set: scale *= backoff, good_steps = 0;
//       else:     ++good_steps, and at `interval`: scale *= growth, good_steps = 0.
// HBM-bound: 12 bytes read + 10 written per element (4 + 2 when the step is skipped).
#include "common.h"

namespace sdconv {

struct LossScaleState { float scale; int32_t good_steps; };

constexpr int kSgdThreads = 256;
constexpr int kSgdVecPerThread = 2;

typedef float float4s __attribute__((ext_vector_type(4)));
typedef _Float16 half4s __attribute__((ext_vector_type(4)));

// The compiler's default for device code is to contract a*b + c into one fused operation, and
// the *_rn helpers are plain operators to it: this file is compiled with -ffp-contract=off
// (see build.py) so that every operation below rounds on its own.
__device__ __forceinline__ void sgd_one(float& w, float& m, float g, float lr, float mu, float wd)
{
    const float t = __fmul_rn(wd, w);
    const float gg = __fadd_rn(g, t);
    const float a = __fmul_rn(mu, m);
    const float b = __fmul_rn(lr, gg);
    m = __fsub_rn(a, b);
    w = __fadd_rn(w, m);
}

__global__ __launch_bounds__(kSgdThreads) void sgd_momentum_kernel(
    float* __restrict__ w, float* __restrict__ mom, const float* __restrict__ g, _Float16* __restrict__ w16,
    size_t n, size_t nvec, float lr, float mu, float wd, const int32_t* __restrict__ flag,
    LossScaleState* __restrict__ state, float growth, float backoff, int32_t interval)
{
    const bool skip = *flag != 0;
    float4s* w4 = reinterpret_cast<float4s*>(w);
    float4s* m4 = reinterpret_cast<float4s*>(mom);
    const float4s* g4 = reinterpret_cast<const float4s*>(g);
    half4s* h4 = reinterpret_cast<half4s*>(w16);
    const size_t base = (size_t)blockIdx.x * (kSgdThreads * kSgdVecPerThread) + threadIdx.x;
#pragma unroll
    for (int j = 0; j < kSgdVecPerThread; ++j) {
        const size_t i = base + (size_t)j * kSgdThreads;
        if (i >= nvec) continue;
        float4s wv = __builtin_nontemporal_load(w4 + i);
        if (!skip) {
            float4s mv = __builtin_nontemporal_load(m4 + i);
            const float4s gv = __builtin_nontemporal_load(g4 + i);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float we = wv[e], me = mv[e];
                sgd_one(we, me, gv[e], lr, mu, wd);
                wv[e] = we;
                mv[e] = me;
            }
            __builtin_nontemporal_store(wv, w4 + i);
            __builtin_nontemporal_store(mv, m4 + i);
        }
        half4s hv;
        hv.x = (_Float16)wv.x; hv.y = (_Float16)wv.y; hv.z = (_Float16)wv.z; hv.w = (_Float16)wv.w;
        __builtin_nontemporal_store(hv, h4 + i);
    }
    if (blockIdx.x == 0) {
        // ragged tail (< 4 elements), then the state machine
        const size_t t = nvec * 4 + threadIdx.x;
        if (t < n) {
            float wv = w[t];
            if (!skip) {
                float mv = mom[t];
                sgd_one(wv, mv, g[t], lr, mu, wd);
                w[t] = wv;
                mom[t] = mv;
            }
            w16[t] = (_Float16)wv;
        }
        if (threadIdx.x == 0) {
            LossScaleState s = *state;
            if (skip) {
                s.scale = __fmul_rn(s.scale, backoff);
                s.good_steps = 0;
            } else if (++s.good_steps >= interval) {
                s.scale = __fmul_rn(s.scale, growth);
                s.good_steps = 0;
            }
            *state = s;
        }
    }
}

hipError_t launch_sgd_momentum(float* w, float* mom, const float* g, void* w16, size_t n, float lr, float mu,
                               float wd, const int32_t* flag, void* state, float growth, float backoff,
                               int32_t interval, hipStream_t st)
{
    const size_t nvec = n / 4;
    const size_t per_block = (size_t)kSgdThreads * kSgdVecPerThread;
    size_t blocks = (nvec + per_block - 1) / per_block;
    if (blocks == 0) blocks = 1;
    hipLaunchKernelGGL(sgd_momentum_kernel, dim3((unsigned)blocks), dim3(kSgdThreads), 0, st, w, mom, g,
                       static_cast<_Float16*>(w16), n, nvec, lr, mu, wd, flag,
                       static_cast<LossScaleState*>(state), growth, backoff, interval);
    return hipGetLastError();
}

}  // namespace sdconv
