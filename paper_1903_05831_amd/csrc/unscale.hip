// Loss-scale removal with overflow detection over a flat fp32 gradient buffer.
// HBM-bound: 4 bytes read + 4 bytes written per element, nothing else.
//   grad[i] <- grad[i] * inv_scale   (one fp32 multiply, no contraction partner)
//   flag    <- any input with all-ones exponent (+-inf, NaN)
// Every element is written even when the flag trips.  Each wave reduces its lanes'
// findings with a ballot; only blocks that saw a non-finite value touch the shared record.
#include "common.h"
#include <atomic>
#include <mutex>

namespace sdconv {

constexpr int kUnscaleThreads = 256;
constexpr int kUnscaleVecPerThread = 4;   // float4 loads in flight per thread

__device__ __forceinline__ unsigned nonfinite_bits(float v)
{
    return ((__float_as_uint(v) & 0x7f800000u) == 0x7f800000u) ? 1u : 0u;
}

// One launch does it all, the flag included.  The flag may hold anything when the call starts,
// and blocks run in no particular order, so no block can clear it for the others: instead every
// block adds one 64-bit word to a small record of the library's own (a slot of a zero-initialised
// device array, handed out round-robin by the host so that calls that overlap in time use
// different ones): 1 in the low half ("I am done") and its finding in the high half.  The block
// whose addition completes the count writes the flag, 0 or 1, and returns the slot to zero.
// Finding and count travel in one atomic, so no fence is needed (a device-scope release costs a
// write-back of the L2 on this chip: with one per block the kernel ran at 0.7 TB/s).  Thousands of
// atomics on one address would serialise as well: the blocks count in 64 sub-counters by block
// number, and a sub-counter that is complete adds its total to the top counter.
constexpr int kUnscaleSub = 64;
struct UnscaleSlot { unsigned long long top; unsigned long long sub[kUnscaleSub]; };
constexpr int kUnscaleSlots = 1024;
static __device__ UnscaleSlot unscale_slots[kUnscaleSlots];
constexpr unsigned long long kBadUnit = 1ull << 32;

// scale_on_device: nullptr, or the current loss scale in device memory: inv_scale is then
// 1/scale, one correctly rounded binary32 division.
__global__ __launch_bounds__(kUnscaleThreads) void unscale_check_kernel(
    float* __restrict__ grad, size_t n, size_t head, size_t nvec, float inv_scale,
    const float* __restrict__ scale_on_device, int32_t* __restrict__ flag, UnscaleSlot* __restrict__ slot)
{
    typedef float float4v __attribute__((ext_vector_type(4)));
    if (scale_on_device) inv_scale = __fdiv_rn(1.0f, *scale_on_device);
    unsigned bad = 0;
    float4v* body = reinterpret_cast<float4v*>(grad + head);
    constexpr size_t kPerBlock = (size_t)kUnscaleThreads * kUnscaleVecPerThread;
    // one chunk of kPerBlock vectors per block
    {
        const size_t base = (size_t)blockIdx.x * kPerBlock + threadIdx.x;
        float4v v[kUnscaleVecPerThread];
#pragma unroll
        for (int j = 0; j < kUnscaleVecPerThread; ++j) {
            size_t i = base + (size_t)j * kUnscaleThreads;
            if (i < nvec) v[j] = __builtin_nontemporal_load(body + i);
        }
#pragma unroll
        for (int j = 0; j < kUnscaleVecPerThread; ++j) {
            size_t i = base + (size_t)j * kUnscaleThreads;
            if (i < nvec) {
                bad |= nonfinite_bits(v[j].x) | nonfinite_bits(v[j].y) | nonfinite_bits(v[j].z) |
                       nonfinite_bits(v[j].w);
                float4v o;
                o.x = __fmul_rn(v[j].x, inv_scale);
                o.y = __fmul_rn(v[j].y, inv_scale);
                o.z = __fmul_rn(v[j].z, inv_scale);
                o.w = __fmul_rn(v[j].w, inv_scale);
                __builtin_nontemporal_store(o, body + i);
            }
        }
    }
    // Unaligned head (< 4 elements) and ragged tail (< 4 elements): block 0, first lanes.
    if (blockIdx.x == 0) {
        size_t tail_start = head + nvec * 4;
        size_t ntail = n - tail_start;
        size_t t = threadIdx.x;
        if (t < head) {
            float g = grad[t];
            bad |= nonfinite_bits(g);
            grad[t] = __fmul_rn(g, inv_scale);
        } else if (t >= 8 && t - 8 < ntail) {
            float g = grad[tail_start + (t - 8)];
            bad |= nonfinite_bits(g);
            grad[tail_start + (t - 8)] = __fmul_rn(g, inv_scale);
        }
    }
    // block-wide OR of the findings, one atomic per block that saw something, then the count
    __shared__ unsigned block_bad;
    if (threadIdx.x == 0) block_bad = 0;
    __syncthreads();
    const unsigned long long any = __ballot(bad != 0);
    if (any != 0ull && (threadIdx.x & 63) == 0) atomicOr(&block_bad, 1u);
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned s = blockIdx.x % kUnscaleSub;
        const unsigned long long members = (gridDim.x - s + kUnscaleSub - 1) / kUnscaleSub;   // blocks that count in sub[s]
        const unsigned long long mine = 1ull + (block_bad ? kBadUnit : 0ull);
        const unsigned long long sum = atomicAdd(&slot->sub[s], mine) + mine;
        if ((sum & 0xffffffffull) == members) {         // this block completes its sub-counter
            atomicExch(&slot->sub[s], 0ull);
            const unsigned long long groups = gridDim.x < kUnscaleSub ? gridDim.x : kUnscaleSub;
            const unsigned long long up = 1ull + ((sum >> 32) ? kBadUnit : 0ull);
            const unsigned long long total = atomicAdd(&slot->top, up) + up;
            if ((total & 0xffffffffull) == groups) {    // ... and the whole call: it is the last one
                atomicExch(&slot->top, 0ull);
                *flag = (total >> 32) ? 1 : 0;
            }
        }
    }
}

static std::mutex g_slot_mu;
static UnscaleSlot* g_slot_base[64];                  // device address of unscale_slots, per device
static std::atomic<unsigned> g_next_slot{0};

hipError_t launch_unscale_check(float* grad, size_t n, float inv_scale, const float* scale_on_device,
                                int32_t* flag, hipStream_t st)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    UnscaleSlot* base;
    {
        std::lock_guard<std::mutex> lock(g_slot_mu);
        if (!g_slot_base[dev]) {
            void* p = nullptr;
            e = hipGetSymbolAddress(&p, HIP_SYMBOL(unscale_slots));
            if (e != hipSuccess) return e;
            g_slot_base[dev] = static_cast<UnscaleSlot*>(p);
        }
        base = g_slot_base[dev];
    }
    UnscaleSlot* slot = base + (g_next_slot.fetch_add(1u) % kUnscaleSlots);
    size_t mis = (reinterpret_cast<uintptr_t>(grad) >> 2) & 3u;     // floats past a 16-byte line
    size_t head = n ? (mis ? (4 - mis) : 0) : 0;
    if (head > n) head = n;
    size_t nvec = (n - head) / 4;
    size_t per_block = (size_t)kUnscaleThreads * kUnscaleVecPerThread;
    size_t chunks = (nvec + per_block - 1) / per_block;
    size_t blocks = chunks ? chunks : 1;
    hipLaunchKernelGGL(unscale_check_kernel, dim3((unsigned)blocks), dim3(kUnscaleThreads), 0, st,
                       grad, n, head, nvec, inv_scale, scale_on_device, flag, slot);
    return hipGetLastError();
}

}  // namespace sdconv
