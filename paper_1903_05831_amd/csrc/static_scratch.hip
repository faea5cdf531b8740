// conv2d_wgrad for callers that cannot allocate device memory (code under HIP graph capture,
// tight serving loops, harnesses that forbid hipMalloc): the scratch that conv2d_wgrad takes
// from its workspace argument (split-K partial sums, padded copies, stem partials) lives in a
// file-scope device array of fixed size instead.
//
// The array's name is a host-side stand-in, not a device address: the device address is asked
// for once per device with hipGetSymbolAddress and kept; every kernel gets that address.
#include "common.h"
#include <mutex>

namespace sdconv {

constexpr size_t kStaticScratchBytes = (size_t)SDCONV_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

static std::mutex g_scratch_mu;
static void* g_scratch_ptr[kMaxDevices];    // device address of `scratch` on each device, once known

// Address of this device's copy of the array (every device holds its own copy at its own
// address).  The first call on a device asks the runtime; later calls only read the table.
static hipError_t static_scratch(void** out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

int wgrad_static_scratch(const Geom& g, const Plan& p, const __half* x, const __half* dy, float* dw, hipStream_t st,
                         hipError_t* hip_error)
{
    *hip_error = hipSuccess;
    if (p.workspace_bytes > kStaticScratchBytes) return SDCONV_EWORKSPACE;
    void* ws = nullptr;
    if (p.workspace_bytes) {
        *hip_error = static_scratch(&ws);
        if (*hip_error != hipSuccess) return SDCONV_EHIP;
    }
    // every route overwrites the part of the scratch it reads (partial sums, padded copies):
    // nothing has to start at zero, whatever the call before left there
    *hip_error = run_wgrad(g, p, x, dy, dw, ws, st);
    return *hip_error == hipSuccess ? SDCONV_OK : SDCONV_EHIP;
}

}  // namespace sdconv
