// LDS-DMA primitives shared by the pipelined kernels: buffer loads that land in LDS without
// passing through registers, issued from inline assembly so that the kernel, not the
// compiler, decides how many of them stay in flight.
#pragma once
#include <hip/hip_runtime.h>

namespace sdconv {

typedef int int4v __attribute__((ext_vector_type(4)));

constexpr unsigned kOutOfRange = 0x80000000u;   // byte offset no tensor here reaches

// Raw buffer descriptor over `bytes` bytes at `p` (stride 0, range-checked on the offset).
__device__ __forceinline__ int4v make_rsrc(const void* p, unsigned bytes)
{
    unsigned long long a = reinterpret_cast<unsigned long long>(p);
    int4v r;
    // readfirstlane pins the words to scalar registers: the descriptor is an "s" operand of
    // the load and the compiler may otherwise keep a copy in vector registers under pressure
    r.x = __builtin_amdgcn_readfirstlane((int)(unsigned)a);
    r.y = __builtin_amdgcn_readfirstlane((int)((a >> 32) & 0xffffu));
    r.z = __builtin_amdgcn_readfirstlane((int)bytes);
    r.w = 0x00020000;
    return r;
}

// 16 bytes per lane from buffer offset voff + soff to LDS address lds_base + lane*16
// (rsrc, soff, lds_base wave-uniform).  A voff at or past the descriptor's size yields zeros
// in LDS and touches no memory.
__device__ __forceinline__ void dma16(unsigned voff, int4v rsrc, unsigned soff, unsigned lds_base)
{
    asm volatile("s_mov_b32 m0, %3\n\ts_nop 0\n\tbuffer_load_dwordx4 %0, %1, %2 offen lds"
                 :: "v"(voff), "s"(rsrc), "s"(soff), "s"(lds_base) : "memory");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

}  // namespace sdconv
