// pex_lds_dma.h -- device helpers shared by the kernels that fill their LDS with direct-to-LDS buffer loads and
// track completion by hand (gfx950).  Device code only; every function is inlined into its caller.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pex {
namespace {

typedef __attribute__((ext_vector_type(4))) int int4_t;
typedef __attribute__((address_space(3))) void* lds_void;

// One direct-to-LDS load: every lane fetches 16 bytes at (descriptor base + voff) and the wave's 1 KiB lands at
// LDS byte address lds_addr + lane*16; lanes whose offset is outside the descriptor's range write zeros.
// Issued as inline assembly so that the compiler does not serialise it against the LDS reads that follow
// (it cannot tell that they touch a different slab of the ring); completion is tracked by hand with vmcnt.
__device__ __forceinline__ void dma_load_16(uint32_t lds_addr, uint32_t voff, int4_t rsrc)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(rsrc)
                 : "memory", "m0");
}

__device__ __forceinline__ int4_t make_rsrc(const void* base, uint32_t num_records)
{
    const uint64_t a = (uint64_t)base;
    int4_t r;
    r[0] = (int)(uint32_t)a;
    r[1] = (int)((uint32_t)(a >> 32) & 0xffffu);     // stride 0, no swizzle
    r[2] = (int)num_records;
    r[3] = 0x00020000;                               // raw buffer, 32-bit data format
    return r;
}

// s_waitcnt vmcnt(N) only.  Written as assembly: the compiler does not know about the direct-to-LDS loads and
// would be free to move or drop a wait it sees no use for.
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// this wave's LDS reads and writes are complete, then the workgroup barrier
__device__ __forceinline__ void wait_lds_and_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }
__device__ __forceinline__ void plain_barrier() { asm volatile("s_barrier" ::: "memory"); }

}  // namespace
}  // namespace pex
