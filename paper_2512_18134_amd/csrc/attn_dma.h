// attn_dma.h -- direct global -> LDS loads (LDS-DMA) and the vector-memory wait, shared by the forward and
// backward kernels (gfx950 only).
//
// A wave-wide global_load_lds writes its 64 lanes' data to LDS linearly from the address in m0.  The load
// needs one wait state after the scalar write of m0 (there is no hardware interlock); m0 is reserved by
// the compiler and cannot be named as a clobber, so each statement saves and restores it.
#pragma once
#include <stdint.h>

#include <hip/hip_runtime.h>

namespace attn {

// 16 bytes per lane: LDS address = lds_addr + lane*16
__device__ __forceinline__ void dma16(uint32_t lds_addr, const void *base, uint32_t voff)
{
    uint32_t m0_saved;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3\n\ts_mov_b32 m0, %0"
                 : "=&s"(m0_saved)
                 : "s"(lds_addr), "v"(voff), "s"(base)
                 : "memory");
}

// 4 bytes per lane: LDS address = lds_addr + lane*4
__device__ __forceinline__ void dma4(uint32_t lds_addr, const void *base, uint32_t voff)
{
    uint32_t m0_saved;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %2, %3\n\ts_mov_b32 m0, %0"
                 : "=&s"(m0_saved)
                 : "s"(lds_addr), "v"(voff), "s"(base)
                 : "memory");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

}  // namespace attn
