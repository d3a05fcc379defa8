// Global -> LDS DMA and wait-count helpers shared by the MFMA kernels (gfx950).
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

namespace dwm {

// One 64-lane DMA: an active lane i's 16 bytes at g land at LDS byte address m0 + 16*i.
// Issued through inline assembly on purpose: the compiler's own bookkeeping would wait for
// ALL outstanding loads before any LDS read, which serialises a multi-stage ring; callers
// wait with wait_vmcnt<N>() and a barrier instead.
__device__ __forceinline__ void dma16(const float* g, uint32_t lds_byte_addr_uniform)
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :
                 : "v"(g), "s"(lds_byte_addr_uniform)
                 : "memory");
}

// The same DMA with the address split into a wave-uniform base (a scalar register pair) and
// the lane's unsigned 32-bit byte offset: stepping the base costs no vector instruction.
__device__ __forceinline__ void dma16s(const float* base_uniform, uint32_t lane_byte_offset,
                                       uint32_t lds_byte_addr_uniform)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(lane_byte_offset), "s"(base_uniform), "s"(lds_byte_addr_uniform)
                 : "memory");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

}  // namespace dwm
