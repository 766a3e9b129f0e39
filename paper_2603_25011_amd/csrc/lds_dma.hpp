// Direct global -> LDS loads (LDS-DMA) and the wait that goes with them, shared by the forward kernel and
// the LDS-tile dW kernel.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lsr {

// 16 bytes per lane from global memory straight into LDS: lane l of the wave lands at
// lds_base + 16 l (lds_base is wave-uniform and travels in M0).  Written as inline assembly on
// purpose: when the compiler sees its own LDS-DMA builtin it stops using partial lgkmcnt waits for
// every later LDS read, which serialises the fragment prefetch.  Completion is tracked by hand with
// vmcnt (wait_vmcnt below) before the workgroup barrier that publishes the data.
__device__ __forceinline__ void dma16_to_lds(const void* gptr, uint32_t lds_base) {
    // (an SALU write of M0 needs one wait state before an LDS-DMA instruction reads it)
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :
                 : "v"(gptr), "s"(lds_base)
                 : "memory", "m0");
}
// Same, 4 bytes per lane: lane l lands at lds_base + 4 l.
__device__ __forceinline__ void dma4_to_lds(const void* gptr, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off"
                 :
                 : "v"(gptr), "s"(lds_base)
                 : "memory", "m0");
}
// The 16-byte load addressed as wave-uniform base (an SGPR pair) + 32-bit byte offset per lane:
// no 64-bit address arithmetic per load, and half the address registers.
__device__ __forceinline__ void dma16_to_lds(const void* sbase, uint32_t voff, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(voff), "s"(sbase), "s"(lds_base)
                 : "memory", "m0");
}
__device__ __forceinline__ uint32_t lds_addr(const void* p) {
    return static_cast<uint32_t>(reinterpret_cast<uintptr_t>(p));   // LDS aperture: low 32 bits are the offset
}

// s_waitcnt vmcnt(n) with the other counters left alone (gfx9 encoding of simm16).
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

}  // namespace lsr
