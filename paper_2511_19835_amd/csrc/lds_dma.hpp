// Direct-to-LDS loads and the explicit waits that go with them (gfx950).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rsa {

// Direct-to-LDS loads (global_load_lds_dwordx4): every lane supplies the address of 16
// bytes; lane L's data lands at lds_addr + 16*L, lds_addr wave-uniform (goes to M0). The
// compiler does not track these loads: the caller waits with s_waitcnt vmcnt before the
// barrier that publishes the buffer, and `fence` names the LDS buffer so that it counts as
// written. Two address forms: scalar base + per-lane 32-bit byte offset, and per-lane pointer.
__device__ __forceinline__ void dma16_sv(uint32_t lds_addr, const void* sbase, uint32_t voff, void* fence) {
  // the base is wave-uniform by construction; make sure it sits in an SGPR pair
  const uint64_t p = (uint64_t)(uintptr_t)sbase;
  // (the builtin returns a signed int: widen through uint32_t, or the low word sign-extends)
  const uint32_t p_lo = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)p);
  const uint32_t p_hi = (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(p >> 32));
  const uint64_t ps = ((uint64_t)p_hi << 32) | (uint64_t)p_lo;
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2"
               ::"s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(voff), "s"(ps), "r"(fence) : "memory");
}
// The same with the LDS address given as a wave-uniform base plus a wave-uniform offset, added straight
// into M0: one scalar instruction and the load, whatever the offset.
__device__ __forceinline__ void dma16_sv_at(uint32_t lds_base, uint32_t lds_off, uint64_t sbase, uint32_t voff, void* fence) {
  asm volatile("s_add_u32 m0, %0, %1\n\tglobal_load_lds_dwordx4 %2, %3"
               ::"s"(lds_base), "s"(lds_off), "v"(voff), "s"(sbase), "r"(fence) : "memory", "scc");
}
// ... and with the offset as a literal of the instruction (no register held for it).
template <uint32_t LDS_OFF>
__device__ __forceinline__ void dma16_sv_imm(uint32_t lds_base, uint64_t sbase, uint32_t voff, void* fence) {
  asm volatile("s_add_u32 m0, %0, %1\n\tglobal_load_lds_dwordx4 %2, %3"
               ::"s"(lds_base), "n"(LDS_OFF), "v"(voff), "s"(sbase), "r"(fence) : "memory", "scc");
}
__device__ __forceinline__ void dma16_v(uint32_t lds_addr, const void* gptr, void* fence) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off"
               ::"s"(__builtin_amdgcn_readfirstlane(lds_addr)), "v"(gptr), "r"(fence) : "memory");
}

template <int NLEFT>
__device__ __forceinline__ void wait_loads_leaving() {
  // vmcnt(NLEFT): bits 3:0 and 15:14 hold the count, exp/lgkm fields stay at "no wait"
  __builtin_amdgcn_s_waitcnt(0x0F70 | (NLEFT & 15) | ((NLEFT >> 4) << 14));
}

}  // namespace rsa
