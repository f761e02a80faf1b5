// Direct global -> LDS transfers (global_load_lds_dwordx4) for gfx950.
// Each lane moves 16 bytes; the 64 lanes of a wave fill 1 KiB of consecutive LDS starting at the
// wave-uniform LDS address.  The transfers are written as inline assembly so that the compiler does
// not order later LDS reads behind them with a full vmcnt(0) wait (it cannot tell ring stages
// apart); kernels that use them wait for the transfers themselves ("s_waitcnt vmcnt(n)" counts the
// transfers still allowed in flight) before the barrier that publishes a stage.
#pragma once
#include <stdint.h>

// Per-lane 64-bit global address.
__device__ __forceinline__ void dma16(const void* gptr, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(gptr) : "memory", "m0");
}
// Wave-uniform 64-bit base (SGPR pair) plus a per-lane 32-bit byte offset.
__device__ __forceinline__ void dma16_base(const void* sbase, uint32_t voff, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(voff), "s"(sbase) : "memory", "m0");
}
// 4 bytes per lane: a wave fills 256 consecutive bytes of LDS.
__device__ __forceinline__ void dma4_base(const void* sbase, uint32_t voff, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2" ::"s"(lds_addr), "v"(voff), "s"(sbase) : "memory", "m0");
}
template <int N>
__device__ __forceinline__ void dma_wait() {  // at most N transfers of this wave still in flight
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
__device__ __forceinline__ uint32_t lds_address(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) void*)p;
}
