// Direct global -> LDS loads (global_load_lds) and the bookkeeping they need.
//
// The data of these loads never pass through registers, so a wave can keep many tiles in flight without
// spending VGPRs on staging.  The instructions are written as inline assembly: the compiler knows nothing
// about them, places no waits for them and (more important) cannot be trusted to place FEWER waits than a
// pipelined loop needs -- its own handling of this instruction waits for all of them before the next LDS
// read.  A kernel that uses them counts them itself (wait_vm before the barrier that publishes a tile) and
// must not issue compiler-visible vector memory loads inside its main loop: a compiler-placed wait for such a
// load would also wait for every tile in flight.  Loads issued before the loop are "consumed" by an empty asm
// statement so that their wait lands before the loop.
#pragma once
#include <type_traits>
#include <utility>
#include "common.h"

namespace dkv {

// Both loads write M0 (the LDS base of the instruction) and say so in their clobber lists: the compiler reserves M0
// and sets it itself right before each of its own uses, but its passes that move or merge M0 initialisations look
// for definitions in between, and an asm statement is one only if it is declared (the compiler's warning about
// reserved registers in clobber lists is switched off for this library).
// 64 lanes x 16 bytes: global address = sbase + voff (per lane), LDS address = lds_addr + 16 * lane.
__device__ __forceinline__ void dma16(const void* sbase, uint32_t voff, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(lds_addr), "v"(voff), "s"(sbase)
               : "memory", "m0");
}
// 64 lanes x 4 bytes: global address = sbase + voff (per lane), LDS address = lds_addr + 4 * lane.
__device__ __forceinline__ void dma4(const void* sbase, uint32_t voff, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
               :
               : "s"(lds_addr), "v"(voff), "s"(sbase)
               : "memory", "m0");
}
// The same with the LDS address given as a wave-uniform base plus a compile-time offset, added into M0 inside the
// statement.  In a loop unrolled over LDS stages every load has a different constant address; given as one value,
// the compiler computes all of them ahead of the loop, runs out of scalar registers and reloads each from a spill
// slot (a vector-register lane read per load) instead of re-adding a constant.
template <int OFF>
__device__ __forceinline__ void dma16_at(const void* sbase, uint32_t voff, uint32_t lds_base) {
  asm volatile("s_add_u32 m0, %0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :
               : "s"(lds_base), "v"(voff), "s"(sbase), "n"(OFF)
               : "memory", "m0", "scc");
}
template <int OFF>
__device__ __forceinline__ void dma4_at(const void* sbase, uint32_t voff, uint32_t lds_base) {
  asm volatile("s_add_u32 m0, %0, %3\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
               :
               : "s"(lds_base), "v"(voff), "s"(sbase), "n"(OFF)
               : "memory", "m0", "scc");
}
// f(std::integral_constant<int, 0>{}), ..., f(std::integral_constant<int, N - 1>{}): a loop whose index is a constant expression
template <typename F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(f, std::make_integer_sequence<int, N>{});
}
template <int N>
__device__ __forceinline__ void wait_vm() {
  asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

__device__ __forceinline__ const u16* uniform_ptr(const u16* ptr) {
  const uint64_t v = reinterpret_cast<uint64_t>(ptr);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return reinterpret_cast<const u16*>(((uint64_t)hi << 32) | lo);
}

}  // namespace dkv
