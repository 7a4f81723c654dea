// Helpers shared by the bf16 grouped GEMM kernels (gfx950): direct global->LDS loads, 16-byte global accesses.
#pragma once
#include <type_traits>

#include "common.h"
#include "gemm_tiles.h"

namespace modse_gemm {

__device__ const uint4 g_zero_chunk[4] = {};
  // source of K-tail chunks that lie beyond K

// tells the compiler that a pointer is the same in every lane (keeps it in scalar registers)
__device__ __forceinline__ const void* uniform_ptr(const void* p) {
  const uint64_t v = reinterpret_cast<uint64_t>(p);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return reinterpret_cast<const void*>(((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ int uniform_int(int v) { return __builtin_amdgcn_readfirstlane(v); }
// 16 bytes per lane from global memory straight into LDS at lds_base + 16 * lane (lds_base wave-uniform).
__device__ __forceinline__ void dma_b128(const void* gptr, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(
                   __builtin_amdgcn_readfirstlane(lds_base)),
               "v"(gptr)
               : "memory");
}
// same, address = wave-uniform base + per-lane unsigned 32-bit byte offset.  STREAM marks data that is read once
// (the non-temporal hint): a plain read stream of 1.9 GB runs at 6.3 TB/s on this chip, a hinted one at 7.2 TB/s.
template <bool STREAM = false>
__device__ __forceinline__ void dma_b128_s(const void* base, uint32_t voff, uint32_t lds_base) {
  if constexpr (STREAM)
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt" ::"s"(
                     __builtin_amdgcn_readfirstlane(lds_base)),
                 "v"(voff), "s"(uniform_ptr(base))
                 : "memory");
  else
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(
                     __builtin_amdgcn_readfirstlane(lds_base)),
                 "v"(voff), "s"(uniform_ptr(base))
                 : "memory");
}
// 16-byte accesses through the global address space (a generic pointer would make them flat accesses)
typedef __attribute__((address_space(1))) bf16x8 global_bf16x8;
__device__ __forceinline__ void global_store16(bf16_t* p, bf16x8 v) { *(global_bf16x8*)(uintptr_t)p = v; }
__device__ __forceinline__ bf16x8 global_load16(const bf16_t* p) { return *(const global_bf16x8*)(uintptr_t)p; }
// 16 bytes per lane to / from wave-uniform base + per-lane unsigned 32-bit byte offset.  (The two wait states
// behind a store: a store of more than 64 bits must not be followed at once by a VALU write of its data
// registers, and the compiler's hazard handling does not look inside assembly.)  The load is issued
// from assembly so that its wait can be written by hand: the compiler waits for every outstanding memory
// operation as soon as loads and stores are mixed.  wait_loaded makes the values usable once at most
// `younger` vector-memory loads issued after them are still in flight (loads complete in order).
__device__ __forceinline__ void global_store16_s(const void* base, uint32_t voff, bf16x8 v) {
  asm volatile("global_store_dwordx4 %0, %1, %2\n\ts_nop 1" ::"v"(voff), "v"(v), "s"(base) : "memory");
}
__device__ __forceinline__ void global_store16_s(const void* base, uint32_t voff, f32x4 v) {
  asm volatile("global_store_dwordx4 %0, %1, %2\n\ts_nop 1" ::"v"(voff), "v"(v), "s"(base) : "memory");
}
__device__ __forceinline__ bf16x8 global_load16_s(const void* base, uint32_t voff) {
  bf16x8 v;
  asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(v) : "v"(voff), "s"(base) : "memory");
  return v;
}
template <int YOUNGER>
__device__ __forceinline__ void wait_loaded(bf16x8& a, bf16x8& b) {
  static_assert(YOUNGER >= 0 && YOUNGER < 16, "vmcnt field");
  asm volatile("s_waitcnt vmcnt(%2)" : "+v"(a), "+v"(b) : "n"(YOUNGER) : "memory");
}
__device__ __forceinline__ uint32_t lds_address(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)p;
}

// logistic function with the hardware reciprocal (1 ulp) instead of an IEEE division: the results are
// rounded to bf16 anyway
__device__ __forceinline__ float sigmoid_fast(float a) { return __builtin_amdgcn_rcpf(1.f + __expf(-a)); }

}  // namespace modse_gemm
