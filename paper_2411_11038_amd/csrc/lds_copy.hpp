// Global -> LDS copies issued as inline assembly, and the vector types of the MFMA fragments, shared by the product
// kernels whose instruction order is pinned by hand.
#pragma once
#include "common.hpp"

namespace efqat {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef short shortx4_t __attribute__((ext_vector_type(4)));
typedef int intx2_t __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) void* lds_ptr_t;

// One wave-wide global -> LDS copy: lane l moves 16 bytes from its own src to lds_dst + 16 l.  Written as inline
// assembly on purpose: the compiler models the LDS transpose-read builtins as possible LDS writes and would make
// every one of them wait for all copies in flight (s_waitcnt vmcnt(0)), which serialises the pipeline.  The
// kernel orders copies against reads itself (s_waitcnt vmcnt(0) + barrier once per stage).  M0 holds the LDS
// destination; nothing else in this kernel uses M0, and volatile statements keep their order, so the copy always
// sees the M0 value written just before it (s_nop: one wait state between an M0 write and its use).
__device__ __forceinline__ void dma16(const char* src, char* lds_dst) {
  const uint32_t m = (uint32_t)(uintptr_t)(lds_ptr_t)lds_dst;
  asm volatile("s_mov_b32 m0, %0" ::"s"(m) : "m0");
  asm volatile("s_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src));
}

// one wave-wide global -> LDS copy of 4 bytes per lane (the 64 scales of a stage)
__device__ __forceinline__ void dma4(const char* src, char* lds_dst) {
  const uint32_t m = (uint32_t)(uintptr_t)(lds_ptr_t)lds_dst;
  asm volatile("s_mov_b32 m0, %0" ::"s"(m) : "m0");
  asm volatile("s_nop 0\n\tglobal_load_lds_dword %0, off" ::"v"(src));
}

}  // namespace efqat
