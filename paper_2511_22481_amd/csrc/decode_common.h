// Device helpers shared by the gfx950 decode kernels (bf16 cache and fp8 cache).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"

namespace omniattn {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

#define LDS_PTR(T, byte_off) ((__attribute__((address_space(3))) T*)(uintptr_t)(byte_off))

__device__ __forceinline__ bool retained(int j, int L, int S, int W) {
  return j < L && (j < S || j >= L - W);
}

// Direct global->LDS load of 16 bytes per lane: lane l's bytes land at LDS address
// M0 + IMM + 16 l and are read from base + off + IMM (base wave-uniform, off per lane;
// the instruction's immediate offset applies to both sides).  Written as assembly so
// that the compiler does not treat it as a store that may alias every later LDS read
// and drain the whole prefetch before the first read of another stage; completion is
// awaited explicitly (wait_vm) before the barrier that publishes the tile.
// M0 carries the LDS base.  Nothing else in these kernels uses M0 (no indirect register
// addressing, no GWS, no compiler-issued LDS-DMA), so it is simply overwritten.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void dma_set_lds_base(uint32_t lds_base) {
  const uint32_t slds = __builtin_amdgcn_readfirstlane(lds_base);
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0" : : "s"(slds) : "m0");
}
template <int IMM>
__device__ __forceinline__ void dma16(const uint8_t* base, uint32_t off) {
  // wave-uniform by construction; make that visible to the register allocator
  const uint64_t b = (uint64_t)(uintptr_t)base;
  const uint32_t b_lo = __builtin_amdgcn_readfirstlane((uint32_t)b);
  const uint32_t b_hi = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32));
  const uint64_t sbase = ((uint64_t)b_hi << 32) | b_lo;
  // nt: cache rows are read once per work unit; marking them as streaming keeps them from
  // pushing Q (shared by the units of a sequence) and the partial results out of the caches
  asm volatile("global_load_lds_dwordx4 %0, %1 offset:%2 nt" : : "v"(off), "s"(sbase), "n"(IMM) : "m0");
}
// 4 bytes per lane: lane l's dword lands at M0 + 4 l.
__device__ __forceinline__ void dma4(const uint8_t* base, uint32_t off) {
  const uint64_t b = (uint64_t)(uintptr_t)base;
  const uint32_t b_lo = __builtin_amdgcn_readfirstlane((uint32_t)b);
  const uint32_t b_hi = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32));
  const uint64_t sbase = ((uint64_t)b_hi << 32) | b_lo;
  asm volatile("global_load_lds_dword %0, %1" : : "v"(off), "s"(sbase) : "m0");
}
#pragma clang diagnostic pop
// Wait until at most N of this wave's vector-memory operations are outstanding.
template <int N>
__device__ __forceinline__ void wait_vm() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// The XCD (accelerator complex die) this wave runs on: compute units of one XCD share an L2.
__device__ __forceinline__ uint32_t xcc_id() {
  uint32_t id;
  asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(id));
  return id & 15u;
}

}  // namespace omniattn
