// Matrix-core and asynchronous-copy primitives shared by the product kernels (gfx950).
#ifndef NM_MMA_H
#define NM_MMA_H

#include "nm_device.h"

namespace nm {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) __bf16 bf16x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((ext_vector_type(8))) uint32_t u32x8_t;

// Asynchronous 16-byte (4-byte) per lane global -> LDS copy: lane i's piece lands at lds + 16*i (4*i).
// `base` is wave-uniform (scalar registers), the lane adds an unsigned 32-bit byte offset; M0 carries
// the LDS byte address and needs one wait state before the load that reads it.
typedef uint64_t uniform_ptr_t;
__device__ __forceinline__ uniform_ptr_t make_uniform(const void* p) {
  const uint64_t v = (uint64_t)(uintptr_t)p;
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return ((uint64_t)hi << 32) | lo;
}
__device__ __forceinline__ void dma16(uniform_ptr_t base, uint32_t lane_byte_offset, uint32_t lds) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds), "v"(lane_byte_offset),
               "s"(base)
               : "memory", "m0");
}
__device__ __forceinline__ void dma4(uniform_ptr_t base, uint32_t lane_byte_offset, uint32_t lds) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2" ::"s"(lds), "v"(lane_byte_offset),
               "s"(base)
               : "memory", "m0");
}
// The same with the LDS address given as two uniform terms (stage buffer + place inside the stage).
__device__ __forceinline__ void dma16_at(uniform_ptr_t base, uint32_t lane_byte_offset, uint32_t lds_stage,
                                         uint32_t lds_offset) {
  asm volatile("s_add_u32 m0, %0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3" ::"s"(lds_stage), "s"(lds_offset),
               "v"(lane_byte_offset), "s"(base)
               : "memory", "m0", "scc");
}
__device__ __forceinline__ void dma4_at(uniform_ptr_t base, uint32_t lane_byte_offset, uint32_t lds_stage,
                                        uint32_t lds_offset) {
  asm volatile("s_add_u32 m0, %0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %2, %3" ::"s"(lds_stage), "s"(lds_offset),
               "v"(lane_byte_offset), "s"(base)
               : "memory", "m0", "scc");
}
// Two floats to a pair of bfloat16 (round to nearest even) with the hardware conversion; lo in bits 0..15.
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  typedef __bf16 hwbf16x2_t __attribute__((ext_vector_type(2)));
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{lo, hi}, hwbf16x2_t));
}

// The asynchronous copies are not tracked by the compiler; a kernel counts its own and waits until at most N
// of the wave's vector memory operations are outstanding (they complete in issue order).
template <int N>
__device__ __forceinline__ void wait_loads_outstanding() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

}  // namespace nm

#endif  // NM_MMA_H
