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
typedef int i32x4_t __attribute__((ext_vector_type(4)));
typedef int i32x8_t __attribute__((ext_vector_type(8)));

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

// Write-out of a wave's accumulator tile of (TT * 16) rows x (OT * 16) columns of a row-major output.
// The matrix instructions leave a lane (r16 = lane % 16, kb = lane / 16) with, for every 16 x 16 block (i, j),
// the four consecutive columns i * 16 + kb * 4 .. + 3 of row j * 16 + r16: get(i, j) returns them as four
// 32-bit patterns (floats, or integers).  ES = 4 stores the patterns, ES = 2 rounds floats to bfloat16.
//
// Aligned outputs (every row start and end on a 16-byte boundary): 16 rows at a time go through the wave's own
// LDS slice (wave_tile_slice_bytes, rows padded by 16 bytes against bank conflicts), so that the global stores
// are 16 bytes per lane and whole row segments of the wave tile are written contiguously.
template <int OT, int ES>
constexpr int wave_tile_slice_bytes() { return 16 * (OT * 16 * ES + 16); }

template <int OT, int TT, int ES, typename Get>
__device__ __forceinline__ void write_wave_tile_pieces(unsigned char* slice, int lane, Get get, void* Y, int64_t ldy,
                                                       int64_t row0, int64_t col0, int64_t n_rows, int64_t n_cols) {
  constexpr int OW = OT * 16;
  constexpr int RS = OW * ES + 16;   // padded LDS row
  constexpr int CPR = OW * ES / 16;  // 16-byte pieces per row
  constexpr int PASSES = (16 * CPR + 63) / 64;
  const int r16 = lane & 15, kb = lane >> 4;
#pragma unroll
  for (int j = 0; j < TT; ++j) {
#pragma unroll
    for (int i = 0; i < OT; ++i) {
      const u32x4_t v = get(i, j);
      unsigned char* dst = slice + r16 * RS + (i * 16 + kb * 4) * ES;
      if constexpr (ES == 2) {
        uint2 pk;
        pk.x = pack_bf16x2(__uint_as_float(v[0]), __uint_as_float(v[1]));
        pk.y = pack_bf16x2(__uint_as_float(v[2]), __uint_as_float(v[3]));
        *reinterpret_cast<uint2*>(dst) = pk;
      } else {
        *reinterpret_cast<u32x4_t*>(dst) = v;
      }
    }
#pragma unroll
    for (int pss = 0; pss < PASSES; ++pss) {
      const int q = pss * 64 + lane;
      const int row = q / CPR, ch = q % CPR;
      if (16 * CPR % 64 == 0 || row < 16) {
        const u32x4_t piece = *reinterpret_cast<const u32x4_t*>(slice + row * RS + ch * 16);
        const int64_t r = row0 + j * 16 + row;
        const int64_t c = col0 + ch * (16 / ES);
        if (r < n_rows && c < n_cols)
          *reinterpret_cast<u32x4_t*>(reinterpret_cast<unsigned char*>(Y) + (r * ldy + c) * ES) = piece;
      }
    }
  }
}

// Any alignment: element by element.
template <int OT, int TT, typename Get>
__device__ __forceinline__ void write_wave_tile_elements(int lane, Get get, void* Y, int64_t ldy, int64_t row0, int64_t col0,
                                                         int64_t n_rows, int64_t n_cols, bool to_bf16) {
  const int r16 = lane & 15, kb = lane >> 4;
#pragma unroll
  for (int j = 0; j < TT; ++j) {
    const int64_t r = row0 + j * 16 + r16;
    if (r >= n_rows) continue;
#pragma unroll
    for (int i = 0; i < OT; ++i) {
      const int64_t c = col0 + i * 16 + kb * 4;
      const u32x4_t v = get(i, j);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        if (c + e >= n_cols) break;
        if (to_bf16) reinterpret_cast<bf16_t*>(Y)[r * ldy + c + e] = (bf16_t)f32_to_bf16_rne(__uint_as_float(v[e]));
        else reinterpret_cast<uint32_t*>(Y)[r * ldy + c + e] = v[e];
      }
    }
  }
}

// The asynchronous copies are not tracked by the compiler; a kernel counts its own and waits until at most N
// of the wave's vector memory operations are outstanding (they complete in issue order).
template <int N>
__device__ __forceinline__ void wait_loads_outstanding() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

}  // namespace nm

#endif  // NM_MMA_H
