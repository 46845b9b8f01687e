// Shared device-side helpers for the N:M kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace nm {

typedef uint16_t bf16_t;  // bfloat16 bit pattern

__host__ __device__ constexpr int log2_of(int m) { return m == 4 ? 2 : (m == 8 ? 3 : (m == 16 ? 4 : 0)); }

__host__ __device__ inline int64_t values_per_row(int64_t K, int N, int M) { return K / M * N; }
__host__ __device__ inline int64_t index_words_per_row(int64_t K, int N, int M) {
  return (values_per_row(K, N, M) * log2_of(M) + 31) / 32;
}
__host__ __device__ inline int64_t mask_words_per_row(int64_t K) { return (K + 31) / 32; }

// Saliency of Eq. (1) with rho = |w|: the bf16 pattern without its sign bit orders like |w|.
__device__ __forceinline__ uint32_t saliency_key(uint32_t bits) { return bits & 0x7FFFu; }

__device__ __forceinline__ float bf16_to_f32(uint32_t bits) { return __uint_as_float(bits << 16); }

// fp32 -> bf16, round to nearest, ties to even; NaN stays NaN.
__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x40u;
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// `nbits` (<= 32) bits of a row's LSB-first bit stream starting at bit `off`; `nwords` words in the row.
__device__ __forceinline__ uint32_t stream_bits(const uint32_t* __restrict__ row, int64_t nwords, int64_t off,
                                                int nbits) {
  const int64_t w = off >> 5;
  const int s = (int)(off & 31);
  uint64_t lo = row[w];
  if (s + nbits > 32 && w + 1 < nwords) lo |= (uint64_t)row[w + 1] << 32;
  uint32_t r = (uint32_t)(lo >> s);
  return nbits >= 32 ? r : (r & ((1u << nbits) - 1u));
}

// Keep mask (bit i = member i kept) of one group by magnitude: order by (key descending, position
// ascending), keep the first N.  rank_i = number of members that precede member i in that order.
template <int N, int M>
__device__ __forceinline__ uint32_t select_top_n(const uint32_t (&key)[M]) {
  if (N >= M) return (1u << M) - 1u;
  uint32_t rank[M];
#pragma unroll
  for (int i = 0; i < M; ++i) rank[i] = 0;
#pragma unroll
  for (int i = 0; i < M; ++i) {
#pragma unroll
    for (int j = i + 1; j < M; ++j) {
      const bool i_first = key[i] >= key[j];  // equal scores: the lower position goes first
      rank[j] += i_first ? 1u : 0u;
      rank[i] += i_first ? 0u : 1u;
    }
  }
  uint32_t keep = 0;
#pragma unroll
  for (int i = 0; i < M; ++i) keep |= (rank[i] < (uint32_t)N ? 1u : 0u) << i;
  return keep;
}

// Runtime-level form of the same rule (general kernels).
__device__ inline uint32_t select_top_n_rt(const uint32_t* key, int N, int M) {
  uint32_t keep = 0;
  for (int i = 0; i < M; ++i) {
    int rank = 0;
    for (int j = 0; j < M; ++j) rank += (key[j] > key[i]) || (key[j] == key[i] && j < i);
    keep |= (rank < N ? 1u : 0u) << i;
  }
  return keep;
}

// A caller's mask made usable: the N lowest set positions; if fewer are set, the lowest unset
// positions complete the group (`filled` marks those: they are stored with value +0).
__device__ __forceinline__ uint32_t legalize_mask(uint32_t bits, int N, int M, uint32_t* filled) {
  uint32_t keep = 0, fill = 0;
  int c = 0;
  for (int i = 0; i < M; ++i)
    if (((bits >> i) & 1u) && c < N) { keep |= 1u << i; ++c; }
  for (int i = 0; i < M && c < N; ++i)
    if (!((bits >> i) & 1u)) { fill |= 1u << i; ++c; }
  *filled = fill;
  return keep | fill;
}

// ---------------------------------------------------------------------------------------------
// "Stream order" of a weight for the persistent product kernel: the LDS image of every (16-row group,
// K step) as one contiguous kilobyte.
//   values (2:4 form, a step = 32 compressed values = 64 dense k) or dense weights (a step = 32 weights):
//     block (row/16, step) at ((row/16) * nk + step) * 1024; inside it the 16-byte piece `chunk` (0..3) of
//     row r = row % 16 at (4 r + (chunk ^ (r/2 % 4))) * 16  (the XOR is the LDS swizzle)
//   selectors of the 2:4 form: block (row/256, step) of 2 KiB; rows r and r+16 of a 32-row pair share the
//     32-bit word of (r % 16, chunk): low half = the first row's 16 selector bits of that chunk, high half
//     = the second row's, which is what the matrix instruction's ABID modifier selects
// ---------------------------------------------------------------------------------------------
__host__ __device__ __forceinline__ int64_t stream_piece_offset(int64_t row, int64_t step, int chunk, int64_t nk) {
  const int r = (int)(row & 15);
  return (((row >> 4) * nk + step) << 10) + ((r * 4 + (chunk ^ ((r >> 1) & 3))) << 4);
}
__host__ __device__ __forceinline__ int64_t stream_selector_offset(int64_t row, int64_t step, int chunk, int64_t nk) {
  const int r = (int)(row & 255);
  return (((row >> 8) * nk + step) << 11) + (r >> 5) * 256 + (r & 15) * 16 + chunk * 4 + ((r >> 4) & 1) * 2;
}

// int8 2:4 form: a lane's 16 compressed values take a whole selector word, so a row has 16 bytes of selectors
// per K step (one word per lane group kb) and a (256-row tile, step) block is 4 KiB: [16-row block][row][kb]
__host__ __device__ __forceinline__ int64_t stream_selector8_offset(int64_t row, int64_t step, int kb, int64_t nk) {
  const int r = (int)(row & 255);
  return (((row >> 8) * nk + step) << 12) + (r >> 4) * 256 + (r & 15) * 16 + kb * 4;
}

}  // namespace nm
