// Magnitude selection of Eq. (1) (Section 3.1) for the levels a layer-wise configuration draws from (N in {1, 2, 4},
// N < M), written for few vector instructions per weight: the packing kernels are bound by them, not by memory,
// when every pair of a group is compared (M (M - 1) / 2 compares and twice as many rank updates per group).
//
// Every weight becomes one 32-bit ORDER KEY whose unsigned order is the selection order:
//     bits 17..31  magnitude (the bfloat16 pattern without its sign)
//     bits  1..4   M - 1 - position in the group   (equal magnitudes: the lower position is the larger key)
//     bit   0      the sign                        (never decides: positions differ)
// so the N kept weights of a group are its N largest keys, found with max/min networks, and a winner's key still
// holds its value and its position.  Rotating a winner's key right by 5 gives its PLACE KEY
//     bits 28..31  M - 1 - position,  bit 27 sign,  bits 12..26 magnitude
// whose descending order is ascending position, the order the packed layout stores kept values in.
// Two instructions build a key (a rotate that brings magnitude and sign into place, a mask-and-or), one more
// extracts a value or a position.
#pragma once
#include "nm_device.h"

namespace nm {

__host__ __device__ __forceinline__ uint32_t rotr32(uint32_t x, int r) { return (x >> r) | (x << ((32 - r) & 31)); }
__host__ __device__ __forceinline__ uint32_t umax(uint32_t a, uint32_t b) { return a > b ? a : b; }
__host__ __device__ __forceinline__ uint32_t umin(uint32_t a, uint32_t b) { return a < b ? a : b; }
// compare-exchange: the larger key ends in a
__host__ __device__ __forceinline__ void order2(uint32_t& a, uint32_t& b) {
  const uint32_t hi = umax(a, b), lo = umin(a, b);
  a = hi; b = lo;
}
// four keys in descending order
__host__ __device__ __forceinline__ void sort4_desc(uint32_t (&k)[4]) {
  order2(k[0], k[1]); order2(k[2], k[3]); order2(k[0], k[2]); order2(k[1], k[3]); order2(k[1], k[2]);
}
// a bitonic run of four (as left by top4_of_sorted) in descending order
__host__ __device__ __forceinline__ void sort4_bitonic_desc(uint32_t (&k)[4]) {
  order2(k[0], k[2]); order2(k[1], k[3]); order2(k[0], k[1]); order2(k[2], k[3]);
}
// the four largest of two descending runs of four (in no particular order: a bitonic run)
__host__ __device__ __forceinline__ void top4_of_sorted(const uint32_t (&a)[4], const uint32_t (&b)[4], uint32_t (&t)[4]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) t[i] = umax(a[i], b[3 - i]);
}

// Order key of weight `pos` (position inside its group of M) taken from dword d of the row: the weight sits in the
// low (HALF = 0) or high (HALF = 1) 16 bits.
template <int HALF>
__host__ __device__ __forceinline__ uint32_t order_key(uint32_t d, int pos, int M) {
  return (rotr32(d, HALF ? 31 : 15) & 0xFFFE0001u) | ((uint32_t)(M - 1 - pos) << 1);
}
__host__ __device__ __forceinline__ uint32_t place_key(uint32_t order_key_) { return rotr32(order_key_, 5); }
__host__ __device__ __forceinline__ uint32_t place_value(uint32_t pk) { return (pk >> 12) & 0xFFFFu; }
__host__ __device__ __forceinline__ uint32_t place_invpos(uint32_t pk) { return pk >> 28; }

// The kept weights of one group of M, as place keys in descending order (= ascending position).
// key[i] is the order key of position i.
template <int N, int M>
__host__ __device__ __forceinline__ void select_group(const uint32_t (&key)[M], uint32_t (&win)[N]) {
  static_assert((N == 1 || N == 2 || N == 4) && N < M && (M == 4 || M == 8 || M == 16), "levels of the fast selection");
  if constexpr (N == 1) {
    uint32_t best = key[0];
#pragma unroll
    for (int i = 1; i + 1 < M; i += 2) best = umax(best, umax(key[i], key[i + 1]));
    best = umax(best, key[M - 1]);
    win[0] = place_key(best);
  } else if constexpr (N == 2) {
    // (largest, second largest) of every pair, merged pairwise
    uint32_t hi[M / 2], lo[M / 2];
#pragma unroll
    for (int i = 0; i < M / 2; ++i) { hi[i] = umax(key[2 * i], key[2 * i + 1]); lo[i] = umin(key[2 * i], key[2 * i + 1]); }
#pragma unroll
    for (int n = M / 2; n > 1; n /= 2) {
#pragma unroll
      for (int i = 0; i < n / 2; ++i) {
        const uint32_t h = umax(hi[2 * i], hi[2 * i + 1]);
        const uint32_t l = umax(umin(hi[2 * i], hi[2 * i + 1]), umax(lo[2 * i], lo[2 * i + 1]));
        hi[i] = h; lo[i] = l;
      }
    }
    const uint32_t a = place_key(hi[0]), b = place_key(lo[0]);
    win[0] = umax(a, b); win[1] = umin(a, b);
  } else {
    uint32_t run[M / 4][4];
#pragma unroll
    for (int r = 0; r < M / 4; ++r) {
#pragma unroll
      for (int i = 0; i < 4; ++i) run[r][i] = key[4 * r + i];
      sort4_desc(run[r]);
    }
    uint32_t top[4];
    if constexpr (M == 4) {
#pragma unroll
      for (int i = 0; i < 4; ++i) top[i] = run[0][i];
    } else if constexpr (M == 8) {
      top4_of_sorted(run[0], run[1], top);
    } else {
      uint32_t t[4], u[4];
      top4_of_sorted(run[0], run[1], t);
      top4_of_sorted(run[2], run[3], u);
      sort4_bitonic_desc(t);
      sort4_bitonic_desc(u);
      top4_of_sorted(t, u, top);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) win[i] = place_key(top[i]);
    sort4_desc(win);
  }
}

// One 16-weight chunk (8 dwords of a row, weight 2i in the low half of d[i]): per group the kept values in
// ascending position, the index fields, and on request the keep mask.
template <int N, int M>
struct FastChunkCoder {
  static constexpr int B = log2_of(M);
  static constexpr int G = 16 / M;
  static constexpr int NV = G * N;
  static constexpr int NB = NV * B;

  uint32_t win[G][N];  // place keys of the kept weights, ascending position
  uint32_t vals[NV];
  uint64_t ibits;

  __host__ __device__ __forceinline__ void run(const uint32_t (&d)[8]) {
    uint64_t inv = 0;  // the fields with M - 1 - position; complemented at the end
#pragma unroll
    for (int g = 0; g < G; ++g) {
      uint32_t key[M];
#pragma unroll
      for (int i = 0; i < M; i += 2) {
        key[i] = order_key<0>(d[(g * M + i) / 2], i, M);
        key[i + 1] = order_key<1>(d[(g * M + i) / 2], i + 1, M);
      }
      select_group<N, M>(key, win[g]);
#pragma unroll
      for (int j = 0; j < N; ++j) {
        vals[g * N + j] = place_value(win[g][j]);
        inv |= (uint64_t)place_invpos(win[g][j]) << (B * (g * N + j));
      }
    }
    ibits = ~inv & (NB == 64 ? ~0ull : ((1ull << NB) - 1ull));
  }

  // bit i = weight i of the chunk is kept
  __host__ __device__ __forceinline__ uint32_t keep16() const {
    uint32_t acc = 0;  // group g's bits mirrored into the slot of group G-1-g, then the whole word is reversed
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int j = 0; j < N; ++j) acc |= (1u << ((G - 1 - g) * M)) << place_invpos(win[g][j]);
    return __builtin_bitreverse32(acc) >> 16;
  }

  // The chunk as a 2:4 operand (N <= 2): per run of four weights two 16-bit slots (kept weights in ascending
  // position, zero-filled) and four selector bits (2-bit positions inside the run).
  __host__ __device__ __forceinline__ void sparse_operand(uint32_t (&piece)[4], uint32_t& sel) const {
    static_assert(N <= 2, "levels with at most two kept weights per run of four");
    constexpr int RUNS = M / 4;
    sel = 0;
#pragma unroll
    for (int r = 0; r < 4; ++r) piece[r] = 0;
#pragma unroll
    for (int g = 0; g < G; ++g) {
      uint32_t prev_run = 0xFFFFFFFFu;
#pragma unroll
      for (int j = 0; j < N; ++j) {
        const uint32_t pos = (uint32_t)(M - 1) - place_invpos(win[g][j]);
        const uint32_t run = pos >> 2, within = pos & 3u;
        const uint32_t second = (j > 0 && run == prev_run) ? 1u : 0u;
        prev_run = run;
        const uint32_t v = vals[g * N + j] << (16 * second);
        if constexpr (RUNS == 1) {
          piece[g] |= v;
        } else {
#pragma unroll
          for (int r = 0; r < RUNS; ++r) piece[g * RUNS + r] |= (run == (uint32_t)r) ? v : 0u;
        }
        sel |= within << (4 * (g * RUNS + run) + 2 * second);
      }
    }
  }
};

// Dwords of a chunk with the pruned weights set to +0.
__host__ __device__ __forceinline__ void mask_chunk(const uint32_t (&d)[8], uint32_t keep16, uint32_t (&out)[8]) {
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const uint32_t lo = (uint32_t)(-(int32_t)((keep16 >> (2 * i)) & 1u)) & 0xFFFFu;
    const uint32_t hi = (uint32_t)(-(int32_t)((keep16 >> (2 * i + 1)) & 1u)) << 16;
    out[i] = d[i] & (lo | hi);
  }
}

}  // namespace nm
