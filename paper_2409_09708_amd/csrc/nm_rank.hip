// Nested N:M levels from one stored rank per weight (Section 3, "Subset-Superset Relationship"): under one
// pruning criterion the weights kept at a sparser level are among those kept at a denser one, so the rank
// of a weight inside its group of M, in the order (magnitude descending, position ascending), holds every
// level of that M at once: the mask of N:M is rank < N.  A supernet that re-derives a layer's mask whenever
// a new level is sampled (Section 3.1, "Dynamic Masking") ranks a weight matrix once per weight update and
// then gets any level's mask or packed form from the ranks.
//
// Ranks are stored 4 bits per weight: weight k of row o in bits [4 (k mod 2), +4) of byte o*K/2 + k/2.
// All kernels stream (HBM-bound): 2 bytes read + 1/2 byte written per weight for the ranking.
#include "nm_device.h"
#include "nm_launch.h"

namespace nm {

// ranks of the M members of one group by pairwise comparison (equal scores: the lower position goes first)
template <int M>
__device__ __forceinline__ uint64_t group_ranks(const uint32_t (&key)[M]) {
  uint32_t rank[M];
#pragma unroll
  for (int i = 0; i < M; ++i) rank[i] = 0;
#pragma unroll
  for (int i = 0; i < M; ++i) {
#pragma unroll
    for (int j = i + 1; j < M; ++j) {
      const bool i_first = key[i] >= key[j];
      rank[j] += i_first ? 1u : 0u;
      rank[i] += i_first ? 0u : 1u;
    }
  }
  uint64_t packed = 0;
#pragma unroll
  for (int i = 0; i < M; ++i) packed |= (uint64_t)rank[i] << (4 * i);
  return packed;
}

// contiguous matrix (ldw = K, 16-byte aligned): one lane per 16 weights = 8 bytes of ranks
template <int M>
__device__ __forceinline__ void rank_chunk(const bf16_t* __restrict__ W, int64_t c, uint64_t* __restrict__ rank);

template <int M>
__global__ void __launch_bounds__(256)
rank_flat_kernel(const bf16_t* __restrict__ W, int64_t n_chunks, uint64_t* __restrict__ rank) {
  const int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (c < n_chunks) rank_chunk<M>(W, c, rank);
}

// the work of one lane on chunk c of a contiguous matrix
template <int M>
__device__ __forceinline__ void rank_chunk(const bf16_t* __restrict__ W, int64_t c, uint64_t* __restrict__ rank) {
  const uint4* src = reinterpret_cast<const uint4*>(W + c * 16);
  const uint4 a = src[0], b = src[1];
  const uint32_t d[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
  uint64_t out = 0;
#pragma unroll
  for (int g = 0; g < 16 / M; ++g) {
    uint32_t key[M];
#pragma unroll
    for (int i = 0; i < M; ++i) {
      const int e = g * M + i;
      key[i] = saliency_key((e & 1) ? (d[e >> 1] >> 16) : (d[e >> 1] & 0xFFFFu));
    }
    out |= group_ranks<M>(key) << (4 * M * g);
  }
  rank[c] = out;
}

// One launch for many matrices (a supernet ranks all its layers after a weight update): a block finds its
// matrix from the running block counts, the descriptors ride in the kernel arguments.
struct RankEntry {
  const bf16_t* W;
  uint64_t* rank;
  int64_t n_chunks;
  uint32_t block_end;  // exclusive prefix end, in blocks
  uint32_t M;
};
constexpr int kRankBatchMax = 96;
struct RankBatchArgs {
  RankEntry e[kRankBatchMax];
  int count;
};

__global__ void __launch_bounds__(256) rank_batched_kernel(const RankBatchArgs args) {
  int m = 0, hi = args.count - 1;  // the first matrix whose blocks end beyond this one, by bisection
  while (m < hi) {
    const int mid = (m + hi) >> 1;
    if (blockIdx.x >= args.e[mid].block_end) m = mid + 1;
    else hi = mid;
  }
  const RankEntry& d = args.e[m];
  const uint32_t first = m ? args.e[m - 1].block_end : 0u;
  const int64_t c = (int64_t)(blockIdx.x - first) * 256 + threadIdx.x;
  if (c >= d.n_chunks) return;
  if (d.M == 4) rank_chunk<4>(d.W, c, d.rank);
  else if (d.M == 8) rank_chunk<8>(d.W, c, d.rank);
  else rank_chunk<16>(d.W, c, d.rank);
}

// any leading dimension and alignment: one thread per group, M/2 bytes of ranks each
__global__ void __launch_bounds__(256)
rank_general_kernel(const bf16_t* __restrict__ W, int64_t O, int64_t K, int64_t ldw, int M, uint8_t* __restrict__ rank) {
  const int64_t G = K / M;
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= O * G) return;
  const int64_t o = id / G, g = id % G;
  uint32_t key[16];
  for (int i = 0; i < M; ++i) key[i] = saliency_key(W[o * ldw + g * M + i]);
  uint8_t* dst = rank + (o * K + g * M) / 2;  // K and M are even: a group starts on a byte
  for (int i = 0; i < M; i += 2) {
    uint32_t r[2];
    for (int h = 0; h < 2; ++h) {
      uint32_t before = 0;
      for (int j = 0; j < M; ++j) before += (key[j] > key[i + h]) || (key[j] == key[i + h] && j < i + h);
      r[h] = before;
    }
    dst[i / 2] = (uint8_t)(r[0] | (r[1] << 4));
  }
}

// mask words of level N from ranks: one thread per 32-bit word
__global__ void __launch_bounds__(256)
rank_mask_kernel(const uint8_t* __restrict__ rank, int64_t O, int64_t K, int N, uint32_t* __restrict__ mask) {
  const int64_t nw = mask_words_per_row(K);
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= O * nw) return;
  const int64_t o = id / nw, w = id % nw;
  uint32_t word = 0;
  const int64_t k_end = (w * 32 + 32 < K) ? w * 32 + 32 : K;
  for (int64_t k = w * 32; k < k_end; k += 2) {
    const uint32_t byte = rank[(o * K + k) / 2];
    word |= ((byte & 15u) < (uint32_t)N ? 1u : 0u) << (k & 31);
    word |= ((byte >> 4) < (uint32_t)N ? 1u : 0u) << ((k & 31) + 1);
  }
  mask[o * nw + w] = word;
}

// Mask words of level N:M from a supplied saliency (Section 3.1: rho may be any score): one lane per mask word.
// Order inside a group: NaN first, then descending value (-0 = +0), then ascending position; a weight is kept
// when fewer than N members of its group come before it.
__device__ __forceinline__ uint32_t score_key(float v) {
  // unsigned key that increases with the score; every NaN maps above +inf
  uint32_t u = __float_as_uint(v);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0xFFFFFFFFu;
  if (u == 0x80000000u) u = 0u;  // -0 ties +0
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__global__ void __launch_bounds__(256)
score_mask_kernel(const float* __restrict__ score, int64_t O, int64_t K, int64_t lds, int N, int M,
                  uint32_t* __restrict__ mask) {
  const int64_t nw = mask_words_per_row(K);
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= O * nw) return;
  const int64_t o = id / nw, w = id % nw;
  const int64_t k_end = (w * 32 + 32 < K) ? w * 32 + 32 : K;
  const float* row = score + o * lds;
  uint32_t word = 0;
  for (int64_t g = w * 32; g < k_end; g += M) {  // M divides 32 and K, so groups never straddle a word
    uint32_t key[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) key[i] = i < M ? score_key(row[g + i]) : 0u;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      if (i >= M) break;
      int before = 0;
#pragma unroll
      for (int j = 0; j < 16; ++j)
        if (j < M) before += (key[j] > key[i] || (key[j] == key[i] && j < i)) ? 1 : 0;
      word |= (before < N ? 1u : 0u) << ((g + i) & 31);
    }
  }
  mask[o * nw + w] = word;
}

static bool rank_flat_ok(const bf16_t* W, int64_t O, int64_t K, int64_t ldw, const uint8_t* rank) {
  return ldw == K && (O * K) % 16 == 0 && (((uintptr_t)W | (uintptr_t)rank) & 15u) == 0 &&
         (O * K / 16 + 255) / 256 <= 0x7FFFFFFF;
}

hipError_t launch_rank(const bf16_t* W, int64_t O, int64_t K, int64_t ldw, int M, uint8_t* rank, hipStream_t s) {
  if (rank_flat_ok(W, O, K, ldw, rank)) {
    const int64_t n_chunks = O * K / 16;
    const dim3 grid((unsigned)((n_chunks + 255) / 256));
    uint64_t* out = reinterpret_cast<uint64_t*>(rank);
    if (M == 4) hipLaunchKernelGGL(rank_flat_kernel<4>, grid, dim3(256), 0, s, W, n_chunks, out);
    else if (M == 8) hipLaunchKernelGGL(rank_flat_kernel<8>, grid, dim3(256), 0, s, W, n_chunks, out);
    else hipLaunchKernelGGL(rank_flat_kernel<16>, grid, dim3(256), 0, s, W, n_chunks, out);
  } else {
    const int64_t n = O * (K / M);
    if ((n + 255) / 256 > 0x7FFFFFFF) return hipErrorInvalidValue;
    hipLaunchKernelGGL(rank_general_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, W, O, K, ldw, M, rank);
  }
  return hipGetLastError();
}

hipError_t launch_rank_batched(const RankDesc* descs, int count, hipStream_t s) {
  RankBatchArgs args;
  args.count = 0;
  uint64_t blocks = 0;
  auto flush = [&]() {
    if (args.count) {
      hipLaunchKernelGGL(rank_batched_kernel, dim3((unsigned)blocks), dim3(256), 0, s, args);
      args.count = 0;
      blocks = 0;
    }
  };
  for (int i = 0; i < count; ++i) {
    const RankDesc& d = descs[i];
    if (!rank_flat_ok(d.W, d.O, d.K, d.K, d.rank)) {
      hipError_t e = launch_rank(d.W, d.O, d.K, d.K, d.M, d.rank, s);
      if (e != hipSuccess) return e;
      continue;
    }
    const int64_t n_chunks = d.O * d.K / 16;
    const uint64_t nb = (uint64_t)((n_chunks + 255) / 256);
    if (args.count == kRankBatchMax || blocks + nb > 0x7FFFFFFFull) flush();
    RankEntry& e = args.e[args.count++];
    e.W = d.W; e.rank = reinterpret_cast<uint64_t*>(d.rank); e.n_chunks = n_chunks; e.M = (uint32_t)d.M;
    blocks += nb;
    e.block_end = (uint32_t)blocks;
  }
  flush();
  return hipGetLastError();
}

hipError_t launch_rank_mask(const uint8_t* rank, int64_t O, int64_t K, int N, uint32_t* mask, hipStream_t s) {
  const int64_t n = O * mask_words_per_row(K);
  if ((n + 255) / 256 > 0x7FFFFFFF) return hipErrorInvalidValue;
  hipLaunchKernelGGL(rank_mask_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, rank, O, K, N, mask);
  return hipGetLastError();
}

hipError_t launch_score_mask(const float* score, int64_t O, int64_t K, int64_t lds, int N, int M, uint32_t* mask,
                             hipStream_t s) {
  const int64_t n = O * mask_words_per_row(K);
  if ((n + 255) / 256 > 0x7FFFFFFF) return hipErrorInvalidValue;
  hipLaunchKernelGGL(score_mask_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, score, O, K, lds, N, M, mask);
  return hipGetLastError();
}

}  // namespace nm
