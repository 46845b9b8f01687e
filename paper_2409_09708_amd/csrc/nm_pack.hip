// Magnitude N:M selection (Section 3.1, Eq. (1)), packing into values + log2(M)-bit indices
// (Section 1; Section 2, Fig. 2 upper part) and the inverse, for gfx950.
//
// Streaming kernels: every weight is read once and every output byte written once, so the bound is
// HBM.  The fast kernels treat a contiguous matrix as a flat run of 16-weight chunks (one per lane,
// two 16-byte loads); because rows are contiguous and unpadded in every output, lane i of a block
// writes the i-th slice of each output and all stores coalesce.  Index fields narrower than a
// byte or not byte aligned (3-bit fields, 1:16) are assembled into words in LDS first.
#include "nm_device.h"
#include "nm_launch.h"
#include "nm_select.h"

#include <type_traits>

namespace nm {

constexpr int kPackThreads = 256;
constexpr int kChunk = 16;          // weights per chunk in the fast kernels (two 16-byte loads)
constexpr int kChunksPerLane = 2;   // chunks a lane handles, all their loads in flight before the first is coded
constexpr int kBlockChunks = kPackThreads * kChunksPerLane;

// One 16-weight chunk: selection, compaction in ascending position, index fields.
template <int N, int M, bool EXTERNAL_MASK>
struct ChunkCoder {
  static constexpr int B = log2_of(M);
  static constexpr int G = kChunk / M;   // groups per chunk
  static constexpr int NV = G * N;       // kept values per chunk
  static constexpr int NB = NV * B;      // index bits per chunk (<= 64)

  uint32_t vals[NV];
  uint64_t ibits;
  uint32_t keep16;    // kept positions of the chunk (bit i = weight i kept and not a filler)

  __device__ __forceinline__ void run(const uint32_t (&e)[kChunk], uint32_t mask16) {
    ibits = 0;
    keep16 = 0;
#pragma unroll
    for (int i = 0; i < NV; ++i) vals[i] = 0;
#pragma unroll
    for (int g = 0; g < G; ++g) {
      uint32_t km, filled = 0;
      if (EXTERNAL_MASK) {
        km = legalize_mask((mask16 >> (g * M)) & ((1u << M) - 1u), N, M, &filled);
      } else {
        uint32_t key[M];
#pragma unroll
        for (int i = 0; i < M; ++i) key[i] = saliency_key(e[g * M + i]);
        km = select_top_n<N, M>(key);
      }
      keep16 |= (km & ~filled) << (g * M);
      uint32_t cnt = 0;
#pragma unroll
      for (int i = 0; i < M; ++i) {
        const bool k = (km >> i) & 1u;
        const uint32_t v = ((filled >> i) & 1u) ? 0u : e[g * M + i];
        // the i-th member can only land in slots max(0, i-(M-N)) .. min(N-1, i)
#pragma unroll
        for (int j = 0; j < N; ++j) {
          if (j <= i && j >= i - (M - N)) vals[g * N + j] = (k && cnt == (uint32_t)j) ? v : vals[g * N + j];
        }
        ibits |= k ? ((uint64_t)i << (B * (g * N) + B * cnt)) : 0ull;
        cnt += k ? 1u : 0u;
      }
    }
  }
};

template <int NV>
__device__ __forceinline__ void store_values(bf16_t* __restrict__ dst, const uint32_t (&v)[NV]) {
  // dst is aligned to the largest power of two dividing 2*NV bytes (at most 16)
  if constexpr (NV % 8 == 0) {
#pragma unroll
    for (int i = 0; i < NV; i += 8) {
      uint4 q;
      q.x = v[i] | (v[i + 1] << 16); q.y = v[i + 2] | (v[i + 3] << 16);
      q.z = v[i + 4] | (v[i + 5] << 16); q.w = v[i + 6] | (v[i + 7] << 16);
      *reinterpret_cast<uint4*>(dst + i) = q;
    }
  } else if constexpr (NV % 4 == 0) {
#pragma unroll
    for (int i = 0; i < NV; i += 4) {
      uint2 q;
      q.x = v[i] | (v[i + 1] << 16); q.y = v[i + 2] | (v[i + 3] << 16);
      *reinterpret_cast<uint2*>(dst + i) = q;
    }
  } else if constexpr (NV % 2 == 0) {
#pragma unroll
    for (int i = 0; i < NV; i += 2) *reinterpret_cast<uint32_t*>(dst + i) = v[i] | (v[i + 1] << 16);
  } else {
#pragma unroll
    for (int i = 0; i < NV; ++i) dst[i] = (bf16_t)v[i];
  }
}

// Levels whose magnitude selection runs on order keys and max/min networks (nm_select.h): about a quarter of the
// vector instructions of the all-pairs ranking, which is what bounds these kernels.
template <int N, int M>
constexpr bool kFastLevel = (N == 1 || N == 2 || N == 4) && N < M;

// Work of one block on kBlockChunks consecutive chunks of one contiguous matrix.
//   values/indices may be NULL (prune only); mask_out / w_masked may be NULL (pack only).
// SRC: where the selection comes from: 0 = magnitude (Eq. (1)), 1 = the caller's mask words, 2 = stored ranks
// (4 bits per weight; kept = rank < N)
// stream_ws (magnitude selection at the fast levels only): the product kernel's operand order, written beside the
// packed form.
template <int N, int M, int SRC>
__device__ __forceinline__ void code_block(const bf16_t* W, int64_t n_chunks, int64_t chunk0,
                                           const uint32_t* __restrict__ mask_in, bf16_t* __restrict__ values,
                                           uint32_t* __restrict__ indices, uint32_t* __restrict__ mask_out,
                                           bf16_t* w_masked, uint32_t* sbits, unsigned char* stream_ws = nullptr,
                                           int64_t K = 0) {
  constexpr bool FAST = SRC == 0 && kFastLevel<N, M>;
  using Coder = std::conditional_t<FAST, FastChunkCoder<N, M>, ChunkCoder<N, M, SRC != 0>>;
  constexpr int NB = Coder::NB;
  constexpr bool DIRECT_INDEX = (NB == 8 || NB == 16 || NB == 32 || NB == 64);
  constexpr int BLOCK_WORDS = kBlockChunks * NB / 32;
  const int tid = threadIdx.x;

  if (!DIRECT_INDEX && indices) {
    for (int i = tid; i < BLOCK_WORDS + 2; i += kPackThreads) sbits[i] = 0;
    __syncthreads();
  }
  // this lane's chunks: tid, tid + 256, ... of the block's run; every load leaves before anything is coded
  uint32_t d[kChunksPerLane][8];
#pragma unroll
  for (int u = 0; u < kChunksPerLane; ++u) {
    const int64_t c = chunk0 + u * kPackThreads + tid;
    if (c < n_chunks) {
      const uint4* src = reinterpret_cast<const uint4*>(W + c * kChunk);
      const uint4 a = src[0], b = src[1];
      d[u][0] = a.x; d[u][1] = a.y; d[u][2] = a.z; d[u][3] = a.w;
      d[u][4] = b.x; d[u][5] = b.y; d[u][6] = b.z; d[u][7] = b.w;
    }
  }
#pragma unroll
  for (int u = 0; u < kChunksPerLane; ++u) {
    const int64_t c = chunk0 + u * kPackThreads + tid;
    if (c >= n_chunks) continue;
    Coder coder;
    uint32_t keep16 = 0;
    if constexpr (FAST) {
      coder.run(d[u]);
      if (mask_out || w_masked || (stream_ws && N > 2)) keep16 = coder.keep16();
    } else {
      uint32_t e[kChunk];
#pragma unroll
      for (int i = 0; i < 8; ++i) { e[2 * i] = d[u][i] & 0xFFFFu; e[2 * i + 1] = d[u][i] >> 16; }
      uint32_t mask16 = 0;
      if (SRC == 1) mask16 = reinterpret_cast<const uint16_t*>(mask_in)[c];
      if (SRC == 2) {
        const uint64_t r = reinterpret_cast<const uint64_t*>(mask_in)[c];
#pragma unroll
        for (int i = 0; i < kChunk; ++i) mask16 |= (((uint32_t)(r >> (4 * i)) & 15u) < (uint32_t)N ? 1u : 0u) << i;
      }
      coder.run(e, mask16);
      keep16 = coder.keep16;
    }

    if (values) store_values<Coder::NV>(values + c * Coder::NV, coder.vals);
    if (indices) {
      if constexpr (NB == 8) reinterpret_cast<uint8_t*>(indices)[c] = (uint8_t)coder.ibits;
      else if constexpr (NB == 16) reinterpret_cast<uint16_t*>(indices)[c] = (uint16_t)coder.ibits;
      else if constexpr (NB == 32) indices[c] = (uint32_t)coder.ibits;
      else if constexpr (NB == 64) reinterpret_cast<uint64_t*>(indices)[c] = coder.ibits;
      else {
        const int off = (u * kPackThreads + tid) * NB;
        const int w = off >> 5, sh = off & 31;
        const uint64_t lo = coder.ibits << sh;
        const uint32_t hi = sh ? (uint32_t)(coder.ibits >> (64 - sh)) : 0u;
        if ((uint32_t)lo) atomicOr(&sbits[w], (uint32_t)lo);
        if ((uint32_t)(lo >> 32)) atomicOr(&sbits[w + 1], (uint32_t)(lo >> 32));
        if (hi) atomicOr(&sbits[w + 2], hi);
      }
    }
    if (mask_out) reinterpret_cast<uint16_t*>(mask_out)[c] = (uint16_t)keep16;
    if constexpr (FAST) {
      if (stream_ws) {
        // this lane's 16 weights are one 16-byte chunk of a row's K step (2:4 form), or two of them (dense form)
        const int64_t per_row = K / kChunk;
        const int64_t o = c / per_row, kc = c % per_row;
        if constexpr (N <= 2) {
          const int64_t nk = K / 64;
          uint32_t piece[4], sel;
          coder.sparse_operand(piece, sel);
          *reinterpret_cast<uint4*>(stream_ws + stream_piece_offset(o, kc >> 2, (int)(kc & 3), nk)) =
              make_uint4(piece[0], piece[1], piece[2], piece[3]);
          unsigned char* sel_s = stream_ws + (size_t)(n_chunks * 16);  // the values take O*K bytes: 16 per chunk
          *reinterpret_cast<uint16_t*>(sel_s + stream_selector_offset(o, kc >> 2, (int)(kc & 3), nk)) = (uint16_t)sel;
        } else {
          const int64_t nk = K / 32;
          uint32_t w[8];
          mask_chunk(d[u], keep16, w);
          const int64_t pc = kc * 2;
          *reinterpret_cast<uint4*>(stream_ws + stream_piece_offset(o, pc >> 2, (int)(pc & 3), nk)) =
              make_uint4(w[0], w[1], w[2], w[3]);
          *reinterpret_cast<uint4*>(stream_ws + stream_piece_offset(o, (pc + 1) >> 2, (int)((pc + 1) & 3), nk)) =
              make_uint4(w[4], w[5], w[6], w[7]);
        }
      }
    }
    if (w_masked) {
      uint32_t o[8];
      mask_chunk(d[u], keep16, o);
      uint4* dst = reinterpret_cast<uint4*>(w_masked + c * kChunk);
      dst[0] = make_uint4(o[0], o[1], o[2], o[3]);
      dst[1] = make_uint4(o[4], o[5], o[6], o[7]);
    }
  }
  if (!DIRECT_INDEX && indices) {
    __syncthreads();
    const int64_t left = n_chunks - chunk0;
    const int nact = left < kBlockChunks ? (int)left : kBlockChunks;
    const int nwords = (nact * NB) >> 5;  // exact: whole rows hold whole words
    uint32_t* dst = indices + (chunk0 * NB >> 5);
    for (int i = tid; i < nwords; i += kPackThreads) dst[i] = sbits[i];
  }
}

constexpr int kSbitsWords = kBlockChunks * 64 / 32 + 2;  // room for the widest per-chunk index field run (<= 64 bits)

template <int N, int M, int SRC>
__global__ void __launch_bounds__(kPackThreads)
code_flat_kernel(const bf16_t* W, int64_t n_chunks, const uint32_t* __restrict__ mask_in,
                 bf16_t* __restrict__ values, uint32_t* __restrict__ indices, uint32_t* __restrict__ mask_out,
                 bf16_t* w_masked) {  // w_masked may be W itself (in-place pruning)
  __shared__ uint32_t sbits[kSbitsWords];
  code_block<N, M, SRC>(W, n_chunks, (int64_t)blockIdx.x * kBlockChunks, mask_in, values, indices,
                                  mask_out, w_masked, sbits);
}

// ---------------------------------------------------------------------------------------------
// One launch for many matrices: a block finds its matrix from the running block counts.
// ---------------------------------------------------------------------------------------------
struct BatchEntry {
  const bf16_t* W;
  bf16_t* values;
  uint32_t* indices;
  unsigned char* stream_ws;  // NULL, or where the product kernel's operand order is written as well
  const uint32_t* rank;      // stored ranks the selection is read from (the ranked launch), else unused
  int64_t n_chunks;
  int64_t K;
  uint32_t block_end;  // exclusive prefix end, in blocks
  uint16_t N, M;
};
static_assert(sizeof(BatchEntry) == 64, "descriptor size");
constexpr int kBatchMax = 56;  // 56 * 64 bytes of descriptors ride in the kernel arguments
struct BatchArgs {
  BatchEntry e[kBatchMax];
  int count;
};

#define NM_FOR_EACH_LEVEL(X)                                                                         \
  X(1, 4) X(2, 4) X(3, 4) X(4, 4)                                                                    \
  X(1, 8) X(2, 8) X(3, 8) X(4, 8) X(5, 8) X(6, 8) X(7, 8) X(8, 8)                                    \
  X(1, 16) X(2, 16) X(3, 16) X(4, 16) X(5, 16) X(6, 16) X(7, 16) X(8, 16) X(9, 16) X(10, 16)         \
  X(11, 16) X(12, 16) X(13, 16) X(14, 16) X(15, 16) X(16, 16)

// Levels the batched kernel carries inline (the ones a layer-wise configuration draws from); other
// levels go through per-matrix launches.
#define NM_FOR_EACH_BATCH_LEVEL(X) X(1, 4) X(2, 4) X(1, 8) X(2, 8) X(4, 8) X(1, 16) X(2, 16) X(4, 16)

template <int SRC>  // 0: selection by magnitude, 2: from stored ranks
__global__ void __launch_bounds__(kPackThreads) pack_batched_kernel(const BatchArgs args) {
  __shared__ uint32_t sbits[kSbitsWords];
  int m = 0, hi = args.count - 1;  // the first matrix whose blocks end beyond this one, by bisection
  while (m < hi) {
    const int mid = (m + hi) >> 1;
    if (blockIdx.x >= args.e[mid].block_end) m = mid + 1;
    else hi = mid;
  }
  const BatchEntry& d = args.e[m];
  const uint32_t first = m ? args.e[m - 1].block_end : 0u;
  const int64_t chunk0 = (int64_t)(blockIdx.x - first) * kBlockChunks;
  const int level = d.N * 32 + d.M;
  switch (level) {
#define X(n, mm)                                                                                      \
  case n * 32 + mm:                                                                                   \
    code_block<n, mm, SRC>(d.W, d.n_chunks, chunk0, SRC ? d.rank : nullptr, d.values, d.indices, nullptr, \
                           nullptr, sbits, d.stream_ws, d.K);                                         \
    break;
    NM_FOR_EACH_BATCH_LEVEL(X)
#undef X
    default: break;
  }
}

// ---------------------------------------------------------------------------------------------
// General kernels: any K % M == 0, any leading dimension, no alignment beyond the element.
// ---------------------------------------------------------------------------------------------
__device__ inline uint32_t group_keep(const bf16_t* __restrict__ W, int64_t ldw, const uint32_t* __restrict__ mask_in,
                                      int64_t K, int64_t o, int64_t g, int N, int M, uint32_t* filled,
                                      const uint8_t* __restrict__ rank_in = nullptr) {
  *filled = 0;
  if (rank_in) {  // stored ranks: kept = rank < N
    uint32_t km = 0;
    for (int i = 0; i < M; i += 2) {
      const uint32_t byte = rank_in[(o * K + g * M + i) / 2];
      km |= ((byte & 15u) < (uint32_t)N ? 1u : 0u) << i;
      km |= ((byte >> 4) < (uint32_t)N ? 1u : 0u) << (i + 1);
    }
    return legalize_mask(km, N, M, filled);
  }
  if (mask_in) {
    const int64_t k0 = g * M;
    const uint32_t word = mask_in[o * mask_words_per_row(K) + (k0 >> 5)];
    return legalize_mask((word >> (k0 & 31)) & ((1u << M) - 1u), N, M, filled);
  }
  uint32_t key[16];
  for (int i = 0; i < M; ++i) key[i] = saliency_key(W[o * ldw + g * M + i]);
  return select_top_n_rt(key, N, M);
}

// j-th set bit of km (0-based)
__device__ inline int nth_set(uint32_t km, int j) {
  for (int i = 0; i < 16; ++i)
    if ((km >> i) & 1u) { if (j == 0) return i; --j; }
  return 0;
}

__global__ void pack_values_general_kernel(const bf16_t* __restrict__ W, int64_t O, int64_t K, int64_t ldw, int N, int M,
                                           const uint32_t* __restrict__ mask_in, bf16_t* __restrict__ values,
                                           const uint8_t* __restrict__ rank_in) {
  const int64_t G = K / M;
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= O * G) return;
  const int64_t o = id / G, g = id % G;
  uint32_t filled;
  const uint32_t km = group_keep(W, ldw, mask_in, K, o, g, N, M, &filled, rank_in);
  int j = 0;
  for (int i = 0; i < M; ++i)
    if ((km >> i) & 1u) {
      values[o * (G * N) + g * N + j] = ((filled >> i) & 1u) ? (bf16_t)0 : W[o * ldw + g * M + i];
      ++j;
    }
}

__global__ void pack_index_general_kernel(const bf16_t* __restrict__ W, int64_t O, int64_t K, int64_t ldw, int N, int M,
                                          const uint32_t* __restrict__ mask_in, uint32_t* __restrict__ indices,
                                          const uint8_t* __restrict__ rank_in) {
  const int b = log2_of(M);
  const int64_t nf = K / M * N;
  const int64_t nw = (nf * b + 31) / 32;
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= O * nw) return;
  const int64_t o = id / nw, w = id % nw;
  const int64_t bit0 = w * 32;
  int64_t f_lo = bit0 / b;
  int64_t f_hi = (bit0 + 31) / b;
  if (f_hi > nf - 1) f_hi = nf - 1;
  uint32_t word = 0;
  int64_t g_cached = -1;
  uint32_t km = 0, filled;
  for (int64_t f = f_lo; f <= f_hi; ++f) {
    const int64_t g = f / N;
    if (g != g_cached) { km = group_keep(W, ldw, mask_in, K, o, g, N, M, &filled, rank_in); g_cached = g; }
    const uint64_t p = (uint64_t)nth_set(km, (int)(f % N));
    const int64_t off = f * b - bit0;  // may be negative for a field that started in the previous word
    word |= off >= 0 ? (uint32_t)(p << off) : (uint32_t)(p >> (-off));
  }
  indices[o * nw + w] = word;
}

__global__ void prune_general_kernel(const bf16_t* W, int64_t O, int64_t K, int64_t ldw, int N, int M,
                                     uint32_t* __restrict__ mask_out, bf16_t* w_masked) {
  const int64_t nw = mask_words_per_row(K);
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= O * nw) return;
  const int64_t o = id / nw, w = id % nw;
  uint32_t word = 0;
  for (int64_t k0 = w * 32; k0 < w * 32 + 32 && k0 < K; k0 += M) {
    uint32_t filled;
    const uint32_t km = group_keep(W, ldw, nullptr, K, o, k0 / M, N, M, &filled);
    word |= km << (k0 & 31);
    if (w_masked)
      for (int i = 0; i < M; ++i) w_masked[o * ldw + k0 + i] = ((km >> i) & 1u) ? W[o * ldw + k0 + i] : (bf16_t)0;
  }
  mask_out[o * nw + w] = word;
}

// thread per group; VEC: 16-byte stores of whole 8-weight runs (needs ldw % 8 == 0 and an aligned base)
template <bool VEC>
__global__ void unpack_kernel(const bf16_t* __restrict__ values, const uint32_t* __restrict__ indices, int64_t O,
                              int64_t K, int N, int M, bf16_t* __restrict__ Wd, int64_t ldw) {
  const int b = log2_of(M);
  const int64_t G = K / M;
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= O * G) return;
  const int64_t o = id / G, g = id % G;
  const int64_t nf = G * N;
  const int64_t nw = (nf * b + 31) / 32;
  const uint32_t* row = indices + o * nw;
  uint32_t out[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) out[i] = 0;
  for (int j = 0; j < N; ++j) {
    const int64_t f = g * N + j;
    const uint32_t p = stream_bits(row, nw, f * b, b);
    const uint32_t v = values[o * nf + f];
#pragma unroll
    for (int i = 0; i < 16; ++i) out[i] = (p == (uint32_t)i) ? v : out[i];
  }
  bf16_t* dst = Wd + o * ldw + g * M;
  if (VEC && M >= 8) {
    *reinterpret_cast<uint4*>(dst) = make_uint4(out[0] | (out[1] << 16), out[2] | (out[3] << 16),
                                                out[4] | (out[5] << 16), out[6] | (out[7] << 16));
    if (M == 16)
      *reinterpret_cast<uint4*>(dst + 8) = make_uint4(out[8] | (out[9] << 16), out[10] | (out[11] << 16),
                                                      out[12] | (out[13] << 16), out[14] | (out[15] << 16));
  } else if (VEC && M == 4) {
    *reinterpret_cast<uint2*>(dst) = make_uint2(out[0] | (out[1] << 16), out[2] | (out[3] << 16));
  } else {
    for (int i = 0; i < M; ++i) dst[i] = (bf16_t)out[i];
  }
}

__global__ void fill_u32_kernel(uint32_t* p, uint32_t v) { *p = v; }

__global__ void mask_check_kernel(const uint32_t* __restrict__ mask, int64_t O, int64_t K, int N, int M,
                                  uint32_t* __restrict__ bad) {
  const int64_t G = K / M;
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  bool is_bad = false;
  if (id < O * G) {
    const int64_t o = id / G, k0 = (id % G) * M;
    const uint32_t word = mask[o * mask_words_per_row(K) + (k0 >> 5)];
    is_bad = __popc((word >> (k0 & 31)) & ((1u << M) - 1u)) != N;
  }
  const unsigned long long ballot = __ballot(is_bad);
  if ((threadIdx.x & 63) == 0 && ballot) {
    const uint32_t n = (uint32_t)__popcll(ballot);
    const uint32_t old = atomicAdd(bad, n);
    if (old + n < old) atomicExch(bad, 0xFFFFFFFFu);  // saturate
  }
}

// ---------------------------------------------------------------------------------------------
// Host-side launchers
// ---------------------------------------------------------------------------------------------
static inline unsigned blocks_for(int64_t n, int per) { return (unsigned)((n + per - 1) / per); }

static bool flat_ok(int64_t O, int64_t K, int64_t ldw, int N, int M, const void* a, const void* b, const void* c,
                    const void* d, const void* e) {
  if (ldw != K || (K % 32) != 0) return false;
  if ((values_per_row(K, N, M) * log2_of(M)) % 32 != 0) return false;
  if ((O * K / kChunk + kBlockChunks - 1) / kBlockChunks > 0x7FFFFFFF) return false;
  const uintptr_t all = (uintptr_t)a | (uintptr_t)b | (uintptr_t)c | (uintptr_t)d | (uintptr_t)e;
  return (all & 15u) == 0;
}

template <int SRC>
static bool launch_flat(int N, int M, dim3 grid, hipStream_t s, const bf16_t* W, int64_t n_chunks, const uint32_t* mask_in,
                        bf16_t* values, uint32_t* indices, uint32_t* mask_out, bf16_t* w_masked) {
  switch (N * 32 + M) {
#define X(n, mm)                                                                                                  \
  case n * 32 + mm:                                                                                               \
    hipLaunchKernelGGL((code_flat_kernel<n, mm, SRC>), grid, dim3(kPackThreads), 0, s, W, n_chunks, mask_in, values, \
                       indices, mask_out, w_masked);                                                              \
    return true;
    NM_FOR_EACH_LEVEL(X)
#undef X
    default: return false;
  }
}

hipError_t launch_prune(const bf16_t* W, int64_t O, int64_t K, int64_t ldw, int N, int M, uint32_t* mask,
                        bf16_t* w_masked, hipStream_t s) {
  if (flat_ok(O, K, ldw, N, M, W, mask, w_masked, nullptr, nullptr)) {
    const int64_t n_chunks = O * K / kChunk;
    launch_flat<0>(N, M, dim3(blocks_for(n_chunks, kBlockChunks)), s, W, n_chunks, nullptr, nullptr, nullptr, mask,
                       w_masked);
  } else {
    const int64_t n = O * mask_words_per_row(K);
    hipLaunchKernelGGL(prune_general_kernel, dim3(blocks_for(n, 256)), dim3(256), 0, s, W, O, K, ldw, N, M, mask,
                       w_masked);
  }
  return hipGetLastError();
}

hipError_t launch_pack(const bf16_t* W, int64_t O, int64_t K, int64_t ldw, int N, int M, const uint32_t* mask,
                       bf16_t* values, uint32_t* indices, hipStream_t s) {
  if (flat_ok(O, K, ldw, N, M, W, mask, values, indices, nullptr)) {
    const int64_t n_chunks = O * K / kChunk;
    const dim3 grid(blocks_for(n_chunks, kBlockChunks));
    if (mask) launch_flat<1>(N, M, grid, s, W, n_chunks, mask, values, indices, nullptr, nullptr);
    else launch_flat<0>(N, M, grid, s, W, n_chunks, nullptr, values, indices, nullptr, nullptr);
  } else {
    const int64_t ng = O * (K / M);
    hipLaunchKernelGGL(pack_values_general_kernel, dim3(blocks_for(ng, 256)), dim3(256), 0, s, W, O, K, ldw, N, M,
                       mask, values, (const uint8_t*)nullptr);
    const int64_t nw = O * index_words_per_row(K, N, M);
    hipLaunchKernelGGL(pack_index_general_kernel, dim3(blocks_for(nw, 256)), dim3(256), 0, s, W, O, K, ldw, N, M, mask,
                       indices, (const uint8_t*)nullptr);
  }
  return hipGetLastError();
}

// nm_pack with the selection read from stored ranks (kept = rank < N)
hipError_t launch_pack_ranked(const bf16_t* W, const uint8_t* rank, int64_t O, int64_t K, int64_t ldw, int N, int M,
                              bf16_t* values, uint32_t* indices, hipStream_t s) {
  if (flat_ok(O, K, ldw, N, M, W, rank, values, indices, nullptr)) {
    const int64_t n_chunks = O * K / kChunk;
    launch_flat<2>(N, M, dim3(blocks_for(n_chunks, kBlockChunks)), s, W, n_chunks,
                   reinterpret_cast<const uint32_t*>(rank), values, indices, nullptr, nullptr);
  } else {
    const int64_t ng = O * (K / M);
    hipLaunchKernelGGL(pack_values_general_kernel, dim3(blocks_for(ng, 256)), dim3(256), 0, s, W, O, K, ldw, N, M,
                       (const uint32_t*)nullptr, values, rank);
    const int64_t nw = O * index_words_per_row(K, N, M);
    hipLaunchKernelGGL(pack_index_general_kernel, dim3(blocks_for(nw, 256)), dim3(256), 0, s, W, O, K, ldw, N, M,
                       (const uint32_t*)nullptr, indices, rank);
  }
  return hipGetLastError();
}

static bool batch_level(int N, int M) {
  switch (N * 32 + M) {
#define X(n, mm) case n * 32 + mm: return true;
    NM_FOR_EACH_BATCH_LEVEL(X)
#undef X
    default: return false;
  }
}

hipError_t launch_pack_batched(const PackDesc* descs, int count, hipStream_t s) {
  BatchArgs args;
  args.count = 0;
  uint64_t blocks = 0;
  auto flush = [&]() {
    if (args.count) {
      hipLaunchKernelGGL(pack_batched_kernel<0>, dim3((unsigned)blocks), dim3(kPackThreads), 0, s, args);
      args.count = 0;
      blocks = 0;
    }
  };
  for (int i = 0; i < count; ++i) {
    const PackDesc& d = descs[i];
    const bool flat = batch_level(d.N, d.M) && flat_ok(d.O, d.K, d.K, d.N, d.M, d.W, d.values, d.indices, nullptr, nullptr);
    if (!flat) {
      hipError_t e = launch_pack(d.W, d.O, d.K, d.K, d.N, d.M, nullptr, d.values, d.indices, s);
      if (e != hipSuccess) return e;
      continue;
    }
    const int64_t n_chunks = d.O * d.K / kChunk;
    const uint64_t nb = blocks_for(n_chunks, kBlockChunks);
    if (args.count == kBatchMax || blocks + nb > 0x7FFFFFFFull) flush();
    BatchEntry& e = args.e[args.count++];
    e.W = d.W; e.values = d.values; e.indices = d.indices; e.n_chunks = n_chunks;
    e.stream_ws = nullptr; e.rank = nullptr; e.K = d.K;
    blocks += nb;
    e.block_end = (uint32_t)blocks;
    e.N = (uint16_t)d.N; e.M = (uint16_t)d.M;
  }
  flush();
  return hipGetLastError();
}

// nm_pack_ranked for many matrices: one launch for those the fast kernel takes, own launches for the rest
hipError_t launch_pack_ranked_batched(const PackRankedDesc* descs, int count, hipStream_t s) {
  BatchArgs args;
  args.count = 0;
  uint64_t blocks = 0;
  auto flush = [&]() {
    if (args.count) {
      hipLaunchKernelGGL(pack_batched_kernel<2>, dim3((unsigned)blocks), dim3(kPackThreads), 0, s, args);
      args.count = 0;
      blocks = 0;
    }
  };
  for (int i = 0; i < count; ++i) {
    const PackRankedDesc& d = descs[i];
    if (!(batch_level(d.N, d.M) && flat_ok(d.O, d.K, d.K, d.N, d.M, d.W, d.rank, d.values, d.indices, nullptr))) {
      hipError_t e = launch_pack_ranked(d.W, d.rank, d.O, d.K, d.K, d.N, d.M, d.values, d.indices, s);
      if (e != hipSuccess) return e;
      continue;
    }
    const int64_t n_chunks = d.O * d.K / kChunk;
    const uint64_t nb = blocks_for(n_chunks, kBlockChunks);
    if (args.count == kBatchMax || blocks + nb > 0x7FFFFFFFull) flush();
    BatchEntry& e = args.e[args.count++];
    e.W = d.W; e.values = d.values; e.indices = d.indices; e.n_chunks = n_chunks;
    e.stream_ws = nullptr; e.rank = reinterpret_cast<const uint32_t*>(d.rank); e.K = d.K;
    blocks += nb;
    e.block_end = (uint32_t)blocks;
    e.N = (uint16_t)d.N; e.M = (uint16_t)d.M;
  }
  flush();
  return hipGetLastError();
}

// nm_pack(mask = NULL) + nm_spmm_prepare for many layers.  A layer whose product reads stream order and whose
// rows fill whole 256-row tiles gets both forms from the one batched launch; any other layer is packed in the
// batch (or alone) and prepared by its own pre-pass afterwards.
hipError_t launch_pack_prepare_batched(const LayerDesc* descs, int count, hipStream_t s, bool* workspace_short) {
  *workspace_short = false;
  for (int i = 0; i < count; ++i) {
    const LayerDesc& d = descs[i];
    const size_t need = spmm_operand_workspace_bytes(d.O, d.K, d.N, d.M, d.T);
    if (need && (d.workspace == nullptr || d.workspace_bytes < need || ((uintptr_t)d.workspace & 255u))) {
      *workspace_short = true;
      return hipSuccess;
    }
  }
  BatchArgs args;
  args.count = 0;
  uint64_t blocks = 0;
  auto flush = [&]() {
    if (args.count) {
      hipLaunchKernelGGL(pack_batched_kernel<0>, dim3((unsigned)blocks), dim3(kPackThreads), 0, s, args);
      args.count = 0;
      blocks = 0;
    }
  };
  for (int i = 0; i < count; ++i) {
    const LayerDesc& d = descs[i];
    const bool flat = batch_level(d.N, d.M) && flat_ok(d.O, d.K, d.K, d.N, d.M, d.W, d.values, d.indices, nullptr, nullptr);
    bool sparse_form = false;
    const bool fused = flat && spmm_stream_order(d.O, d.K, d.T, d.N, d.M, &sparse_form) && (d.O % 256) == 0;
    if (flat) {
      const int64_t n_chunks = d.O * d.K / kChunk;
      const uint64_t nb = blocks_for(n_chunks, kBlockChunks);
      if (args.count == kBatchMax || blocks + nb > 0x7FFFFFFFull) flush();
      BatchEntry& e = args.e[args.count++];
      e.W = d.W; e.values = d.values; e.indices = d.indices; e.n_chunks = n_chunks;
      e.stream_ws = fused ? reinterpret_cast<unsigned char*>(d.workspace) : nullptr;
      e.rank = nullptr;
      e.K = d.K;
      blocks += nb;
      e.block_end = (uint32_t)blocks;
      e.N = (uint16_t)d.N; e.M = (uint16_t)d.M;
    } else {
      hipError_t e = launch_pack(d.W, d.O, d.K, d.K, d.N, d.M, nullptr, d.values, d.indices, s);
      if (e != hipSuccess) return e;
    }
  }
  flush();
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  for (int i = 0; i < count; ++i) {
    const LayerDesc& d = descs[i];
    const bool flat = batch_level(d.N, d.M) && flat_ok(d.O, d.K, d.K, d.N, d.M, d.W, d.values, d.indices, nullptr, nullptr);
    bool sparse_form = false;
    if (flat && spmm_stream_order(d.O, d.K, d.T, d.N, d.M, &sparse_form) && (d.O % 256) == 0) continue;
    SpmmArgs a;
    a.values = d.values; a.indices = d.indices; a.O = d.O; a.K = d.K; a.N = d.N; a.M = d.M;
    a.X = nullptr; a.T = d.T; a.ldx = d.K; a.bias = nullptr; a.Y = nullptr; a.ldy = d.O; a.out_bf16 = 0;
    a.workspace = d.workspace; a.workspace_bytes = d.workspace_bytes;
    bool ws_short = false;
    if ((e = launch_spmm(a, s, &ws_short, SPMM_PREPARE)) != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_unpack(const bf16_t* values, const uint32_t* indices, int64_t O, int64_t K, int N, int M,
                         bf16_t* Wd, int64_t ldw, hipStream_t s) {
  const int64_t ng = O * (K / M);
  const bool vec = (ldw % 8 == 0) && (((uintptr_t)Wd & 15u) == 0);
  if (vec) hipLaunchKernelGGL(unpack_kernel<true>, dim3(blocks_for(ng, 256)), dim3(256), 0, s, values, indices, O, K, N, M, Wd, ldw);
  else hipLaunchKernelGGL(unpack_kernel<false>, dim3(blocks_for(ng, 256)), dim3(256), 0, s, values, indices, O, K, N, M, Wd, ldw);
  return hipGetLastError();
}

hipError_t launch_mask_check(const uint32_t* mask, int64_t O, int64_t K, int N, int M, uint32_t* bad, hipStream_t s) {
  hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(1), 0, s, bad, 0u);
  const int64_t ng = O * (K / M);
  hipLaunchKernelGGL(mask_check_kernel, dim3(blocks_for(ng, 256)), dim3(256), 0, s, mask, O, K, N, M, bad);
  return hipGetLastError();
}

}  // namespace nm
