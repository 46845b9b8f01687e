// Sparse-weight x dense-activation product for few tokens (T <= 208: a batch of one image, Section 4's latency
// setting), straight from the packed format of Section 1 / Fig. 2 (upper part): kept values + log2(M)-bit
// positions.  The weight is read once, in its packed form, and decoded in registers into matrix-core operands
// (Fig. 2, lower part: the positions select the activations); there is no operand-order copy and no workspace.
// It is the path of a product call that comes WITHOUT a workspace: with one, the tiled kernel of nm_spmm.hip reads
// the operand-order copy and is the faster of the two (measured on the 48 linears of the model at 197 tokens:
// 73 us against 89 us here; this kernel reads 112 MB where the other reads 170 MB, but its windows are bound by
// the LDS traffic of the activation fragments, a kilobyte per matrix instruction).
//
// Work item = 128 out-features of one layer over the whole reduction, all tokens: one block of 8 waves per compute
// unit; wave (rw, th) owns 32 out-features (two 16-row blocks) x one half of the 13 token blocks of 16.  Items are
// listed deepest reduction first and the hardware hands them to compute units as blocks retire.
// Everything a window of 64 reduction positions needs arrives in LDS through asynchronous copies, counted exactly:
//   X[all tokens, 64 k]: a ring of 3 buffers (swizzled against bank conflicts), two windows ahead;
//   the packed 16-position chunk every lane owns for a 16-row block (2 .. 16 bytes of values and the 32-bit words
//   that hold its index fields), gathered lane by lane: a ring of 4, three windows ahead of its use, which covers
//   the latency of the one pass over the weight in HBM.
// A lane then reads its chunk back, decodes it to the 2:4 operand of v_smfmac_f32_16x16x64_bf16 (levels with
// N <= 2: any such group has at most two kept weights per run of four) or to a zero-filled dense operand of
// v_mfma_f32_16x16x32_bf16 (N = 4), and multiplies it with the token blocks of its half.
#include "nm_launch.h"
#include "nm_mma.h"

namespace nm {
namespace {

constexpr int kTB = 13;                  // token blocks of 16
constexpr int kTokens = kTB * 16;        // 208
constexpr int kTBW = 7;                  // token blocks of a wave (the second half has 6)
constexpr int kRows = 128;               // out-features per block
constexpr int kWaves = 8;
constexpr int kXLoads = 4;               // per wave and window: 32 copies of 8 token rows x 128 bytes
constexpr int kXStage = kXLoads * kWaves * 1024;  // 256 rows of 128 bytes
constexpr int kXRing = 3, kARing = 4;
constexpr int kASlice = 1024 + 2 * 256;  // one 16-row block of one window: values, two index words per lane
constexpr int kAStage = 8 * kASlice;     // eight 16-row blocks
constexpr int kA0 = kXRing * kXStage;
constexpr int kLdsBytes = kA0 + kARing * kAStage;
static_assert(kLdsBytes <= 160 * 1024, "LDS budget");
constexpr int kLayersMax = 52;

struct FtLayer {
  const bf16_t* values;
  const uint32_t* indices;
  const bf16_t* X;
  const float* bias;  // nullable
  void* Y;
  int32_t O, K, ldx, ldy, T;
  int32_t level;       // index into the level list below
  int32_t out_kind;    // bit 0: bfloat16 output; bit 1: rows of Y are not made of aligned 8- / 16-byte pieces
};
struct FtGroup {
  int32_t count, n_items;
  int32_t first_item[kLayersMax];  // items of the layers before each one (ascending)
  FtLayer layer[kLayersMax];
};
static_assert(sizeof(FtGroup) <= 4096, "the table must fit the kernel argument segment");

// the levels this kernel decodes: the set a layer-wise configuration draws from, without 2:4 (whose packed layout
// the tiled kernel reads as it is, so a 2:4 layer never needs a workspace)
constexpr int kLevels = 7;
__host__ __device__ constexpr int level_n(int code) { return code == 0 ? 1 : code == 1 ? 1 : code == 2 ? 2 : code == 3 ? 4 : code == 4 ? 1 : code == 5 ? 2 : 4; }
__host__ __device__ constexpr int level_m(int code) { return code < 1 ? 4 : code < 4 ? 8 : 16; }
int level_code(int N, int M) {
  for (int c = 0; c < kLevels; ++c)
    if (level_n(c) == N && level_m(c) == M) return c;
  return -1;
}

// What a lane holds of one packed 16-position chunk of one row: the raw value bytes and the 32-bit window(s) of the
// row's index stream that contain the chunk's fields.
template <int N, int M>
struct Chunk {
  static constexpr int B = log2_of(M);
  static constexpr int VPC = 16 * N / M;   // kept values per chunk
  static constexpr int VBYTES = VPC * 2;
  static constexpr int IBITS = VPC * B;
  static constexpr bool STRADDLE = (32 % IBITS) != 0;  // a chunk's fields may cross a word boundary
  static constexpr bool SPARSE = N <= 2;
  uint32_t v[VBYTES >= 4 ? VBYTES / 4 : 1];
  uint32_t w0, w1;

  // Copies of one chunk per lane into a slice of LDS: values at lane * 16 (16 bytes), or dword d at d * 256 + lane * 4;
  // index words at 1024 + lane * 4 and 1280 + lane * 4.  DMAS = copies issued.
  static constexpr int VD = VBYTES == 16 ? 1 : (VBYTES == 8 ? 2 : 1);
  static constexpr int DMAS = VD + (STRADDLE ? 2 : 1);
  __device__ __forceinline__ static void issue(uniform_ptr_t values, uniform_ptr_t indices, uint32_t vrow_off,
                                               uint32_t irow_off, int chunk, int last_word, uint32_t slice) {
    if constexpr (VBYTES == 16) {
      dma16_at(values, vrow_off + (uint32_t)chunk * 16u, slice, 0u);
    } else if constexpr (VBYTES == 8) {
      dma4_at(values, vrow_off + (uint32_t)chunk * 8u, slice, 0u);
      dma4_at(values, vrow_off + (uint32_t)chunk * 8u + 4u, slice, 256u);
    } else if constexpr (VBYTES == 4) {
      dma4_at(values, vrow_off + (uint32_t)chunk * 4u, slice, 0u);
    } else {
      dma4_at(values, vrow_off + (uint32_t)(chunk >> 1) * 4u, slice, 0u);  // the aligned word that holds the value
    }
    const int word = (chunk * IBITS) >> 5;
    dma4_at(indices, irow_off + (uint32_t)word * 4u, slice, 1024u);
    if constexpr (STRADDLE)
      dma4_at(indices, irow_off + (uint32_t)(word + 1 <= last_word ? word + 1 : last_word) * 4u, slice, 1280u);
  }
  __device__ __forceinline__ void fill(const unsigned char* slice, int lane, int chunk) {
    if constexpr (VBYTES == 16) {
      const u32x4_t t = *reinterpret_cast<const u32x4_t*>(slice + lane * 16);
      v[0] = t[0]; v[1] = t[1]; v[2] = t[2]; v[3] = t[3];
    } else if constexpr (VBYTES == 8) {
      v[0] = *reinterpret_cast<const uint32_t*>(slice + lane * 4);
      v[1] = *reinterpret_cast<const uint32_t*>(slice + 256 + lane * 4);
    } else if constexpr (VBYTES == 4) {
      v[0] = *reinterpret_cast<const uint32_t*>(slice + lane * 4);
    } else {
      v[0] = (*reinterpret_cast<const uint32_t*>(slice + lane * 4) >> (16 * (chunk & 1))) & 0xFFFFu;
    }
    w0 = *reinterpret_cast<const uint32_t*>(slice + 1024 + lane * 4);
    w1 = 0;
    if constexpr (STRADDLE) w1 = *reinterpret_cast<const uint32_t*>(slice + 1280 + lane * 4);
  }
  // the chunk's index fields, field 0 in the low bits
  __device__ __forceinline__ uint32_t fields(int chunk) const {
    const int sh = (chunk * IBITS) & 31;
    if constexpr (STRADDLE) return (uint32_t)((((uint64_t)w1 << 32) | w0) >> sh);
    else return w0 >> sh;
  }
  __device__ __forceinline__ uint32_t value(int f) const { return (v[f / 2] >> (16 * (f & 1))) & 0xFFFFu; }

  // 2:4 operand: per run of four positions two 16-bit slots (kept weights in ascending position, zero-filled) and
  // four selector bits (2-bit positions inside the run)
  __device__ __forceinline__ void sparse_operand(int chunk, u32x4_t& a, uint32_t& sel) const {
    const uint32_t fld = fields(chunk);
    constexpr int G = 16 / M, RUNS = M / 4;
    uint32_t piece[4] = {0u, 0u, 0u, 0u};
    sel = 0;
#pragma unroll
    for (int g = 0; g < G; ++g) {
      uint32_t prev_run = 0xFFFFFFFFu;
#pragma unroll
      for (int j = 0; j < N; ++j) {
        const int f = g * N + j;
        const uint32_t pos = (fld >> (B * f)) & (uint32_t)(M - 1);
        const uint32_t run = pos >> 2, within = pos & 3u;
        const uint32_t second = (j > 0 && run == prev_run) ? 1u : 0u;
        prev_run = run;
        const uint32_t val = value(f) << (16 * second);
        if constexpr (RUNS == 1) {
          piece[g] |= val;
        } else {
#pragma unroll
          for (int r = 0; r < RUNS; ++r) piece[g * RUNS + r] |= (run == (uint32_t)r) ? val : 0u;
        }
        sel |= within << (4 * ((uint32_t)(g * RUNS) + run) + 2 * second);
      }
    }
    a = u32x4_t{piece[0], piece[1], piece[2], piece[3]};
  }
  // dense operand: the 16 positions with zeros in the pruned places; lo = positions 0..7, hi = 8..15
  __device__ __forceinline__ void dense_operand(int chunk, u32x4_t& lo, u32x4_t& hi) const {
    const uint32_t fld = fields(chunk);
    uint32_t d[8] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};
    constexpr int G = 16 / M;
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
      for (int j = 0; j < N; ++j) {
        const int f = g * N + j;
        const uint32_t pos = (fld >> (B * f)) & (uint32_t)(M - 1);
        const uint32_t val = value(f) << (16 * (pos & 1u));
        const uint32_t reg = pos >> 1;  // inside the group
#pragma unroll
        for (int r = 0; r < M / 2; ++r) d[g * (M / 2) + r] |= (reg == (uint32_t)r) ? val : 0u;
      }
    }
    lo = u32x4_t{d[0], d[1], d[2], d[3]};
    hi = u32x4_t{d[4], d[5], d[6], d[7]};
  }
};

// swizzle of the 16-byte pieces of a 128-byte token row in LDS: any 8 consecutive rows, and the 8 even (odd) ones
// of 16 consecutive rows, put a given piece into 8 different slots
__device__ __forceinline__ int row_key(int row) { return (row & 7) ^ ((row >> 3) & 1); }

template <int N, int M>
__device__ __forceinline__ void fewtok_item(const FtLayer& L, int row_group, unsigned char* smem, uint32_t lds0) {
  using C = Chunk<N, M>;
  constexpr bool SPARSE = C::SPARSE;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int rw = wave & 3, th = wave >> 2;  // 32-row group, token half
  const int t16 = lane & 15, kb = lane >> 4;
  const int O = L.O, K = L.K, T = L.T;
  const int nw = K >> 6;  // windows
  const int o0 = row_group * kRows + rw * 32;

  // ---- X copies: this wave brings token rows 8 q .. 8 q + 7 for q = wave, wave + 8, ... (rows past T repeat the
  // last one: their outputs are never stored)
  uint32_t x_voff[kXLoads];
#pragma unroll
  for (int n = 0; n < kXLoads; ++n) {
    const int row = 8 * (wave + kWaves * n) + (lane >> 3);
    const int src = row < T ? row : T - 1;
    x_voff[n] = (uint32_t)((int64_t)src * L.ldx * 2 + (((lane & 7) ^ row_key(row)) * 16));
  }
  const unsigned char* xk = reinterpret_cast<const unsigned char*>(L.X);
  auto issue_x = [&](int window) {
    const int wc = window < nw ? window : nw - 1;  // past the end: the last window again, into a buffer nobody reads
    const uniform_ptr_t base = make_uniform(xk + (int64_t)wc * 128);
    const uint32_t stage = __builtin_amdgcn_readfirstlane(lds0 + (uint32_t)((window % kXRing) * kXStage));
#pragma unroll
    for (int n = 0; n < kXLoads; ++n) dma16_at(base, x_voff[n], stage, (uint32_t)((wave + kWaves * n) * 1024));
  };

  // ---- weight copies: this wave brings the chunks of 16-row block th of its row group (the other wave of the pair
  // brings the other block); rows past O repeat the last one and are never stored
  const uint32_t vrow_bytes = (uint32_t)(K / M * N * 2);
  const int iwords = (K / M * N * C::B + 31) / 32;
  uint32_t vrow_off, irow_off;
  {
    const int r = o0 + 16 * th + t16;
    const int row = r < O ? r : O - 1;
    vrow_off = (uint32_t)row * vrow_bytes;
    irow_off = (uint32_t)row * (uint32_t)iwords * 4u;
  }
  const uniform_ptr_t vbase = make_uniform(L.values), ibase = make_uniform(L.indices);
  auto issue_a = [&](int window) {
    const int wc = window < nw ? window : nw - 1;
    const uint32_t slice =
        __builtin_amdgcn_readfirstlane(lds0 + (uint32_t)(kA0 + (window % kARing) * kAStage + (rw * 2 + th) * kASlice));
    C::issue(vbase, ibase, vrow_off, irow_off, wc * 4 + kb, iwords - 1, slice);
  };
  constexpr int LW = kXLoads + C::DMAS;  // copies of a wave per window

  // ---- fragment addresses of this lane inside an X buffer: token row t16 of block j is at j * 2048.
  // The sparse instruction pairs the 16 positions of the weight lane (row, kb), 16 kb .. 16 kb + 15, with activation
  // lanes that hold positions 8 kb .. 8 kb + 7 and 32 + 8 kb .. 32 + 8 kb + 7: pieces kb and 4 + kb of the window's
  // row.  The dense instruction pairs lane with lane: pieces 2 kb and 2 kb + 1, the two halves of the lane's chunk.
  const int key = row_key(t16);
  const int p_lo = SPARSE ? kb : 2 * kb, p_hi = SPARSE ? 4 + kb : 2 * kb + 1;
  const uint32_t b_lo = (uint32_t)((th * kTBW * 16 + t16) * 128 + ((p_lo ^ key) * 16));
  const uint32_t b_hi = (uint32_t)((th * kTBW * 16 + t16) * 128 + ((p_hi ^ key) * 16));
  // the second half has 6 token blocks; it multiplies a seventh (rows 208 .. 223 of the buffer, never stored) so that
  // the fragment reads of a window are one straight run the compiler can issue ahead of the matrix instructions

  f32x4_t acc[2][kTBW];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < kTBW; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  // ---- prologue: the copies of the three batches before window 0 (the first X copy of window 0 is issued twice,
  // so that every batch has the same number of copies and the waits below are constants)
  issue_x(0); issue_a(0);
  issue_x(0); issue_a(1);
  issue_x(1); issue_a(2);

  for (int w = 0; w < nw; ++w) {
    // Outstanding, oldest first: [X w-?, A w] [X w, A w+1] [X w+1, A w+2].  This window needs A w and X w: everything
    // but the last A w+1 and the last batch may stay in flight.  After the barrier every wave has finished window
    // w-1, whose buffers the copies below refill.
    wait_loads_outstanding<C::DMAS + LW>();
    __builtin_amdgcn_s_barrier();
    issue_x(w + 2);
    issue_a(w + 3);
    const int chunk = w * 4 + kb;
    u32x4_t a0[2], a1[2];
    uint32_t sel[2] = {0u, 0u};
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      C raw;
      raw.fill(smem + kA0 + (w % kARing) * kAStage + (rw * 2 + i) * kASlice, lane, chunk);
      if constexpr (SPARSE) raw.sparse_operand(chunk, a0[i], sel[i]);
      else raw.dense_operand(chunk, a0[i], a1[i]);
    }
    const unsigned char* xs = smem + (w % kXRing) * kXStage;
#pragma unroll
    for (int j = 0; j < kTBW; ++j) {
      {
        const u32x4_t lo = *reinterpret_cast<const u32x4_t*>(xs + b_lo + j * 2048);
        const u32x4_t hi = *reinterpret_cast<const u32x4_t*>(xs + b_hi + j * 2048);
        if constexpr (SPARSE) {
          const u32x8_t b = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
          for (int i = 0; i < 2; ++i)
            acc[i][j] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(__builtin_bit_cast(bf16x8_t, a0[i]),
                                                                  __builtin_bit_cast(bf16x16_t, b), acc[i][j],
                                                                  (int)sel[i], 0, 0);
        } else {
#pragma unroll
          for (int i = 0; i < 2; ++i) {
            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a0[i]),
                                                                __builtin_bit_cast(bf16x8_t, lo), acc[i][j], 0, 0, 0);
            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a1[i]),
                                                                __builtin_bit_cast(bf16x8_t, hi), acc[i][j], 0, 0, 0);
          }
        }
      }
    }
  }
  // the surplus copies of the last windows: nothing may be in flight into LDS when the block ends
  wait_loads_outstanding<0>();

  // ---- write out: a lane holds out-features o .. o + 3 of token 16 j + t16 for each of its two row blocks
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int o = o0 + 16 * i + 4 * kb;
    if (o >= O) continue;
    f32x4_t b = f32x4_t{0.f, 0.f, 0.f, 0.f};
    if (L.bias != nullptr) b = f32x4_t{L.bias[o], L.bias[o + 1], L.bias[o + 2], L.bias[o + 3]};
    const int kind = L.out_kind;
#pragma unroll
    for (int j = 0; j < kTBW; ++j) {
      const int t = 16 * (th * kTBW + j) + t16;
      if (t >= T) continue;
      const f32x4_t y = acc[i][j] + b;
      uint2 pk;
      pk.x = pack_bf16x2(y[0], y[1]);
      pk.y = pack_bf16x2(y[2], y[3]);
      if (kind == 1) {
        *reinterpret_cast<uint2*>(reinterpret_cast<bf16_t*>(L.Y) + (int64_t)t * L.ldy + o) = pk;
      } else if (kind == 0) {
        *reinterpret_cast<f32x4_t*>(reinterpret_cast<float*>(L.Y) + (int64_t)t * L.ldy + o) = y;
      } else if (kind == 3) {
        bf16_t* dst = reinterpret_cast<bf16_t*>(L.Y) + (int64_t)t * L.ldy + o;
        dst[0] = (bf16_t)(pk.x & 0xFFFFu); dst[1] = (bf16_t)(pk.x >> 16);
        dst[2] = (bf16_t)(pk.y & 0xFFFFu); dst[3] = (bf16_t)(pk.y >> 16);
      } else {
        float* dst = reinterpret_cast<float*>(L.Y) + (int64_t)t * L.ldy + o;
        dst[0] = y[0]; dst[1] = y[1]; dst[2] = y[2]; dst[3] = y[3];
      }
    }
  }
}

__global__ void __launch_bounds__(kWaves * 64) nm_fewtok_kernel(const FtGroup g) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;
  const int item = (int)blockIdx.x;
  // the layer of this item: the prefix table sits in the argument segment next to itself, so the search is a few
  // wide scalar loads and compares, not a chain of dependent loads
  int l = 0;
#pragma unroll
  for (int i = 1; i < kLayersMax; ++i) l += (i < g.count && item >= g.first_item[i]) ? 1 : 0;
  const FtLayer& L = g.layer[l];
  const int row_group = item - g.first_item[l];
  switch (L.level) {
    case 0: fewtok_item<level_n(0), level_m(0)>(L, row_group, smem, lds0); break;
    case 1: fewtok_item<level_n(1), level_m(1)>(L, row_group, smem, lds0); break;
    case 2: fewtok_item<level_n(2), level_m(2)>(L, row_group, smem, lds0); break;
    case 3: fewtok_item<level_n(3), level_m(3)>(L, row_group, smem, lds0); break;
    case 4: fewtok_item<level_n(4), level_m(4)>(L, row_group, smem, lds0); break;
    case 5: fewtok_item<level_n(5), level_m(5)>(L, row_group, smem, lds0); break;
    default: fewtok_item<level_n(6), level_m(6)>(L, row_group, smem, lds0); break;
  }
}

inline bool aligned_to(const void* p, uintptr_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

}  // namespace

// Shapes the few-token kernel takes (the workspace and operand-form decisions depend on the shape alone).
bool fewtok_shape(int64_t O, int64_t K, int N, int M, int64_t T) {
  // per-lane byte offsets into the packed rows are 32-bit
  return T >= 1 && T <= kTokens && level_code(N, M) >= 0 && K % 64 == 0 && K <= (1 << 22) && O % 4 == 0 &&
         O <= (1 << 24) && O * K / M * N * 2 < (1ll << 32);
}

// ... and the operands: 16-byte aligned rows of X and of the packed values (any output alignment).
bool fewtok_takes(const SpmmArgs& a) {
  if (!fewtok_shape(a.O, a.K, a.N, a.M, a.T)) return false;
  if (!aligned_to(a.X, 16) || (a.ldx % 8) || a.ldx > (1 << 22)) return false;
  if (!aligned_to(a.values, 16) || !aligned_to(a.indices, 4)) return false;
  if (a.ldy > 0x7FFFFFFF) return false;
  return true;
}

// The products of `count` layers (each accepted by fewtok_takes), in as few launches as the table allows.
hipError_t launch_fewtok(const SpmmArgs* const* layers, int count, hipStream_t s) {
  static PerDeviceOnce lds_limit;
  if (hipError_t e = raise_dynamic_lds_limit(nm_fewtok_kernel, kLdsBytes, lds_limit); e != hipSuccess) return e;
  // deepest reductions first: the blocks of a launch start in this order, so the longest items start first and the
  // short ones fill in behind them
  int order[kLayersMax];
  for (int first = 0; first < count; first += kLayersMax) {
    const int n = count - first < kLayersMax ? count - first : kLayersMax;
    for (int i = 0; i < n; ++i) {
      int j = i;
      const int64_t cost = layers[first + i]->K * (layers[first + i]->N > 2 ? 2 : 1);
      for (; j > 0; --j) {
        const SpmmArgs& p = *layers[first + order[j - 1]];
        if (p.K * (p.N > 2 ? 2 : 1) >= cost) break;
        order[j] = order[j - 1];
      }
      order[j] = i;
    }
    FtGroup grp;
    grp.count = n;
    int64_t items = 0;
    for (int i = 0; i < n; ++i) {
      const SpmmArgs& a = *layers[first + order[i]];
      FtLayer& L = grp.layer[i];
      L.values = a.values; L.indices = a.indices; L.X = a.X; L.bias = a.bias; L.Y = a.Y;
      L.O = (int32_t)a.O; L.K = (int32_t)a.K; L.ldx = (int32_t)a.ldx; L.ldy = (int32_t)a.ldy; L.T = (int32_t)a.T;
      L.level = level_code(a.N, a.M);
      grp.first_item[i] = (int32_t)items;
      const bool pieces = (a.ldy % 4 == 0) && aligned_to(a.Y, a.out_bf16 ? 8 : 16);
      L.out_kind = (a.out_bf16 ? 1 : 0) | (pieces ? 0 : 2);
      items += (a.O + kRows - 1) / kRows;
      if (items > 0x7FFFFFF0) return hipErrorInvalidValue;
    }
    for (int i = n; i < kLayersMax; ++i) grp.first_item[i] = 0x7FFFFFFF;
    grp.n_items = (int32_t)items;
    hipLaunchKernelGGL(nm_fewtok_kernel, dim3((unsigned)items), dim3(kWaves * 64), kLdsBytes, s, grp);
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace nm
