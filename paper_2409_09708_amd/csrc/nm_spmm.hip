// Sparse-weight x dense-activation product from the packed N:M layout (Section 2, Fig. 2 lower
// part): Y[t, o] = sum_g sum_{j<N} X[t, g*M + idx[o,g,j]] * val[o,g,j], fp32 accumulation.
//
// Two matrix-core formulations on gfx950, W as the first (row) operand so that a lane's four
// accumulators are four consecutive out-features of one token (contiguous in Y):
//
//  * levels with N <= 2: every aligned run of 4 weights holds at most 2 kept values, which is the
//    pattern v_smfmac_f32_16x16x64_bf16 consumes (8 compressed values + eight 2-bit selectors per
//    lane per instruction).  The packed 2:4 layout already IS that operand order; the other levels
//    are re-coded into it (explicit zeros fill the free slots) by a small pre-pass.  The instruction
//    then performs half of the dense multiply-accumulates.
//  * levels with N > 2 (4:8, 4:16, 3:8, ... and N = M): the packed weight is expanded to a dense
//    zero-filled operand by the pre-pass and multiplied with v_mfma_f32_16x16x32_bf16.
//
// Tiling: a block owns BO x BT outputs; per 64-wide K step the W tile (compressed rows + selector
// words, or dense rows) and the X tile are staged global -> registers -> LDS (two LDS stages, one
// barrier per step); each wave reads its operand fragments with 16-byte LDS reads from rows padded
// to an odd number of 16-byte slots (conflict free) and keeps an (OT*16) x (TT*16) accumulator tile.
// Shapes the tiles cannot take (K % 64 != 0, unaligned pointers) run a plain gather kernel.
#include "nm_device.h"
#include "nm_launch.h"

namespace nm {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) __bf16 bf16x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((ext_vector_type(8))) uint32_t u32x8_t;

// ---------------------------------------------------------------------------------------------
// Pre-pass: re-code an N:M weight with N <= 2 as a 2:4 weight (values [O, K/2], one 32-bit
// selector word per 32 weights).  One lane per 32 consecutive weights.
// Slot rule: run q (4 weights) owns slots 2q and 2q+1; the first kept value of the run goes to
// slot 2q with selector = its offset in the run, a second one to slot 2q+1; free slots hold +0
// with selector 0 (the matrix instruction is a plain multiplexer per slot, so any selector of a
// zero slot is harmless).
// ---------------------------------------------------------------------------------------------
template <int N, int M>
__global__ void __launch_bounds__(256)
recode_to_2of4_kernel(const bf16_t* __restrict__ values, const uint32_t* __restrict__ indices, int64_t O, int64_t K,
                      bf16_t* __restrict__ values24, uint32_t* __restrict__ sel24) {
  constexpr int B = log2_of(M);
  constexpr int G = 32 / M;       // groups per lane
  constexpr int RUNS = M / 4;     // 4-runs per group
  const int64_t per_row = K / 32;
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= O * per_row) return;
  const int64_t o = id / per_row, blk = id % per_row;
  const int64_t nf = K / M * N;
  const int64_t nw = (nf * B + 31) / 32;
  const int64_t f0 = blk * G * N;  // first field of this lane
  const uint32_t fields = stream_bits(indices + o * nw, nw, f0 * B, G * N * B);
  uint32_t out[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) out[i] = 0;
  uint32_t sel = 0;
#pragma unroll
  for (int g = 0; g < G; ++g) {
    uint32_t prev_run = 0xFFFFFFFFu;
#pragma unroll
    for (int j = 0; j < N; ++j) {
      const uint32_t p = (fields >> ((g * N + j) * B)) & (M - 1);
      const uint32_t v = values[o * nf + f0 + g * N + j];
      const uint32_t run = p >> 2, within = p & 3u;
      const uint32_t second = (run == prev_run) ? 1u : 0u;
      prev_run = run;
#pragma unroll
      for (int r = 0; r < RUNS; ++r) out[g * RUNS + r] |= (run == (uint32_t)r) ? (v << (16 * second)) : 0u;
      sel |= within << (4 * (g * RUNS + run) + 2 * second);
    }
  }
  uint4* dst = reinterpret_cast<uint4*>(values24 + o * (K / 2) + blk * 16);
  dst[0] = make_uint4(out[0], out[1], out[2], out[3]);
  dst[1] = make_uint4(out[4], out[5], out[6], out[7]);
  sel24[o * per_row + blk] = sel;
}

// ---------------------------------------------------------------------------------------------
// Tiled matrix-core product.
// ---------------------------------------------------------------------------------------------
struct GemmArgs {
  const bf16_t* A;      // SPARSE: compressed values [O, K/2]; dense: W_s [O, K]
  const uint32_t* sel;  // SPARSE: selector words [O, K/32]
  const bf16_t* X;
  const float* bias;
  void* Y;
  int64_t O, K, T, ldx, ldy;
  int n_o_tiles, n_t_tiles;
  int out_bf16;
  int vec_store;  // Y rows allow 4-wide stores (ldy % 4 == 0, aligned base, O % 4 == 0)
};

template <bool SPARSE, int WO, int WT, int OT, int TT>
struct GemmCfg {
  static constexpr int NT = WO * WT * 64;
  static constexpr int BO = WO * OT * 16;
  static constexpr int BT = WT * TT * 16;
  static constexpr int KC = 64;                       // dense k per stage
  static constexpr int A_ROW = SPARSE ? 80 : 144;     // bytes: 64 + 8 selector + 8 pad | 128 + 16 pad
  static constexpr int X_ROW = 144;                   // 128 + 16 pad
  static constexpr int A_BYTES = BO * A_ROW;
  static constexpr int X_BYTES = BT * X_ROW;
  static constexpr int STAGE = A_BYTES + X_BYTES;
  static constexpr int A_CPR = SPARSE ? 4 : 8;        // 16-byte chunks per row per stage
  static constexpr int A_PER_THREAD = BO * A_CPR / NT;
  static constexpr int X_PER_THREAD = BT * 8 / NT;
  static constexpr int LDS_BYTES = 2 * STAGE;
  static_assert(BO * A_CPR % NT == 0 && BT * 8 % NT == 0, "tile must split evenly over the block");
  static_assert(BO <= NT, "one selector row per thread");
};

template <bool SPARSE, int WO, int WT, int OT, int TT>
__global__ void __launch_bounds__(WO * WT * 64)
nm_gemm_kernel(const GemmArgs a) {
  using C = GemmCfg<SPARSE, WO, WT, OT, TT>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  // XCD-aware tile order: consecutive block ids land on different XCDs (8 of them, each with its
  // own L2); give every XCD a contiguous range of tiles so that the blocks sharing an L2 share X rows.
  const int n_tiles = a.n_o_tiles * a.n_t_tiles;
  const int per_xcd = (n_tiles + 7) >> 3;
  const int tile = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
  if (tile >= n_tiles) return;
  const int o_tile = tile % a.n_o_tiles;
  const int t_tile = tile / a.n_o_tiles;
  const int64_t o0 = (int64_t)o_tile * C::BO;
  const int64_t t0 = (int64_t)t_tile * C::BT;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wo = wave % WO;
  const int wt = wave / WO;
  const int r16 = lane & 15;
  const int kb = lane >> 4;

  // ---- global -> register staging
  uint4 a_reg[C::A_PER_THREAD];
  uint4 x_reg[C::X_PER_THREAD];
  uint2 s_reg = make_uint2(0, 0);
  const int64_t a_ld = SPARSE ? (a.K >> 1) : a.K;  // elements per row of A

  auto load_stage = [&](int ks) {
#pragma unroll
    for (int i = 0; i < C::A_PER_THREAD; ++i) {
      const int q = tid + i * C::NT;
      const int row = q / C::A_CPR, cc = q % C::A_CPR;
      const int64_t o = o0 + row;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (o < a.O) v = *reinterpret_cast<const uint4*>(a.A + o * a_ld + (int64_t)ks * (SPARSE ? 32 : 64) + cc * 8);
      a_reg[i] = v;
    }
    if (SPARSE && tid < C::BO) {
      const int64_t o = o0 + tid;
      s_reg = make_uint2(0, 0);
      if (o < a.O) s_reg = *reinterpret_cast<const uint2*>(a.sel + o * (a.K >> 5) + (int64_t)ks * 2);
    }
#pragma unroll
    for (int i = 0; i < C::X_PER_THREAD; ++i) {
      const int q = tid + i * C::NT;
      const int row = q >> 3, cc = q & 7;
      const int64_t t = t0 + row;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (t < a.T) v = *reinterpret_cast<const uint4*>(a.X + t * a.ldx + (int64_t)ks * 64 + cc * 8);
      x_reg[i] = v;
    }
  };
  auto store_stage = [&](int buf) {
    unsigned char* base = smem + buf * C::STAGE;
#pragma unroll
    for (int i = 0; i < C::A_PER_THREAD; ++i) {
      const int q = tid + i * C::NT;
      const int row = q / C::A_CPR, cc = q % C::A_CPR;
      *reinterpret_cast<uint4*>(base + row * C::A_ROW + cc * 16) = a_reg[i];
    }
    if (SPARSE && tid < C::BO) *reinterpret_cast<uint2*>(base + tid * C::A_ROW + 64) = s_reg;
#pragma unroll
    for (int i = 0; i < C::X_PER_THREAD; ++i) {
      const int q = tid + i * C::NT;
      const int row = q >> 3, cc = q & 7;
      *reinterpret_cast<uint4*>(base + C::A_BYTES + row * C::X_ROW + cc * 16) = x_reg[i];
    }
  };

  f32x4_t acc[OT][TT];
#pragma unroll
  for (int i = 0; i < OT; ++i)
#pragma unroll
    for (int j = 0; j < TT; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  const int nk = (int)(a.K / C::KC);
  load_stage(0);
  store_stage(0);
  __syncthreads();

  const int a_row0 = (wo * OT * 16 + r16) * C::A_ROW;
  const int x_row0 = C::A_BYTES + (wt * TT * 16 + r16) * C::X_ROW;

  for (int ks = 0; ks < nk; ++ks) {
    const int buf = ks & 1;
    if (ks + 1 < nk) load_stage(ks + 1);
    const unsigned char* base = smem + buf * C::STAGE;

    if (SPARSE) {
      // lane (r16, kb) of the W operand covers dense k = 16*kb .. 16*kb+15 of the step: compressed
      // values 8*kb .. 8*kb+7 and 16 selector bits; the X operand holds k = 8*kb+e (e < 8) and
      // 32 + 8*kb + e - 8 (e >= 8).
      u32x4_t af[OT];
      int sel[OT];
#pragma unroll
      for (int i = 0; i < OT; ++i) {
        const unsigned char* row = base + a_row0 + i * 16 * C::A_ROW;
        af[i] = *reinterpret_cast<const u32x4_t*>(row + kb * 16);
        const uint32_t w = *reinterpret_cast<const uint32_t*>(row + 64 + (kb >> 1) * 4);
        sel[i] = (int)(w >> ((kb & 1) * 16));
      }
#pragma unroll
      for (int j = 0; j < TT; ++j) {
        const unsigned char* row = base + x_row0 + j * 16 * C::X_ROW;
        u32x8_t bfrag;
        const u32x4_t lo = *reinterpret_cast<const u32x4_t*>(row + kb * 16);
        const u32x4_t hi = *reinterpret_cast<const u32x4_t*>(row + 64 + kb * 16);
        bfrag = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
        for (int i = 0; i < OT; ++i)
          acc[i][j] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(__builtin_bit_cast(bf16x8_t, af[i]),
                                                                __builtin_bit_cast(bf16x16_t, bfrag), acc[i][j],
                                                                sel[i], 0, 0);
      }
    } else {
#pragma unroll
      for (int s = 0; s < 2; ++s) {
        u32x4_t af[OT];
#pragma unroll
        for (int i = 0; i < OT; ++i)
          af[i] = *reinterpret_cast<const u32x4_t*>(base + a_row0 + i * 16 * C::A_ROW + s * 64 + kb * 16);
#pragma unroll
        for (int j = 0; j < TT; ++j) {
          const u32x4_t bfrag =
              *reinterpret_cast<const u32x4_t*>(base + x_row0 + j * 16 * C::X_ROW + s * 64 + kb * 16);
#pragma unroll
          for (int i = 0; i < OT; ++i)
            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, af[i]),
                                                                __builtin_bit_cast(bf16x8_t, bfrag), acc[i][j], 0, 0,
                                                                0);
        }
      }
    }
    if (ks + 1 < nk) store_stage(buf ^ 1);
    __syncthreads();
  }

  // ---- epilogue: lane holds out-features o .. o+3 (accumulator i -> row 4*kb + i) of token r16
#pragma unroll
  for (int j = 0; j < TT; ++j) {
    const int64_t t = t0 + (wt * TT + j) * 16 + r16;
    if (t >= a.T) continue;
#pragma unroll
    for (int i = 0; i < OT; ++i) {
      const int64_t o = o0 + (wo * OT + i) * 16 + kb * 4;
      if (o >= a.O) continue;
      f32x4_t v = acc[i][j];
      if (a.vec_store) {
        if (a.bias) {
          const float4 b = *reinterpret_cast<const float4*>(a.bias + o);
          v[0] += b.x; v[1] += b.y; v[2] += b.z; v[3] += b.w;
        }
        if (a.out_bf16) {
          uint2 p;
          p.x = f32_to_bf16_rne(v[0]) | (f32_to_bf16_rne(v[1]) << 16);
          p.y = f32_to_bf16_rne(v[2]) | (f32_to_bf16_rne(v[3]) << 16);
          *reinterpret_cast<uint2*>(reinterpret_cast<bf16_t*>(a.Y) + t * a.ldy + o) = p;
        } else {
          *reinterpret_cast<float4*>(reinterpret_cast<float*>(a.Y) + t * a.ldy + o) = make_float4(v[0], v[1], v[2], v[3]);
        }
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (o + e >= a.O) break;
          float y = v[e];
          if (a.bias) y += a.bias[o + e];
          if (a.out_bf16) reinterpret_cast<bf16_t*>(a.Y)[t * a.ldy + o + e] = (bf16_t)f32_to_bf16_rne(y);
          else reinterpret_cast<float*>(a.Y)[t * a.ldy + o + e] = y;
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Plain gather kernel for shapes the tiles cannot take: one thread per output.
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
spmm_general_kernel(const bf16_t* __restrict__ values, const uint32_t* __restrict__ indices, int64_t O, int64_t K, int N,
                    int M, const bf16_t* __restrict__ X, int64_t T, int64_t ldx, const float* __restrict__ bias,
                    void* __restrict__ Y, int64_t ldy, int out_bf16, int64_t n_o_tiles) {
  const int b = log2_of(M);
  const int64_t o = (blockIdx.x % n_o_tiles) * 16 + (threadIdx.x & 15);
  const int64_t t = (blockIdx.x / n_o_tiles) * 16 + (threadIdx.x >> 4);
  if (o >= O || t >= T) return;
  const int64_t nf = K / M * N;
  const int64_t nw = (nf * b + 31) / 32;
  const uint32_t* row = indices + o * nw;
  float acc = 0.f;
  for (int64_t g = 0; g < K / M; ++g) {
    for (int j = 0; j < N; ++j) {
      const int64_t f = g * N + j;
      const uint32_t p = stream_bits(row, nw, f * b, b);
      acc = fmaf(bf16_to_f32(X[t * ldx + g * M + p]), bf16_to_f32(values[o * nf + f]), acc);
    }
  }
  if (bias) acc += bias[o];
  if (out_bf16) reinterpret_cast<bf16_t*>(Y)[t * ldy + o] = (bf16_t)f32_to_bf16_rne(acc);
  else reinterpret_cast<float*>(Y)[t * ldy + o] = acc;
}

// ---------------------------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------------------------
static inline bool aligned_to(const void* p, uintptr_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

static bool tiles_ok(const SpmmArgs& a) {
  if (a.K % 64) return false;
  if (!aligned_to(a.X, 16) || (a.ldx % 8)) return false;
  if (!aligned_to(a.values, 16) || !aligned_to(a.indices, 8)) return false;
  if (a.O > (1 << 24) || a.T > (1ll << 31)) return false;
  return true;
}

size_t spmm_workspace_bytes(int64_t O, int64_t K, int N, int M, int64_t T) {
  (void)T;
  if (K % 64) return 0;                     // general kernel
  if (N == 2 && M == 4) return 0;           // packed layout is the operand layout
  if (N == M) return 0;                     // values are the dense weight
  if (N <= 2) return (size_t)(O * K) + (size_t)(O * K / 8);  // 2:4 re-coding: values + selectors
  return (size_t)(O * K) * 2;               // dense expansion
}

template <bool SPARSE, int WO, int WT, int OT, int TT>
static hipError_t launch_gemm(GemmArgs g, hipStream_t s) {
  using C = GemmCfg<SPARSE, WO, WT, OT, TT>;
  auto kern = nm_gemm_kernel<SPARSE, WO, WT, OT, TT>;
  static bool attr_done = false;  // raising the dynamic LDS limit is idempotent; a race only repeats it
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       C::LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  g.n_o_tiles = (int)((g.O + C::BO - 1) / C::BO);
  g.n_t_tiles = (int)((g.T + C::BT - 1) / C::BT);
  const int64_t n_tiles = (int64_t)g.n_o_tiles * g.n_t_tiles;
  const int64_t grid = ((n_tiles + 7) / 8) * 8;
  if (grid > 0x7FFFFFFF) return hipErrorInvalidValue;
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(C::NT), C::LDS_BYTES, s, g);
  return hipGetLastError();
}

template <bool SPARSE>
static hipError_t dispatch_gemm(const GemmArgs& g, hipStream_t s) {
  // tile choice: large tiles when there is enough work to fill 256 CUs, smaller ones otherwise
  const int64_t tiles_big = ((g.O + 255) / 256) * ((g.T + 255) / 256);
  const int64_t tiles_mid = ((g.O + 127) / 128) * ((g.T + 127) / 128);
  if (tiles_big >= 256) return launch_gemm<SPARSE, 2, 4, 8, 4>(g, s);
  if (tiles_mid >= 256) return launch_gemm<SPARSE, 2, 2, 4, 4>(g, s);
  return launch_gemm<SPARSE, 2, 2, 2, 2>(g, s);
}

hipError_t launch_spmm(const SpmmArgs& a, hipStream_t s, bool* workspace_short) {
  *workspace_short = false;
  if (!tiles_ok(a)) {
    const int64_t n_o_tiles = (a.O + 15) / 16, n_t_tiles = (a.T + 15) / 16;
    if (n_o_tiles * n_t_tiles > 0x7FFFFFFF) return hipErrorInvalidValue;
    hipLaunchKernelGGL(spmm_general_kernel, dim3((unsigned)(n_o_tiles * n_t_tiles)), dim3(256), 0, s, a.values,
                       a.indices, a.O, a.K, a.N, a.M, a.X, a.T, a.ldx, a.bias, a.Y, a.ldy, a.out_bf16, n_o_tiles);
    return hipGetLastError();
  }
  const size_t need = spmm_workspace_bytes(a.O, a.K, a.N, a.M, a.T);
  if (need && (a.workspace == nullptr || a.workspace_bytes < need || !aligned_to(a.workspace, 256))) {
    *workspace_short = true;
    return hipSuccess;
  }
  GemmArgs g;
  g.X = a.X; g.bias = a.bias; g.Y = a.Y;
  g.O = a.O; g.K = a.K; g.T = a.T; g.ldx = a.ldx; g.ldy = a.ldy;
  g.out_bf16 = a.out_bf16;
  g.n_o_tiles = g.n_t_tiles = 0;
  const uintptr_t y_align = a.out_bf16 ? 8 : 16;
  g.vec_store = (a.ldy % 4 == 0) && aligned_to(a.Y, y_align) && (a.O % 4 == 0) &&
                (a.bias == nullptr || aligned_to(a.bias, 16));
  if (a.N <= 2 && a.N < a.M) {
    if (a.N == 2 && a.M == 4) {
      g.A = a.values; g.sel = a.indices;
    } else {
      bf16_t* v24 = reinterpret_cast<bf16_t*>(a.workspace);
      uint32_t* s24 = reinterpret_cast<uint32_t*>(reinterpret_cast<unsigned char*>(a.workspace) + (size_t)(a.O * a.K));
      const int64_t n = a.O * (a.K / 32);
      const dim3 grid((unsigned)((n + 255) / 256));
      switch (a.N * 32 + a.M) {
#define X(n_, m_)                                                                                                 \
  case n_ * 32 + m_:                                                                                              \
    hipLaunchKernelGGL((recode_to_2of4_kernel<n_, m_>), grid, dim3(256), 0, s, a.values, a.indices, a.O, a.K, v24, s24); \
    break;
        X(1, 4) X(1, 8) X(2, 8) X(1, 16) X(2, 16)
#undef X
        default: return hipErrorInvalidValue;
      }
      hipError_t e = hipGetLastError();
      if (e != hipSuccess) return e;
      g.A = v24; g.sel = s24;
    }
    return dispatch_gemm<true>(g, s);
  }
  g.sel = nullptr;
  if (a.N == a.M) {
    g.A = a.values;
  } else {
    bf16_t* wd = reinterpret_cast<bf16_t*>(a.workspace);
    hipError_t e = launch_unpack(a.values, a.indices, a.O, a.K, a.N, a.M, wd, a.K, s);
    if (e != hipSuccess) return e;
    g.A = wd;
  }
  return dispatch_gemm<false>(g, s);
}

}  // namespace nm
