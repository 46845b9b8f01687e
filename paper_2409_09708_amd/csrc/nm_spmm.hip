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
// words, or dense rows) and the X tile are copied global -> LDS asynchronously, two or three stages
// deep with one barrier per step; each wave reads its operand fragments with 16-byte LDS reads
// (XOR-swizzled rows, conflict free) and keeps an (OT*16) x (TT*16) accumulator tile.
// Shapes the tiles cannot take (K % 64 != 0, unaligned pointers) run a plain gather kernel.
#include "nm_device.h"
#include "nm_launch.h"
#include "nm_mma.h"

#include <type_traits>
#include <utility>

namespace nm {

// ---------------------------------------------------------------------------------------------
// Pre-pass: the weight in "stream order", the form every matrix-core kernel here reads it in (the persistent
// kernel always; the tiled kernel except at 2:4 and N = M, whose packed layouts it reads as they lie): exactly the LDS image
// of every (16-row group, K step) as one contiguous 1 KB block, so that the product kernel's
// loads are whole contiguous kilobytes (a 16-row x 64-byte slice of a row-major weight touches 16
// cache lines for one kilobyte, and the selector words one line per 8 bytes).
//   values/dense block (rg, ks) at ((rg * nk) + ks) * 1024: piece i (16 bytes) = row 16*rg + i/4,
//     16-byte chunk (i & 3) ^ ((i >> 4) & 3) of that row's 64 bytes of step ks  (the XOR is the
//     LDS swizzle; a step is 32 compressed values = 64 dense k, or 32 dense weights)
//   selector block (o_tile, ks) at ((o_tile * nk) + ks) * 2048: row r of the tile at r*8, 2 words
// Rows from O up to the next multiple of 256 are written as zeros.
// Levels with N <= 2 are re-coded as a 2:4 weight.  Slot rule: run q (4 weights) owns slots 2q and 2q+1; the first
// kept value of the run goes to slot 2q with selector = its offset in the run, a second one to slot 2q+1; free slots
// hold +0 with selector 0 (the matrix instruction is a plain multiplexer per slot, so any selector of a zero slot
// is harmless).
// ---------------------------------------------------------------------------------------------

template <int N, int M>
__global__ void __launch_bounds__(256)
recode_stream_kernel(const bf16_t* __restrict__ values, const uint32_t* __restrict__ indices, int64_t O, int64_t O_pad,
                     int64_t K, unsigned char* __restrict__ vals_s, unsigned char* __restrict__ sel_s) {
  constexpr int B = log2_of(M);
  constexpr int G = 32 / M;
  constexpr int RUNS = M / 4;
  const int64_t per_row = K / 32;
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= O_pad * per_row) return;
  const int64_t o = id / per_row, blk = id % per_row;
  uint32_t out[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) out[i] = 0;
  uint32_t sel = 0;
  if (o < O) {
    const int64_t nf = K / M * N;
    const int64_t nw = (nf * B + 31) / 32;
    const int64_t f0 = blk * G * N;
    const uint32_t fields = stream_bits(indices + o * nw, nw, f0 * B, G * N * B);
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
  }
  // 32 weights = 16 slots = chunks 2*half, 2*half+1 of step blk/2
  const int64_t nk = K / 64, ks = blk >> 1;
  const int half = (int)(blk & 1);
  *reinterpret_cast<uint4*>(vals_s + stream_piece_offset(o, ks, 2 * half, nk)) = make_uint4(out[0], out[1], out[2], out[3]);
  *reinterpret_cast<uint4*>(vals_s + stream_piece_offset(o, ks, 2 * half + 1, nk)) = make_uint4(out[4], out[5], out[6], out[7]);
  // selectors: per (tile, step) a 2 KiB block; rows r and r+16 of a 32-row pair share the word of a lane
  // (r mod 16, kb): low half = the first row's 16 bits, high half = the second row's, which is what the
  // matrix instruction's ABID modifier selects
  *reinterpret_cast<uint16_t*>(sel_s + stream_selector_offset(o, ks, 2 * half, nk)) = (uint16_t)sel;
  *reinterpret_cast<uint16_t*>(sel_s + stream_selector_offset(o, ks, 2 * half + 1, nk)) = (uint16_t)(sel >> 16);
}

// dense form: one lane per 8 consecutive weights (one 16-byte piece)
__global__ void __launch_bounds__(256)
expand_stream_kernel(const bf16_t* __restrict__ values, const uint32_t* __restrict__ indices, int64_t O, int64_t O_pad,
                     int64_t K, int N, int M, unsigned char* __restrict__ dense_s) {
  const int64_t per_row = K / 8;
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= O_pad * per_row) return;
  const int64_t o = id / per_row, pc = id % per_row;
  uint32_t w[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) w[i] = 0;
  if (o < O) {
    const int b = log2_of(M);
    const int64_t nf = K / M * N;
    const int64_t nw = (nf * b + 31) / 32;
    const uint32_t* row = indices + o * nw;
    const int64_t k0 = pc * 8;
    const int64_t g_first = k0 / M, g_last = (k0 + 7) / M;
    for (int64_t g = g_first; g <= g_last; ++g) {
      for (int j = 0; j < N; ++j) {
        const int64_t f = g * N + j;
        const int64_t k = g * M + stream_bits(row, nw, f * b, b);
        const uint32_t v = values[o * nf + f];
#pragma unroll
        for (int i = 0; i < 8; ++i) w[i] = (k == k0 + i) ? v : w[i];
      }
    }
  }
  const int64_t nk = K / 32, ks = pc >> 2;
  *reinterpret_cast<uint4*>(dense_s + stream_piece_offset(o, ks, (int)(pc & 3), nk)) =
      make_uint4(w[0] | (w[1] << 16), w[2] | (w[3] << 16), w[4] | (w[5] << 16), w[6] | (w[7] << 16));
}

// dense form of a TRANSPOSED weight: the operand rows are the columns of Ws [R, I] (row-major, ld ldw), the
// reduction runs over its rows.  One lane per (column i, 8 consecutive reduction rows); lanes run along i, so
// each of the 8 reads of a wave is one contiguous row segment.  Columns past I (up to the tile edge) are zero.
__global__ void __launch_bounds__(256)
transpose_stream_kernel(const bf16_t* __restrict__ Ws, int64_t R, int64_t I, int64_t ldw, int64_t I_pad,
                        unsigned char* __restrict__ dense_s) {
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= I_pad * (R / 8)) return;
  const int64_t i = id % I_pad, pc = id / I_pad;
  uint32_t w[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) w[e] = i < I ? (uint32_t)Ws[(pc * 8 + e) * ldw + i] : 0u;
  const int64_t nk = R / 32, ks = pc >> 2;
  *reinterpret_cast<uint4*>(dense_s + stream_piece_offset(i, ks, (int)(pc & 3), nk)) =
      make_uint4(w[0] | (w[1] << 16), w[2] | (w[3] << 16), w[4] | (w[5] << 16), w[6] | (w[7] << 16));
}

// ---------------------------------------------------------------------------------------------
// Tiled matrix-core product.
//
// Operand tiles travel global -> LDS directly (global_load_lds_dwordx4: each lane names its own
// 16 global bytes, the wave's 64 pieces land in 1 KB of consecutive LDS), STAGES buffers deep, so
// that two K steps of loads are in flight while a third is multiplied and no register is spent on
// staging.  The compiler does not track these loads; the kernel counts them itself: every wave
// issues exactly LPW loads per stage and waits with s_waitcnt vmcnt(LPW) (one younger stage may
// still be in flight) or vmcnt(0) before the one barrier of the step.
// LDS rows are not padded (the DMA writes 1 KB runs); instead the 16-byte pieces of a row are
// XOR-swizzled with the row number on the way in, and the fragment reads apply the same XOR, which
// keeps 8 consecutive rows on distinct banks.
// ---------------------------------------------------------------------------------------------
struct GemmArgs {
  const bf16_t* A;      // SPARSE: compressed values [O, K/2]; dense: W_s [O, K]
  const uint32_t* sel;  // SPARSE: selector words [O, K/32]
  const bf16_t* X;
  const float* bias;
  void* Y;
  float* partial;       // splits > 1: fp32 partial sums [splits][T][O] (rows of O floats), added up by the reduce kernel
  int64_t O, K, T, ldx, ldy;
  int n_o_tiles, n_t_tiles;
  uint8_t out_bf16;
  uint8_t vec_store;    // Y rows split into whole aligned 16-byte pieces (ldy, O multiples of 8 (bf16) / 4 (fp32))
  uint8_t stream_form;  // A (and sel) lie in stream order (the pre-pass's output), else row-major as packed
  uint8_t splits;       // ranges the reduction is cut into (tiled kernel only; 1 = the whole K in one block)
  uint8_t rot;          // tiled kernel: XCD x takes the layer's share number (x + rot) mod 8
};

template <bool SPARSE, int WO, int WT, int OT, int TT, int STAGES_>
struct GemmCfg {
  static constexpr int STAGES = STAGES_;
  static constexpr int NW = WO * WT;
  static constexpr int NT = NW * 64;
  static constexpr int BO = WO * OT * 16;
  static constexpr int BT = WT * TT * 16;
  static constexpr int KC = 64;                         // dense k per stage
  static constexpr int H = SPARSE ? 1 : 2;              // sub-steps (32 matrix instructions each) per stage
  static constexpr int A_ROWB = SPARSE ? 64 : 128;      // bytes of one W row per stage
  static constexpr int X_BYTES = BT * 128;
  static constexpr int A_BYTES = BO * A_ROWB;
  static constexpr int S_BYTES = SPARSE ? BO * 8 : 0;   // two selector words per row per stage
  static constexpr int STAGE = X_BYTES + A_BYTES + S_BYTES;
  static constexpr int LDS_BYTES = STAGES * STAGE;
  static constexpr int X_LOADS = X_BYTES / 1024;        // wave-wide 16-byte loads per stage
  static constexpr int A_LOADS = A_BYTES / 1024;
  static constexpr int S_LOADS = S_BYTES / 256;         // wave-wide 4-byte loads per stage
  static constexpr int X_PW = (X_LOADS + NW - 1) / NW;  // per wave (surplus waves repeat a load)
  static constexpr int A_PW = (A_LOADS + NW - 1) / NW;
  static constexpr int S_PW = SPARSE ? (S_LOADS + NW - 1) / NW : 0;
  static constexpr int LPW = X_PW + A_PW + S_PW;
  static_assert(STAGES == 2 || STAGES == 3, "two or three LDS stages");
  static_assert(STAGES * LPW < 64, "vmcnt is a 6-bit counter");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
};

// Accumulator start value of the 16 x 16 block whose four out-features start at o: the bias (so
// that no load sits between the stores of the epilogue), or zero.
__device__ __forceinline__ f32x4_t bias_init(const float* bias, int64_t o, int64_t O, bool vec) {
  f32x4_t v = f32x4_t{0.f, 0.f, 0.f, 0.f};
  if (bias) {
    if (vec) {
      if (o < O) {
        const float4 b = *reinterpret_cast<const float4*>(bias + o);
        v = f32x4_t{b.x, b.y, b.z, b.w};
      }
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (o + e < O) v[e] = bias[o + e];
    }
  }
  return v;
}

// One tile of one layer; `block` is the block's number among the layer's blocks (a multiple of 8 of them, so
// that block mod 8 is the XCD the block runs on).
// STREAM: the weight lies in stream order (the pre-pass's output: every 16-row x K-step slice one contiguous,
// already swizzled kilobyte; selector words interleaved per 32-row pair), else row-major (the packed 2:4 layout
// or a dense level's values, read as they lie).
template <bool SPARSE, int WO, int WT, int OT, int TT, int STAGES, bool STREAM>
__device__ __forceinline__ void gemm_tile(const GemmArgs& a, unsigned block, unsigned char* smem) {
  using C = GemmCfg<SPARSE, WO, WT, OT, TT, STAGES>;
  static_assert(!STREAM || (OT % 2 == 0 && C::BO % 32 == 0 && 256 % C::BO == 0), "stream order: whole 32-row pairs inside one 256-row tile");
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;

  // XCD-aware tile order: consecutive block ids land on different XCDs (8 of them, each with its
  // own L2); give every XCD a contiguous range of tiles so that the blocks sharing an L2 share X rows.
  // A layer with few tiles and a long reduction is cut along K as well: unit = (tile, K range); every range of a
  // tile writes fp32 partial sums of its own, which splitk_reduce_kernel adds in range order.
  const int n_splits = a.splits > 1 ? a.splits : 1;
  const int n_units = a.n_o_tiles * a.n_t_tiles * n_splits;
  const int per_xcd = (n_units + 7) >> 3;
  // (the shares at the end of the list may be short or empty; `rot` says which XCDs get those, so that the layers
  // of a launch can leave them to different ones)
  const int unit = (int)((block + a.rot) & 7) * per_xcd + (int)(block >> 3);
  if (unit >= n_units) return;
  const int tile = unit / n_splits, split = unit - tile * n_splits;
  const int o_tile = tile % a.n_o_tiles;
  const int t_tile = tile / a.n_o_tiles;
  const int64_t o0 = (int64_t)o_tile * C::BO;
  const int64_t t0 = (int64_t)t_tile * C::BT;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wo = wave % WO;
  const int wt = wave / WO;
  const int r16 = lane & 15;
  const int kb = lane >> 4;

  // ---- per-lane source offsets and per-wave LDS destinations of this wave's loads (fixed over K)
  const int64_t a_ld = SPARSE ? (a.K >> 1) : a.K;  // elements per row of A
  uint32_t x_voff[C::X_PW], a_voff[C::A_PW], s_voff[C::S_PW > 0 ? C::S_PW : 1];
  uint32_t x_dst[C::X_PW], a_dst[C::A_PW], s_dst[C::S_PW > 0 ? C::S_PW : 1];
  const int64_t t_last = a.T - 1 - t0, o_last = a.O - 1 - o0;  // rows past the edge re-read the last valid row
#pragma unroll
  for (int i = 0; i < C::X_PW; ++i) {
    const int j = (wave + i * C::NW) % C::X_LOADS;
    int64_t row = 8 * j + (lane >> 3);
    const int c = (lane & 7) ^ (int)(row & 7);
    if (row > t_last) row = t_last;
    x_voff[i] = (uint32_t)((row * a.ldx + c * 8) * 2);
    x_dst[i] = (uint32_t)(j * 1024);
  }
  const int nk_all = (int)(a.K / C::KC);               // K steps of the layer
  const int per_split = (nk_all + n_splits - 1) / n_splits;
  const int ks0 = split * per_split;                    // this block's steps: ks0 .. ks0 + nk - 1
  const int nk = nk_all - ks0 < per_split ? nk_all - ks0 : per_split;
#pragma unroll
  for (int i = 0; i < C::A_PW; ++i) {
    const int j = (wave + i * C::NW) % C::A_LOADS;
    if constexpr (STREAM) {
      // load j brings one kilobyte: 16-row group rg of the tile at the stage's K step (2:4 form), or at its
      // first (h = 0) or second (h = 1) 32-wide step (dense form, two stream steps per stage)
      constexpr int GROUPS = C::BO / 16;
      const int rg = j % GROUPS, h = j / GROUPS;
      a_voff[i] = (uint32_t)((((o0 >> 4) + rg) * (int64_t)(SPARSE ? nk_all : 2 * nk_all) + h) << 10) + (uint32_t)(lane * 16);
      a_dst[i] = (uint32_t)(C::X_BYTES + h * (C::BO * 64) + rg * 1024);
    } else {
      int64_t row;
      int c;
      if (SPARSE) { row = 16 * j + (lane >> 2); c = (lane & 3) ^ (int)((row >> 1) & 3); }
      else { row = 8 * j + (lane >> 3); c = (lane & 7) ^ (int)(row & 7); }
      if (row > o_last) row = o_last;
      a_voff[i] = (uint32_t)((row * a_ld + c * 8) * 2);
      a_dst[i] = (uint32_t)(C::X_BYTES + j * 1024);
    }
  }
  if (SPARSE) {
#pragma unroll
    for (int i = 0; i < C::S_PW; ++i) {
      const int j = (wave + i * C::NW) % C::S_LOADS;
      if constexpr (STREAM) {
        // the tile's share of the (256-row tile, step) selector block: 256 bytes per 32-row pair
        s_voff[i] = (uint32_t)(((o0 >> 8) * (int64_t)nk_all << 11) + (((o0 & 255) >> 5) + j) * 256 + lane * 4);
      } else {
        int64_t row = 32 * j + (lane >> 1);
        if (row > o_last) row = o_last;
        s_voff[i] = (uint32_t)((row * (a.K >> 5) + (lane & 1)) * 4);
      }
      s_dst[i] = (uint32_t)(C::X_BYTES + C::A_BYTES + j * 256);
    }
  }
  // elements the weight and selector pointers advance per stage
  constexpr int A_STEP = STREAM ? (SPARSE ? 512 : 1024) : (SPARSE ? 32 : 64);
  constexpr int S_STEP = STREAM ? 512 : 2;
  const bf16_t* x_base = a.X + t0 * a.ldx + (int64_t)ks0 * 64;
  const bf16_t* a_base = (STREAM ? a.A : a.A + o0 * a_ld) + (int64_t)ks0 * A_STEP;
  const uint32_t* s_base = SPARSE ? (STREAM ? a.sel : a.sel + o0 * (a.K >> 5)) + (int64_t)ks0 * S_STEP : nullptr;
  // where the block's sums go: the output, or its range's partial sums (plain fp32 rows of O, no bias yet)
  void* out_ptr = a.Y;
  int64_t out_ld = a.ldy;
  bool out_bf16 = a.out_bf16 != 0, out_vec = a.vec_store != 0;
  const float* bias = a.bias;
  if (a.splits > 1) {
    out_ptr = a.partial + (int64_t)split * a.T * a.O;
    out_ld = a.O;
    out_bf16 = false;
    out_vec = (a.O & 3) == 0;
    bias = nullptr;
  }

  // The stage to be loaded next, as three running uniform pointers (X rows at the stage's k, weight, selectors),
  // advanced by constants: the step loop then holds no address products.
  uniform_ptr_t x_next = make_uniform(x_base), a_next = make_uniform(a_base), s_next = make_uniform(s_base);
  // the d-th of this wave's LPW loads of that stage into LDS buffer buf (d is a compile-time index)
  auto issue_one = [&](auto d_tag, int buf) {
    constexpr int d = decltype(d_tag)::value;
    const uint32_t lds = __builtin_amdgcn_readfirstlane(lds0 + (uint32_t)buf * C::STAGE);
    if constexpr (d < C::X_PW) {
      dma16(x_next, x_voff[d], lds + x_dst[d]);
    } else if constexpr (d < C::X_PW + C::A_PW) {
      dma16(a_next, a_voff[d - C::X_PW], lds + a_dst[d - C::X_PW]);
    } else {
      dma4(s_next, s_voff[d - C::X_PW - C::A_PW], lds + s_dst[d - C::X_PW - C::A_PW]);
    }
    if constexpr (d == C::LPW - 1) {  // the stage is out: on to the next one
      x_next += 64 * sizeof(bf16_t);
      a_next += A_STEP * sizeof(bf16_t);
      s_next += S_STEP * sizeof(uint32_t);
    }
  };
  auto issue_stage = [&](int buf) {
    [&]<int... D>(std::integer_sequence<int, D...>) {
      (issue_one(std::integral_constant<int, D>{}, buf), ...);
    }(std::make_integer_sequence<int, C::LPW>{});
  };

  f32x4_t acc[OT][TT];
#pragma unroll
  for (int i = 0; i < OT; ++i) {
    const f32x4_t b = bias_init(bias, o0 + (wo * OT + i) * 16 + kb * 4, a.O, a.vec_store);
#pragma unroll
    for (int j = 0; j < TT; ++j) acc[i][j] = b;
  }

  // fragment read offsets inside a stage (the XOR undoes the swizzle applied by the loads)
  const int x_sw = r16 & 7;
  const int x_row = (wt * TT * 16 + r16) * 128;
  // stream order keeps 64-byte weight rows in both forms (the dense stage is two such sub-tiles)
  constexpr int A_ROWB = STREAM ? 64 : C::A_ROWB;
  const int a_row = C::X_BYTES + (wo * OT * 16 + r16) * A_ROWB;
  const int a_sw = (SPARSE || STREAM) ? ((r16 >> 1) & 3) : (r16 & 7);
  const int s_row = STREAM ? C::X_BYTES + C::A_BYTES + (wo * OT / 2) * 256 + r16 * 16 + kb * 4
                           : C::X_BYTES + C::A_BYTES + (wo * OT * 16 + r16) * 8 + (kb >> 1) * 4;

  // One sub-step = 32 matrix instructions per wave.  SPARSE: a stage is one sub-step (K = 64 through
  // v_smfmac 16x16x64).  Dense: a stage is two sub-steps of K = 32 (v_mfma 16x16x32), h selects the half.
  // SPARSE lane (r16, kb) of the W operand covers dense k = 16*kb .. 16*kb+15 of the step (compressed
  // values 8*kb .. 8*kb+7 and 16 selector bits); the X operand holds k = 8*kb+e (e < 8) and
  // 32 + 8*kb + e - 8 (e >= 8).
  constexpr int H = C::H;
  u32x4_t af[OT];
  int sel[OT];
  u32x8_t bs[SPARSE ? TT : 1];
  u32x4_t bd[SPARSE ? 1 : TT];
  auto read_frags = [&](int buf, int h) {
    const unsigned char* base = smem + buf * C::STAGE;
    if (SPARSE) {
#pragma unroll
      for (int i = 0; i < OT; ++i) {
        af[i] = *reinterpret_cast<const u32x4_t*>(base + a_row + i * 16 * A_ROWB + ((kb ^ a_sw) * 16));
        if constexpr (STREAM) {
          // one word serves the two 16-row blocks of a pair: low half / high half, picked by the instruction
          sel[i] = (int)*reinterpret_cast<const uint32_t*>(base + s_row + (i / 2) * 256);
        } else {
          const uint32_t w = *reinterpret_cast<const uint32_t*>(base + s_row + i * 16 * 8);
          sel[i] = (int)(w >> ((kb & 1) * 16));
        }
      }
#pragma unroll
      for (int j = 0; j < TT; ++j) {
        const unsigned char* row = base + x_row + j * 16 * 128;
        const u32x4_t lo = *reinterpret_cast<const u32x4_t*>(row + ((kb ^ x_sw) * 16));
        const u32x4_t hi = *reinterpret_cast<const u32x4_t*>(row + (((4 + kb) ^ x_sw) * 16));
        bs[j] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      }
    } else {
#pragma unroll
      for (int i = 0; i < OT; ++i) {
        if constexpr (STREAM)
          af[i] = *reinterpret_cast<const u32x4_t*>(base + a_row + h * (C::BO * 64) + i * 16 * A_ROWB + ((kb ^ a_sw) * 16));
        else
          af[i] = *reinterpret_cast<const u32x4_t*>(base + a_row + i * 16 * A_ROWB + (((h * 4 + kb) ^ a_sw) * 16));
      }
#pragma unroll
      for (int j = 0; j < TT; ++j)
        bd[j] = *reinterpret_cast<const u32x4_t*>(base + x_row + j * 16 * 128 + (((h * 4 + kb) ^ x_sw) * 16));
    }
  };
  // 32 matrix instructions; when `load` is set, this wave's LPW loads of stage (lks -> lbuf) are issued
  // between them, one every few instructions, so that the memory pipe is fed evenly instead of in bursts
  constexpr int MMA = OT * TT;
  constexpr int EVERY = MMA / C::LPW > 0 ? MMA / C::LPW : 1;
  auto multiply = [&](bool load, int lbuf) {
    [&]<int... Q>(std::integer_sequence<int, Q...>) {
      ([&] {
        constexpr int j = Q / OT, i = Q % OT;
        if (SPARSE)
          acc[i][j] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(__builtin_bit_cast(bf16x8_t, af[i]),
                                                                __builtin_bit_cast(bf16x16_t, bs[j]), acc[i][j],
                                                                sel[i], 0, STREAM ? (i & 1) : 0);
        else
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, af[i]),
                                                              __builtin_bit_cast(bf16x8_t, bd[j]), acc[i][j], 0, 0, 0);
        if constexpr (Q % EVERY == EVERY - 1 && Q / EVERY < C::LPW) {
          if (load) issue_one(std::integral_constant<int, Q / EVERY>{}, lbuf);
          __builtin_amdgcn_sched_barrier(0);
        }
      }(), ...);
    }(std::make_integer_sequence<int, MMA>{});
  };
  // stage s has landed in this wave's view once at most the loads of the younger stages issued so far
  // are outstanding: `younger` of them (0, 1 or 2)
  auto wait_stage = [&](int younger) {
    if (younger >= 2) wait_loads_outstanding<2 * C::LPW>();
    else if (younger == 1) wait_loads_outstanding<C::LPW>();
    else wait_loads_outstanding<0>();
  };

#pragma unroll
  for (int s = 0; s < STAGES; ++s)
    if (s < STAGES - 1 && s < nk) issue_stage(s);

  // One barrier per stage; the buffer multiplied in the previous step is refilled right after the barrier,
  // STAGES-1 stages ahead.  A wave issues one instruction at a time, so whatever the step spends on addresses and
  // conditions its matrix instructions do not get: the steady state (every step has a stage to load) runs STAGES
  // steps at a time, which makes every LDS buffer a constant and leaves the step without branches; the last steps
  // run the general form.
  int ks = 0;
  for (; ks + 2 * STAGES - 2 < nk; ks += STAGES) {
    [&]<int... B>(std::integer_sequence<int, B...>) {
      ([&] {
        constexpr int buf = B, nbuf = (B + STAGES - 1) % STAGES;
        wait_stage(STAGES == 3 ? 1 : 0);
        __builtin_amdgcn_s_barrier();
#pragma unroll
        for (int h = 0; h < H; ++h) {
          read_frags(buf, h);
          multiply(h == 0, nbuf);
        }
      }(), ...);
    }(std::make_integer_sequence<int, STAGES>{});
  }
  {
    int buf = 0;  // ks is a multiple of STAGES here
    for (; ks < nk; ++ks) {
      wait_stage((STAGES == 3 && ks + 1 < nk) ? 1 : 0);
      __builtin_amdgcn_s_barrier();
      int nbuf = buf + STAGES - 1;
      if (nbuf >= STAGES) nbuf -= STAGES;
#pragma unroll
      for (int h = 0; h < H; ++h) {
        read_frags(buf, h);
        multiply(h == 0 && ks + STAGES - 1 < nk, nbuf);
      }
      if (++buf == STAGES) buf = 0;
    }
  }

  // ---- epilogue.  A lane holds out-features o .. o+3 (accumulator element e -> row 4*kb + e of the
  // 16-row tile) of token r16, i.e. 8 or 16 contiguous bytes of a Y row.  For aligned outputs every
  // wave transposes 16 tokens at a time through its own LDS slice so that the global stores are
  // 16 bytes per lane and whole row segments of the wave tile (OW elements) are written contiguously.
  __builtin_amdgcn_s_barrier();  // every wave is done with the operand stages
  auto get = [&](int i, int j) { return __builtin_bit_cast(u32x4_t, acc[i][j]); };
  const int64_t row0 = t0 + wt * TT * 16, col0 = o0 + wo * OT * 16;
  static_assert(C::NW * wave_tile_slice_bytes<OT, 4>() <= C::LDS_BYTES, "write-out slices");
  if (out_vec) {
    if (out_bf16)
      write_wave_tile_pieces<OT, TT, 2>(smem + wave * wave_tile_slice_bytes<OT, 2>(), lane, get, out_ptr, out_ld, row0, col0, a.T, a.O);
    else
      write_wave_tile_pieces<OT, TT, 4>(smem + wave * wave_tile_slice_bytes<OT, 4>(), lane, get, out_ptr, out_ld, row0, col0, a.T, a.O);
  } else {
    write_wave_tile_elements<OT, TT>(lane, get, out_ptr, out_ld, row0, col0, a.T, a.O, out_bf16);
  }
}

// Both weight orders live in one kernel (a block-uniform branch): the layers of a launch may differ in it (2:4 and
// N = M are read as packed, the other levels in stream order), and every launch more is a partly filled chip more.
template <bool SPARSE, int WO, int WT, int OT, int TT, int STAGES>
__global__ void __launch_bounds__(WO * WT * 64)
nm_gemm_kernel(const GemmArgs a) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  if (a.stream_form) gemm_tile<SPARSE, WO, WT, OT, TT, STAGES, true>(a, blockIdx.x, smem);
  else gemm_tile<SPARSE, WO, WT, OT, TT, STAGES, false>(a, blockIdx.x, smem);
}

// The tiles of many small layers in one launch, whatever their operand form and weight order: products of a few
// tokens are a handful of tiles each, far fewer than the chip has compute units, and independent ones fill it
// together (two launches, one per form, would each end in a partly filled chip and run one after the other).
// A block finds its layer in the running block counts (whole multiples of 8 per layer) by bisection and takes the
// branch of that layer's form; the table entry is the layer's arguments packed to 80 bytes, so that the 48 linears
// of a 12-block model fit one kernel argument segment.
constexpr int kTileLayersMax = 50;
struct TileLayer {
  const bf16_t* A;
  const uint32_t* sel;
  const bf16_t* X;
  const float* bias;
  void* Y;
  float* partial;
  int64_t ldy;
  uint32_t O, T;           // O <= 2^24, T < 2^31
  uint32_t K : 23, rot : 3;  // K <= 2^22
  uint32_t ldx : 23, out_bf16 : 1, vec_store : 1, stream_form : 1, sparse_form : 1, splits : 4;
  uint32_t block_end;      // exclusive prefix end, in blocks
};
struct TileGroup {
  int32_t count;
  TileLayer layer[kTileLayersMax];
};
static_assert(sizeof(TileLayer) == 80 && sizeof(TileGroup) <= 4096, "the table must fit the kernel argument segment");

// SS, SD: LDS stages of the 2:4-form and of the dense-form tiles (the launch's LDS is the larger of the two).
template <int WO, int WT, int OT, int TT, int SS, int SD>
__global__ void __launch_bounds__(WO * WT * 64)
nm_gemm_group_kernel(const TileGroup g) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  int lo = 0, hi = g.count - 1;  // the first layer whose end lies beyond this block
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (blockIdx.x >= g.layer[mid].block_end) lo = mid + 1;
    else hi = mid;
  }
  const TileLayer& L = g.layer[lo];
  const unsigned block = blockIdx.x - (lo ? g.layer[lo - 1].block_end : 0u);
  GemmArgs a;
  a.A = L.A; a.sel = L.sel; a.X = L.X; a.bias = L.bias; a.Y = L.Y; a.partial = L.partial;
  a.O = L.O; a.K = L.K; a.T = L.T; a.ldx = L.ldx; a.ldy = L.ldy;
  a.n_o_tiles = (int)((L.O + WO * OT * 16 - 1) / (WO * OT * 16));
  a.n_t_tiles = (int)((L.T + WT * TT * 16 - 1) / (WT * TT * 16));
  a.out_bf16 = L.out_bf16; a.vec_store = L.vec_store; a.stream_form = L.stream_form; a.splits = L.splits;
  a.rot = L.rot;
  if (L.sparse_form) {
    if (L.stream_form) gemm_tile<true, WO, WT, OT, TT, SS, true>(a, block, smem);
    else gemm_tile<true, WO, WT, OT, TT, SS, false>(a, block, smem);
  } else {
    if (L.stream_form) gemm_tile<false, WO, WT, OT, TT, SD, true>(a, block, smem);
    else gemm_tile<false, WO, WT, OT, TT, SD, false>(a, block, smem);
  }
}

// The partial sums of layers whose reduction was cut into ranges, added up in range order (so the result does not
// depend on which block finished first), plus the bias, rounded to the output type.  One launch serves every such
// layer of a call; a thread owns four consecutive out-features of one token.
constexpr int kSplitLayersMax = 60;
struct SplitLayer {
  const float* partial;  // [splits][T][O]
  const float* bias;     // nullable
  void* Y;
  int64_t ldy;
  int32_t T, O, splits, out_bf16;
  uint32_t block_end;    // exclusive prefix end, in blocks of 256 threads
  int32_t vec;           // Y rows in whole aligned pieces of four outputs
};
struct SplitGroup {
  int32_t count;
  SplitLayer layer[kSplitLayersMax];
};
static_assert(sizeof(SplitGroup) <= 4096, "the table must fit the kernel argument segment");

__global__ void __launch_bounds__(256) splitk_reduce_kernel(const SplitGroup g) {
  int l = 0;
#pragma unroll 4
  for (int i = 0; i + 1 < g.count; ++i) l += blockIdx.x >= g.layer[i].block_end ? 1 : 0;
  const SplitLayer& L = g.layer[l];
  const unsigned first = l ? g.layer[l - 1].block_end : 0u;
  const int quads = (L.O + 3) >> 2;
  const int64_t q = (int64_t)(blockIdx.x - first) * 256 + threadIdx.x;
  if (q >= (int64_t)L.T * quads) return;
  const int64_t t = q / quads;
  const int o = (int)(q - t * quads) * 4;
  const int64_t plane = (int64_t)L.T * L.O;
  const float* src = L.partial + t * L.O + o;
  float y[4] = {0.f, 0.f, 0.f, 0.f};
  const int n = L.O - o < 4 ? L.O - o : 4;
  if ((L.O & 3) == 0) {
    for (int sp = 0; sp < L.splits; ++sp) {
      const float4 v = *reinterpret_cast<const float4*>(src + sp * plane);
      y[0] += v.x; y[1] += v.y; y[2] += v.z; y[3] += v.w;
    }
  } else {
    for (int sp = 0; sp < L.splits; ++sp)
      for (int e = 0; e < n; ++e) y[e] += src[sp * plane + e];
  }
  if (L.bias != nullptr)
    for (int e = 0; e < n; ++e) y[e] += L.bias[o + e];
  if (L.out_bf16) {
    bf16_t* dst = reinterpret_cast<bf16_t*>(L.Y) + t * L.ldy + o;
    if (L.vec) {
      uint2 pk;
      pk.x = pack_bf16x2(y[0], y[1]);
      pk.y = pack_bf16x2(y[2], y[3]);
      *reinterpret_cast<uint2*>(dst) = pk;
    } else {
      for (int e = 0; e < n; ++e) dst[e] = (bf16_t)f32_to_bf16_rne(y[e]);
    }
  } else {
    float* dst = reinterpret_cast<float*>(L.Y) + t * L.ldy + o;
    if (L.vec) *reinterpret_cast<float4*>(dst) = make_float4(y[0], y[1], y[2], y[3]);
    else
      for (int e = 0; e < n; ++e) dst[e] = y[e];
  }
}

// ---------------------------------------------------------------------------------------------
// Persistent streamed product for large layers.
//
// One block of 8 waves (4 along O x 2 along T, 64 x 128 outputs each) per CU walks over its share of
// the 256 x 256 output tiles; the LDS stage ring and the load pipeline run across tile boundaries,
// so the first stages of the next tile are already in flight (and its first fragments in registers)
// while the current tile is being written out, and the stores of one tile drain while the next one
// is multiplied.  A K step is 32 matrix instructions per wave for both operand forms: K = 64 of
// the 2:4 form through v_smfmac_f32_16x16x64_bf16, K = 32 of the dense form through
// v_mfma_f32_16x16x32_bf16.
// Per step a wave keeps its 4 W fragments in registers and streams the 8 X fragments through a ring
// of four, three ahead of the instructions that consume them; the fragments of the next step are
// fetched during the last groups of the current one.  Before anything of stage g+1 is read (group
// TT-3 of stage g) every wave has issued all its reads of stage g: it drains them, makes sure its
// share of stage g+1 has landed, meets the others at the step's only barrier and then refills the
// buffer of stage g with stage g+3, two full steps ahead of its use.
// The tiles that share X rows (same tokens, other out-features) run on one XCD at the same time; each
// walks K from its own starting step and wraps around, so that they do not miss on the same lines together.
// The weight arrives in stream order (see the pre-pass above): every W load is one contiguous
// kilobyte.  A ragged last token tile is shifted back inside X (it recomputes a few rows of its
// neighbour but stores only its own) and the weight is zero-padded to whole tiles, so every tile is
// full and lane offsets never change.
// ---------------------------------------------------------------------------------------------
template <bool SPARSE, int WO_, int WT_, int STAGES_, bool I8 = false>
struct StreamCfg {
  // Tiles are 256 out-features x 256 tokens on 8 waves (one block per CU, two waves per SIMD), three stages (four
  // for the dense form, whose stages are 32 KiB); a wave holds 32 accumulator blocks of 16 x 16.  The layout in
  // use is WO 4, WT 2 (64 out-features x 128 tokens per wave, 20 KiB of fragment reads per wave and step).
  // Measured and no faster on transformer-sized layers: WO 2, WT 4 (128 x 64 per wave: a fifth fewer fragment
  // bytes, the same time in the 2:4 form and 4 % more in the dense form), 4 waves of 128 x 128 (one per SIMD
  // with the 512-register budget: a lone wave does not hide its own LDS and issue latency), and 256 x 128 tiles
  // with two stages (two blocks of 4 waves per CU).
  static constexpr int WO = WO_, WT = WT_, BO = 256, OT = BO / (WO * 16), TT = 32 / OT;  // 32 accumulator blocks per wave
  static constexpr int TW = TT * 16, BT = TW * WT;       // tokens per wave, per tile
  static constexpr int NW = WO * WT, NT = NW * 64, STAGES = STAGES_;
  static constexpr int PER_CU = (NW == 4 && STAGES == 2) ? 2 : 1;  // co-resident blocks
  static constexpr int OW = OT * 16;                     // out-features per wave
  // The int8 forms (v_smfmac_i32_16x16x128_i8, v_mfma_i32_16x16x64_i8) have the same geometry in bytes with
  // twice the K per step; only the selectors differ: a lane's 16 compressed values need a whole 32-bit word,
  // so a row takes 16 bytes of selectors per step instead of 8 and no two rows share a word.
  static constexpr int ES = I8 ? 1 : 2;                  // bytes per operand element
  static constexpr int X_ROWB = SPARSE ? 128 : 64;       // bytes of one X row per stage
  static constexpr int KSTEP = X_ROWB / ES;              // dense k per stage
  static constexpr int A_ROWB = 64;                      // compressed values of the 2:4 form, or dense weights
  static constexpr int X_BYTES = BT * X_ROWB;
  static constexpr int A_BYTES = BO * A_ROWB;
  static constexpr int S_ROWB = I8 ? 16 : 8;
  static constexpr int S_BYTES = SPARSE ? BO * S_ROWB : 0;
  static constexpr int STAGE = X_BYTES + A_BYTES + S_BYTES;
  // Per-out-feature constants of a tile travel through LDS: the bias (one slice of BO floats per stage buffer,
  // read when the tile starts), or for int8 the weight scales and the bias (read when the tile ends, so the
  // slices alternate with the tile's parity instead: two pairs)
  static constexpr int BIAS0 = STAGES * STAGE;
  static constexpr int LDS_BYTES = BIAS0 + (I8 ? 4 : STAGES) * BO * 4;
  static constexpr int X_PW = X_BYTES / 1024 / NW;
  static constexpr int A_PW = A_BYTES / 1024 / NW;
  static constexpr int S_PW = SPARSE ? S_BYTES / 256 / NW : 0;
  static constexpr int LPW = X_PW + A_PW + S_PW;
  static_assert(WO == 2 || WO == 4, "wave layouts");
  static_assert(BO * 4 == 1024, "the bias slice of a tile is one wave-load");
  static_assert(LDS_BYTES * PER_CU <= 160 * 1024 && STAGES * (LPW + 2) < 64, "LDS budget and vmcnt range");
};

// One launch serves a list of layers of the same operand form: their tiles form one list (layer after layer),
// which the blocks share as they share the tiles of a single layer.  A stack of independent products then ends
// in ONE partial round of tiles instead of one per layer (591 tiles on 256 compute units are 2.3 rounds and
// cost 3).  The table travels in the kernel arguments.
struct StreamLayer {
  const bf16_t* A;      // stream-order values (2:4 form) or dense weight
  const uint32_t* sel;  // stream-order selectors (2:4 form)
  const bf16_t* X;
  const float* bias;    // nullable
  const float* scale;   // int8: per-out-feature weight scales, nullable (= 1)
  void* Y;
  int32_t O, T, nk, ldx, ldy;  // nk: K steps of the form; ldx, ldy in elements
  int32_t n_o_tiles;
  int32_t n_tiles;      // tiles of this layer
  float x_scale;        // int8: activation scale
  int32_t out_kind;     // NM_OUT_F32 / NM_OUT_BF16 / NM_OUT_I32 (int8 only)
  int32_t reserved;
};
constexpr int kStreamWO = 4, kStreamWT = 2;  // wave layout of the bfloat16 launches
constexpr int kStreamLayersMax = 44;
struct StreamGroup {
  int32_t count, n_tiles;
  StreamLayer layer[kStreamLayersMax];
};
static_assert(sizeof(StreamGroup) <= 4096, "the table must fit the kernel argument segment");

template <bool SPARSE, int WO_, int WT_, int STAGES_, bool I8 = false>
__global__ void __launch_bounds__(WO_ * WT_ * 64, (WO_ * WT_ == 4 && STAGES_ == 2) ? 2 : (WO_ * WT_) / 4)
nm_stream_kernel(const StreamGroup g) {
  using C = StreamCfg<SPARSE, WO_, WT_, STAGES_, I8>;
  constexpr int OT = C::OT, TT = C::TT, STAGES = C::STAGES;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;

  // ---- this block's tiles: every XCD (block id mod 8) owns a contiguous eighth of the tiles of EVERY layer,
  // out-feature tiles fastest; its list is those ranges layer after layer, and its blocks take the entries
  // round-robin.  So the blocks sharing an L2 work on neighbouring tiles (same X rows) at the same time, and
  // every XCD gets the same share of each layer's work, whatever the layers' K.
  const int xcd = (int)(blockIdx.x & 7);
  const int slots = (int)(gridDim.x >> 3);
  auto xcd_share = [&](int layer) {  // how many tiles of the layer this XCD owns
    const int n = g.layer[layer].n_tiles;
    const int per = (n + 7) >> 3;
    const int left = n - xcd * per;
    return left < 0 ? 0 : (left < per ? left : per);
  };
  int entries = 0;
  for (int l = 0; l < g.count; ++l) entries += xcd_share(l);
  const int first = (int)(blockIdx.x >> 3);
  if (first >= entries) return;
  const int my_tiles = (entries - first + slots - 1) / slots;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wo = wave % C::WO;
  const int wt = wave / C::WO;
  const int r16 = lane & 15;
  const int kb = lane >> 4;

  // ---- per-lane source offsets (they depend on the layer: its row pitch and K steps) and per-wave LDS
  // destinations of this wave's loads.  The W piece a load brings is the one of 16-row group (wave + 8 i) of
  // the tile: group and lane are folded into the lane offset, so every load of a stage uses one of three
  // running base pointers.
  uint32_t x_voff[C::X_PW], w_voff[C::A_PW];
  uint32_t x_dst[C::X_PW], a_dst[C::A_PW];
#pragma unroll
  for (int i = 0; i < C::X_PW; ++i) x_dst[i] = (uint32_t)((wave + i * C::NW) * 1024);
#pragma unroll
  for (int i = 0; i < C::A_PW; ++i) a_dst[i] = (uint32_t)(C::X_BYTES + (wave + i * C::NW) * 1024);
  auto layer_offsets = [&](int ldx, int nk) {
#pragma unroll
    for (int i = 0; i < C::X_PW; ++i) {
      const int j = wave + i * C::NW;
      int row, c;
      if (SPARSE) { row = 8 * j + (lane >> 3); c = (lane & 7) ^ (row & 7); }
      else { row = 16 * j + (lane >> 2); c = (lane & 3) ^ ((row >> 1) & 3); }
      x_voff[i] = (uint32_t)((int64_t)row * ldx * C::ES + c * 16);
    }
#pragma unroll
    for (int i = 0; i < C::A_PW; ++i)
      w_voff[i] = ((uint32_t)((wave + i * C::NW) * nk) << 10) + (uint32_t)(lane * 16);  // < 16 * 2^16 * 2^10
  };
  uint32_t s_voff[C::S_PW > 0 ? C::S_PW : 1], s_dst[C::S_PW > 0 ? C::S_PW : 1];
#pragma unroll
  for (int i = 0; i < C::S_PW; ++i) {
    s_voff[i] = (uint32_t)((wave + i * C::NW) * 256 + lane * 4);
    s_dst[i] = (uint32_t)(C::X_BYTES + C::A_BYTES + (wave + i * C::NW) * 256);
  }

  // ---- the block's n-th tile: its layer (tiles come in ascending order, so the search resumes where it
  // stopped), out-feature tile and token rows.  A ragged last token tile is shifted back inside X.
  struct ListPos { int layer, begin; };  // a layer and the XCD-list entry its range starts at
  auto tile_place = [&](int n, ListPos& at, int& o_tile, int64_t& t_lo, int64_t& t0) {
    const int entry = first + n * slots;
    int share = xcd_share(at.layer);
    while (entry >= at.begin + share) {
      at.begin += share;
      share = xcd_share(++at.layer);
    }
    // The table is read at this point of the program and not earlier: a scalar load the compiler starts before
    // the K steps for use after them stays in flight through the steps, and with it in flight every wait for a
    // fragment read has to drain the wave's whole LDS queue (scalar loads return out of order).
    int layer = at.layer;
    asm volatile("" : "+s"(layer));
    const int local = xcd * ((g.layer[layer].n_tiles + 7) >> 3) + (entry - at.begin);
    const int n_o = g.layer[layer].n_o_tiles;
    o_tile = local % n_o;
    t_lo = (int64_t)(local / n_o) * C::BT;
    const int64_t T = g.layer[layer].T;
    t0 = t_lo + C::BT <= T ? t_lo : T - C::BT;
  };

  // ---- load cursor = the stage to be issued next (tile number in this block, k step) as running pointers: X
  // rows of the tile at the step's k, W and selector blocks of the step
  int ld_n = 0, ld_ks = 0, ld_nk = 1, ld_wrap = 1, ld_offsets_of = -1;
  ListPos ld_at{0, 0};
  uint32_t ld_bias_voff = 0;
  int ld_consts = 0;  // nonzero while the cursor's tile still has per-out-feature constants for this wave to fetch
  const float* ld_bias = nullptr;
  const float* ld_scale = nullptr;
  const unsigned char* ld_x = nullptr;
  const unsigned char* ld_w = nullptr;
  const unsigned char* ld_s = nullptr;
  auto cursor_tile = [&](int n) {
    int o_tile;
    int64_t t_lo, t0;
    tile_place(n, ld_at, o_tile, t_lo, t0);
    const int ld_layer = ld_at.layer;
    const StreamLayer& L = g.layer[ld_layer];
    ld_nk = L.nk;
    if (ld_offsets_of != ld_layer) {
      layer_offsets(L.ldx, ld_nk);
      ld_offsets_of = ld_layer;
    }
    ld_x = reinterpret_cast<const unsigned char*>(L.X) + t0 * L.ldx * C::ES;
    ld_w = reinterpret_cast<const unsigned char*>(L.A) + (((int64_t)o_tile * 16 * ld_nk) << 10);
    ld_s = SPARSE ? reinterpret_cast<const unsigned char*>(L.sel) + (int64_t)o_tile * ld_nk * C::S_BYTES : nullptr;
    // bias[o0 + 4 lane ..]: past the last out-feature re-read the last four (never stored)
    const int64_t ob = (int64_t)o_tile * C::BO + lane * 4;
    ld_bias = L.bias;
    ld_scale = L.scale;
    ld_bias_voff = (uint32_t)((ob + 4 <= L.O ? ob : L.O - 4) * 4);
    ld_consts = (wave == 0 && (ld_bias != nullptr || (I8 && ld_scale != nullptr))) ? 1 : 0;
    // The tiles that share the tile's X rows (same tokens, other out-features) run on the same XCD at the
    // same time, and so do a few that share its W rows (same out-features, other tokens); each starts at its
    // own K step and wraps around, so they ask for different slices of those rows at any moment and find the
    // others' slices in L2 instead of missing on them together.
    ld_wrap = ld_nk - (int)((unsigned)(o_tile + (int)(t_lo / C::BT)) % (unsigned)ld_nk);  // steps until the walk wraps to K step 0
    const int64_t k0 = ld_nk - ld_wrap;
    ld_x += k0 * C::X_ROWB;
    ld_w += k0 * 1024;
    if (SPARSE) ld_s += k0 * C::S_BYTES;
    ld_n = n;
    ld_ks = 0;
  };
  auto cursor_advance = [&]() {
    ld_x += C::X_ROWB;
    ld_w += 1024;
    if (SPARSE) ld_s += C::S_BYTES;
    // past the block's last stage the cursor walks the last tile again: the step below then needs no
    // conditions (the surplus stages land in buffers nobody reads any more)
    if (++ld_ks == ld_wrap) {
      ld_x -= (int64_t)ld_nk * C::X_ROWB;
      ld_w -= (int64_t)ld_nk * 1024;
      if (SPARSE) ld_s -= (int64_t)ld_nk * C::S_BYTES;
    }
    if (ld_ks == ld_nk) cursor_tile(ld_n + 1 < my_tiles ? ld_n + 1 : ld_n);
  };
  // the d-th of this wave's LPW loads of the cursor's stage into the stage buffer at LDS offset stage_off
  auto issue_one = [&](auto d_tag, uint32_t stage_off) {
    constexpr int d = decltype(d_tag)::value;
    const uint32_t lds = __builtin_amdgcn_readfirstlane(lds0 + stage_off);
    if constexpr (d == 0) {
      // a tile's first stage brings the tile's bias slice along (older than the stage's own loads, so
      // every wait that covers the stage covers it); slice s belongs to stage buffer s
      if (ld_consts) {  // wave 0 also fetches the tile's per-out-feature constants, once (one test per step)
        ld_consts = 0;
        if constexpr (I8) {
          const uint32_t pair = __builtin_amdgcn_readfirstlane(lds0 + (uint32_t)C::BIAS0 + (uint32_t)(ld_n & 1) * (2 * C::BO * 4));
          if (ld_scale != nullptr) dma16(make_uniform(ld_scale), ld_bias_voff, pair);
          if (ld_bias != nullptr) dma16(make_uniform(ld_bias), ld_bias_voff, pair + C::BO * 4);
        } else if (ld_bias != nullptr) {
          dma16(make_uniform(ld_bias), ld_bias_voff,
                __builtin_amdgcn_readfirstlane(lds0 + (uint32_t)C::BIAS0 + stage_off / (uint32_t)C::STAGE * (C::BO * 4)));
        }
      }
    }
    if constexpr (d < C::X_PW) {
      dma16_at(make_uniform(ld_x), x_voff[d], lds, __builtin_amdgcn_readfirstlane(x_dst[d]));
    } else if constexpr (d < C::X_PW + C::A_PW) {
      constexpr int q = d - C::X_PW;
      dma16_at(make_uniform(ld_w), w_voff[q], lds, __builtin_amdgcn_readfirstlane(a_dst[q]));
    } else {
      constexpr int q = d - C::X_PW - C::A_PW;
      dma4_at(make_uniform(ld_s), s_voff[q], lds, __builtin_amdgcn_readfirstlane(s_dst[q]));
    }
  };
  auto wait_stage = [&](int younger) {
    if (younger >= 2) wait_loads_outstanding<2 * C::LPW>();
    else if (younger == 1) wait_loads_outstanding<C::LPW>();
    else wait_loads_outstanding<0>();
  };

  // ---- fragment readers (the XOR undoes the swizzle applied by the loads).  A lane's four fragment
  // addresses inside a stage buffer (W values, its 16 selector bits, the two halves of an X row) are kept
  // for the current and for the next buffer; the two sets swap roles from step to step, so a step spends
  // four vector additions on addresses and none on moving fragments: vector ALU instructions take issue
  // slots from the matrix instructions of both waves of the SIMD.
  using bfrag_t = std::conditional_t<SPARSE, u32x8_t, u32x4_t>;
  struct FragAddr { uint32_t a, s, xlo, xhi; };  // byte offsets into the dynamic LDS
  FragAddr at0;
  at0.a = (uint32_t)(C::X_BYTES + (wo * C::OW + r16) * C::A_ROWB + ((kb ^ ((r16 >> 1) & 3)) * 16));
  at0.s = (uint32_t)(C::X_BYTES + C::A_BYTES + (I8 ? wo * OT : wo * C::OW / 32) * 256 + r16 * 16 + kb * 4);
  at0.xlo = (uint32_t)((wt * C::TW + r16) * C::X_ROWB + (SPARSE ? ((kb ^ (r16 & 7)) * 16) : ((kb ^ ((r16 >> 1) & 3)) * 16)));
  at0.xhi = (uint32_t)((wt * C::TW + r16) * C::X_ROWB + ((4 + kb) ^ (r16 & 7)) * 16);
  auto frag_addr = [&](uint32_t stage_off) {
    return FragAddr{at0.a + stage_off, at0.s + stage_off, at0.xlo + stage_off, at0.xhi + stage_off};
  };
  // W fragments come in pairs of 16-row blocks: for bfloat16 one selector word serves both (low / high half),
  // for int8 each block has its own word (sv holds the pair)
  constexpr int SV = I8 ? 2 : 1;  // selector registers per pair of blocks
  auto read_a2 = [&](const FragAddr& at, int ip, u32x4_t& av0, u32x4_t& av1, int* sv) {
    av0 = *reinterpret_cast<const u32x4_t*>(smem + at.a + (2 * ip) * 16 * C::A_ROWB);
    av1 = *reinterpret_cast<const u32x4_t*>(smem + at.a + (2 * ip + 1) * 16 * C::A_ROWB);
#pragma unroll
    for (int q = 0; q < SV; ++q)
      sv[q] = SPARSE ? (int)*reinterpret_cast<const uint32_t*>(smem + at.s + (ip * SV + q) * 256) : 0;
  };
  auto read_b = [&](const FragAddr& at, int j, bfrag_t& bv) {
    if constexpr (SPARSE) {
      const u32x4_t lo = *reinterpret_cast<const u32x4_t*>(smem + at.xlo + j * 16 * C::X_ROWB);
      const u32x4_t hi = *reinterpret_cast<const u32x4_t*>(smem + at.xhi + j * 16 * C::X_ROWB);
      bv = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    } else {
      bv = *reinterpret_cast<const u32x4_t*>(smem + at.xlo + j * 16 * C::X_ROWB);
    }
  };

  // ---- prologue: three stages in flight, the first one landed, its first fragments in registers
  // A stage's loads leave LPG at a time (one, when there are as many groups as loads), SPREAD groups apart, from
  // the barrier that frees the buffer (after group TT-3) round to the groups before the next step's barrier:
  // loads d LPG .. d LPG + LPG - 1 after group (TT - 3 + d SPREAD) mod TT.
  // HEAD of them fall into the step that freed the buffer, the others into the next one.  The requests of the
  // eight waves then reach the CU's one load path spread over the step instead of in one burst, behind which
  // every wave's matrix instructions would queue (a wave issues in order).
  constexpr int LPG = (C::LPW + C::TT - 1) / C::TT;                     // loads that leave together
  constexpr int SLOTS = (C::LPW + LPG - 1) / LPG;
  constexpr int SPREAD = 2 * SLOTS <= C::TT ? 2 : 1;
  constexpr int HEAD = ((3 + SPREAD - 1) / SPREAD) * LPG < C::LPW ? ((3 + SPREAD - 1) / SPREAD) * LPG : C::LPW;
  static_assert((SLOTS - 1) * SPREAD < C::TT, "the last load must be out before the next step's wait");
  cursor_tile(0);
#pragma unroll
  for (int s = 0; s < STAGES; ++s) {
    if (s + 1 < STAGES) {
      [&]<int... D>(std::integer_sequence<int, D...>) {
        (issue_one(std::integral_constant<int, D>{}, (uint32_t)(s * C::STAGE)), ...);
      }(std::make_integer_sequence<int, C::LPW>{});
      cursor_advance();
    } else {  // the last one's tail leaves in the first step
      [&]<int... D>(std::integer_sequence<int, D...>) {
        (issue_one(std::integral_constant<int, D>{}, (uint32_t)(s * C::STAGE)), ...);
      }(std::make_integer_sequence<int, HEAD>{});
    }
  }
  wait_loads_outstanding<(STAGES - 2) * C::LPW + HEAD>();
  __builtin_amdgcn_s_barrier();

  u32x4_t afr[2][OT];  // W fragments of the current step and of the next one; the roles alternate
  int sfr[2][OT / 2 * SV];
  FragAddr at[2];      // likewise the fragment addresses in the current and in the next buffer
  bfrag_t bq[4];
  at[0] = at0;
#pragma unroll
  for (int ip = 0; ip < OT / 2; ++ip) read_a2(at[0], ip, afr[0][2 * ip], afr[0][2 * ip + 1], &sfr[0][ip * SV]);
#pragma unroll
  for (int j = 0; j < 3; ++j) read_b(at[0], j, bq[j]);

  uint32_t cur_off = 0;  // LDS offset of the buffer that holds the current stage
  using acc_t = std::conditional_t<I8, i32x4_t, f32x4_t>;
  acc_t acc[OT][TT];

  // One K step, free of conditions: a wave issues one instruction at a time, in order, so every other
  // instruction of the step is time its matrix instructions do not get.  PP names the fragment and address
  // set the step multiplies with.  Every step refills the buffer it has consumed and prefetches fragments
  // of the next stage, also past the block's last stage.
  constexpr int AG = OT > 4 ? 3 : 2;  // groups that fetch the next step's W fragments (all after the barrier)
  auto step = [&](auto pp_tag) {
    constexpr int PP = decltype(pp_tag)::value;
    uint32_t nxt_off = cur_off + C::STAGE;
    if (nxt_off == (uint32_t)(STAGES * C::STAGE)) nxt_off = 0;
    at[PP ^ 1] = frag_addr(nxt_off);
    const uint32_t prev_off = cur_off == 0 ? (uint32_t)((STAGES - 1) * C::STAGE) : cur_off - (uint32_t)C::STAGE;
    [&]<int... J>(std::integer_sequence<int, J...>) {
      ([&] {
        constexpr int j = J;
        if constexpr (j == TT - 3) {
          asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");  // all this wave's reads of the stage are back
          wait_loads_outstanding<(STAGES - 2) * C::LPW>();    // this wave's share of the next stage has landed
          __builtin_amdgcn_s_barrier();
        }
        if constexpr (j + 3 < TT) read_b(at[PP], j + 3, bq[(j + 3) & 3]);
        else read_b(at[PP ^ 1], j + 3 - TT, bq[(j + 3) & 3]);
        if constexpr (j >= TT - AG) {
          // the next step's W fragments, a share in each of the last AG groups
          constexpr int part = j - (TT - AG);
#pragma unroll
          for (int ip = part * (OT / 2) / AG; ip < (part + 1) * (OT / 2) / AG; ++ip)
            read_a2(at[PP ^ 1], ip, afr[PP ^ 1][2 * ip], afr[PP ^ 1][2 * ip + 1], &sfr[PP ^ 1][ip * SV]);
        }
        [&]<int... I>(std::integer_sequence<int, I...>) {
          ([&] {
            constexpr int i = I;
            if constexpr (SPARSE && I8)
              acc[i][j] = __builtin_amdgcn_smfmac_i32_16x16x128_i8(__builtin_bit_cast(i32x4_t, afr[PP][i]),
                                                                   __builtin_bit_cast(i32x8_t, bq[j & 3]), acc[i][j],
                                                                   sfr[PP][i], 0, 0);
            else if constexpr (I8)
              acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(i32x4_t, afr[PP][i]),
                                                                __builtin_bit_cast(i32x4_t, bq[j & 3]), acc[i][j], 0, 0, 0);
            else if constexpr (SPARSE)
              acc[i][j] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(__builtin_bit_cast(bf16x8_t, afr[PP][i]),
                                                                    __builtin_bit_cast(bf16x16_t, bq[j & 3]),
                                                                    acc[i][j], sfr[PP][i / 2], 0, i & 1);
            else
              acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, afr[PP][i]),
                                                                  __builtin_bit_cast(bf16x8_t, bq[j & 3]), acc[i][j],
                                                                  0, 0, 0);
          }(), ...);
        }(std::make_integer_sequence<int, OT>{});
        {
          // the load that leaves after this group, if any: into the buffer this step has consumed (free since the
          // barrier), or the rest of the stage begun in the previous step into the buffer consumed there
          constexpr int since = (j - (TT - 3) + TT) % TT;  // groups since the barrier
          if constexpr (since % SPREAD == 0 && since / SPREAD < SLOTS) {
            [&]<int... Q>(std::integer_sequence<int, Q...>) {
              ([&] {
                constexpr int d = since / SPREAD * LPG + Q;
                if constexpr (d < C::LPW) {
                  issue_one(std::integral_constant<int, d>{}, j >= TT - 3 ? cur_off : prev_off);
                  if constexpr (d == C::LPW - 1) cursor_advance();
                }
              }(), ...);
            }(std::make_integer_sequence<int, LPG>{});
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }(), ...);
    }(std::make_integer_sequence<int, TT>{});
    cur_off = nxt_off;
  };

  ListPos cp_at{0, 0};
  for (int n = 0; n < my_tiles; ++n) {
    int o_tile;
    int64_t t_lo, t0;
    tile_place(n, cp_at, o_tile, t_lo, t0);
    const StreamLayer& L = g.layer[cp_at.layer];
    const int nk = L.nk;
    const int64_t o0 = (int64_t)o_tile * C::BO;
#pragma unroll
    for (int i = 0; i < OT; ++i) {
      if constexpr (I8) {
#pragma unroll
        for (int j = 0; j < TT; ++j) acc[i][j] = i32x4_t{0, 0, 0, 0};
      } else {
        // the accumulators start from the bias, which came with the tile's first stage
        f32x4_t b = f32x4_t{0.f, 0.f, 0.f, 0.f};
        if (L.bias != nullptr)
          b = *reinterpret_cast<const f32x4_t*>(smem + C::BIAS0 + cur_off / (uint32_t)C::STAGE * (C::BO * 4) +
                                                (wo * C::OW + i * 16 + kb * 4) * 4);
#pragma unroll
        for (int j = 0; j < TT; ++j) acc[i][j] = b;
      }
    }

    // The layer's output geometry goes into registers now: read through the table entry after the steps, every
    // store would wait for a scalar load of its own (and for everything else the wave has in flight with it).
    int32_t ldy_s = L.ldy, o_s = L.O, kind_s = L.out_kind;
    uint64_t y_s = reinterpret_cast<uint64_t>(L.Y);
    asm volatile("" : "+s"(ldy_s), "+s"(o_s), "+s"(kind_s), "+s"(y_s));
    // Nothing of this wave's LDS or scalar reads is in flight when the steps begin (it costs nothing here: all of
    // them have just been used); the compiler then counts the fragment reads inside the steps exactly instead of
    // draining the queue at the first waits of every pair of steps.
    __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0) only

    // steps in pairs, so that every tile starts with fragment set 0; an odd count ends with a copy
    for (int ks = 0; ks + 1 < nk; ks += 2) {
      step(std::integral_constant<int, 0>{});
      step(std::integral_constant<int, 1>{});
    }
    if (nk & 1) {
      step(std::integral_constant<int, 0>{});
      at[0] = at[1];
#pragma unroll
      for (int i = 0; i < OT; ++i) afr[0][i] = afr[1][i];
#pragma unroll
      for (int i = 0; i < OT / 2 * SV; ++i) sfr[0][i] = sfr[1][i];
    }
    if (n + 1 == my_tiles) wait_loads_outstanding<0>();  // the surplus stages: nothing in flight when the block ends

    // ---- write the tile out (no LDS memory: the stage ring already holds the next tile).  A lane holds
    // out-features o .. o+3 of token r16 per 16 x 16 block; for bfloat16 two blocks are exchanged between
    // the lane rows kb and kb^1, so that every lane owns 8 consecutive out-features (16 bytes), and a lane
    // permutation then puts the eight pieces of a token row's 128 bytes (the wave's 64 out-features) into eight
    // consecutive lanes: a store instruction is merged only across consecutive lanes, and whole lines leave as
    // single requests.  The stores carry the non-temporal hint: the output is never read back by this kernel, and
    // lines that linger in L2 until write-back push out the X rows the neighbouring tiles still need (with the
    // hint the launch fetches a quarter less; on half lines the same hint costs 40 % more written bytes).
    // int8: the sums are rescaled first, y = fma(float(acc), x_scale * w_scale[o], bias[o]); the tile's scales
    // and bias came with its first stage (pair n mod 2, so the next tile's do not overwrite them)
    f32x4_t sc[I8 ? OT : 1], bi[I8 ? OT : 1];
    if constexpr (I8) {
      const unsigned char* pair = smem + C::BIAS0 + (n & 1) * (2 * C::BO * 4);
#pragma unroll
      for (int i = 0; i < OT; ++i) {
        const int off = (wo * C::OW + i * 16 + kb * 4) * 4;
        sc[i] = f32x4_t{L.x_scale, L.x_scale, L.x_scale, L.x_scale};
        bi[i] = f32x4_t{0.f, 0.f, 0.f, 0.f};
        if (L.scale != nullptr) sc[i] *= *reinterpret_cast<const f32x4_t*>(pair + off);
        if (L.bias != nullptr) bi[i] = *reinterpret_cast<const f32x4_t*>(pair + C::BO * 4 + off);
      }
    }
    auto value = [&](int i, int j) -> f32x4_t {
      if constexpr (I8) {
        f32x4_t y;
#pragma unroll
        for (int e = 0; e < 4; ++e) y[e] = fmaf((float)acc[i][j][e], sc[i][e], bi[i][e]);
        return y;
      } else {
        return acc[i][j];
      }
    };
    // global address space, so that the stores are not counted with the LDS operations
    using gbyte_t = __attribute__((address_space(1))) unsigned char;
    using gpiece_t = __attribute__((address_space(1))) u32x4_t;
    const int first_row = (int)(t_lo - t0);  // rows of a shifted last tile below this one belong to its neighbour
    if (kind_s == 1) {
      // Whole 128-byte lines per store: a wave's 64 out-features are one line of a token row.  The two 16-byte
      // pieces a lane holds for a token block (out-feature pairs 0 and 1, after the exchange between lane rows)
      // are pushed to the lanes that store them: lane 8m + p stores piece p (0..7) of token row m (first store) and
      // of token row m + 8 (second store).
      static_assert(OT % 4 == 0, "a line is two out-feature pairs");
      constexpr int LINES = OT / 4;  // 128-byte lines per token row of the wave
      const int qk = ((kb & 1) << 1) | (kb >> 1);            // place of this lane's piece inside its pair's 64 bytes
      const int hi_rows = r16 >> 3;                          // this lane's token row belongs to the second store
      const int dest_a = (8 * (r16 & 7) + 4 * hi_rows + qk) * 4;
      const int dest_b = (8 * (r16 & 7) + 4 * (1 - hi_rows) + qk) * 4;
      const bool upper = (lane >> 2) & 1;                    // as a storing lane: pieces 4..7 (out-feature pair 1)
      auto swapped = [&](int j, int ip) {  // ip: out-feature pair (blocks 2 ip and 2 ip + 1)
        const f32x4_t v0 = value(2 * ip, j), v1 = value(2 * ip + 1, j);
        const uint32_t a0 = pack_bf16x2(v0[0], v0[1]), a1 = pack_bf16x2(v0[2], v0[3]);
        const uint32_t b0 = pack_bf16x2(v1[0], v1[1]), b1 = pack_bf16x2(v1[2], v1[3]);
        const auto s0 = __builtin_amdgcn_permlane16_swap(a0, b0, false, false);
        const auto s1 = __builtin_amdgcn_permlane16_swap(a1, b1, false, false);
        return u32x4_t{(uint32_t)s0[0], (uint32_t)s1[0], (uint32_t)s0[1], (uint32_t)s1[1]};
      };
      struct Lines { u32x4_t first, second; };
      auto lines_of = [&](int q) {  // q = j * LINES + line
        const int j = q / LINES, h = q % LINES;
        const u32x4_t p0 = swapped(j, 2 * h), p1 = swapped(j, 2 * h + 1);
        u32x4_t ra, rb;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          // rows 0..7 send pair 0 the first way and pair 1 the second way, rows 8..15 the other way round
          const int send_a = hi_rows ? (int)p1[e] : (int)p0[e];
          const int send_b = hi_rows ? (int)p0[e] : (int)p1[e];
          ra[e] = (uint32_t)__builtin_amdgcn_ds_permute(dest_a, send_a);
          rb[e] = (uint32_t)__builtin_amdgcn_ds_permute(dest_b, send_b);
        }
        Lines l;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          l.first[e] = upper ? rb[e] : ra[e];
          l.second[e] = upper ? ra[e] : rb[e];
        }
        return l;
      };
      const int row = wt * C::TW + (lane >> 3);                            // this lane's row of the tile in block j = 0, first store
      const int64_t col = o0 + wo * C::OW + (lane & 7) * 8;              // its out-features in line 0
      gbyte_t* dst = (gbyte_t*)y_s + ((t0 + row) * (int64_t)ldy_s + col) * 2;
      const int64_t half_bytes = (int64_t)ldy_s * 16;                    // 8 token rows further
      bool col_ok[LINES];
#pragma unroll
      for (int h = 0; h < LINES; ++h) col_ok[h] = col + h * 64 < o_s;
      Lines cur = lines_of(0);
#pragma unroll
      for (int q = 0; q < TT * LINES; ++q) {
        const int j = q / LINES, h = q % LINES;
        Lines nxt = cur;
        if (q + 1 < TT * LINES) nxt = lines_of(q + 1);
        if (row + j * 16 >= first_row && col_ok[h]) __builtin_nontemporal_store(cur.first, (gpiece_t*)(dst + h * 128));
        if (row + j * 16 + 8 >= first_row && col_ok[h])
          __builtin_nontemporal_store(cur.second, (gpiece_t*)(dst + half_bytes + h * 128));
        if (h == LINES - 1) dst += 2 * half_bytes;
        cur = nxt;
      }
    } else {
      const int row = wt * C::TW + r16;
      const int64_t col = o0 + wo * C::OW + kb * 4;
      gbyte_t* dst = (gbyte_t*)y_s + ((t0 + row) * (int64_t)ldy_s + col) * 4;
      const int64_t block_bytes = (int64_t)ldy_s * 64;
      bool col_ok[OT];
#pragma unroll
      for (int i = 0; i < OT; ++i) col_ok[i] = col + i * 16 < o_s;
#pragma unroll
      for (int j = 0; j < TT; ++j) {
#pragma unroll
        for (int i = 0; i < OT; ++i) {
          u32x4_t piece;
          if (I8 && kind_s == 2) piece = __builtin_bit_cast(u32x4_t, acc[i][j]);  // the integer sums themselves
          else piece = __builtin_bit_cast(u32x4_t, value(i, j));
          if (row + j * 16 >= first_row && col_ok[i]) *(gpiece_t*)(dst + i * 64) = piece;
        }
        dst += block_bytes;
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

static bool tiles_ok(int64_t K, const void* X, int64_t ldx, const void* values, const void* indices, int64_t O,
                     int64_t T) {
  if (K % 64) return false;
  if (!aligned_to(X, 16) || (ldx % 8)) return false;
  if (!aligned_to(values, 16) || !aligned_to(indices, 8)) return false;
  if (O > (1 << 24) || T >= (1ll << 31)) return false;
  if (ldx > (1 << 22) || K > (1 << 22)) return false;  // per-lane byte offsets inside a tile stay below 2^32
  return true;
}

// Which product kernel a layer of O out-features runs at T tokens: 0 = the persistent 256 x 256 kernel, 2 = the
// tiled kernel with 128 x 128 tiles, 3 = with 64 x 64 tiles.  The choice is the smaller of two estimated durations
// (microseconds), a model fitted to measured launches on DeiT- and Swin-shaped layers (28 shapes from 197 to 50176
// tokens; it picks the faster kernel on 27 of them and loses 19 % on the other):
//   persistent: one block per compute unit walks ceil(tiles / 256) tiles of `stream_steps` K steps each, about
//               0.7 us per step plus 4.5 us to write a tile out, plus the launch;
//   tiled:      a compute unit works through ceil(tiles / 256) tiles of 128 x 128 (one after the other or two at
//               a time, the rate per unit is the same), `tiled_step_us` per K step of 64 (0.34 us in the 2:4
//               form, 0.5 us in the dense form, whose step holds twice the matrix instructions).
// A layer with fewer than 64 tiles of 128 x 128 takes 64 x 64 tiles: the few tiles there are finish sooner.
static int pick_tile(int64_t O, int64_t T, int64_t stream_steps, int64_t tiled_steps, double tiled_step_us) {
  const int64_t tiles_big = ((O + 255) / 256) * ((T + 255) / 256);
  const int64_t tiles_mid = ((O + 127) / 128) * ((T + 127) / 128);
  if (tiles_mid < 64) return 3;
  if (T < 256) return 2;
  const double est_stream = (double)((tiles_big + 255) / 256) * ((double)stream_steps * 0.7 + 4.5) + 4.0;
  const double est_tiled = (double)((tiles_mid + 255) / 256) * ((double)tiled_steps * tiled_step_us + 1.5) + 3.0;
  return est_stream <= est_tiled ? 0 : 2;
}
static int pick_tile(int64_t O, int64_t K, int64_t T, bool sparse_form) {
  return pick_tile(O, T, sparse_form ? K / 64 : K / 32, K / 64, sparse_form ? 0.34 : 0.5);
}

// The form in which the product kernels read a layer's weight at T tokens.
//   FORM_PACKED  as packed: the gather kernel (K % 64 != 0), or the tiled kernel at 2:4 and at N = M, whose packed
//                layouts already are the row-major 2:4 / dense operands
//   FORM_STREAM  stream order in the workspace (2:4 form for N <= 2, dense form otherwise): every other level, and
//                every level on the persistent kernel
enum { FORM_PACKED = 0, FORM_STREAM = 1 };
static int operand_form(int64_t O, int64_t K, int64_t T, int N, int M, bool* sparse_form) {
  *sparse_form = N <= 2 && N < M;
  if (K % 64) return FORM_PACKED;
  const bool as_packed = (N == 2 && M == 4) || N == M;
  return (pick_tile(O, K, T, *sparse_form) != 0 && as_packed) ? FORM_PACKED : FORM_STREAM;
}

bool spmm_stream_order(int64_t O, int64_t K, int64_t T, int N, int M, bool* sparse_form) {
  return operand_form(O, K, T, N, M, sparse_form) == FORM_STREAM;
}

// Ranges the reduction of a layer on the tiled kernel is cut into: a layer with far fewer tiles than the chip has
// compute units and a long K (one image through a wide MLP: 197 tokens, K = 3072) leaves most units idle for many
// steps; cut into ranges of at least 12 steps, it fills them, at the price of fp32 partial sums through memory and
// a reduce launch (about 5 us: below 64 steps the cut gains nothing; measured on ViT-S .. ViT-H shaped layers).
// A function of the shape alone.
static int split_count(int64_t O, int64_t K, int64_t T, bool sparse_form) {
  if (K % 64) return 1;
  const int pick = pick_tile(O, K, T, sparse_form);
  if (pick == 0) return 1;
  const int64_t side = pick == 2 ? 128 : 64;
  const int64_t tiles = ((O + side - 1) / side) * ((T + side - 1) / side);
  const int64_t steps = K / 64;
  if (tiles >= 128 || steps < 64) return 1;
  int64_t n = 256 / tiles;
  if (n > steps / 12) n = steps / 12;
  if (n > 8) n = 8;
  while (n > 1 && (n - 1) * ((steps + n - 1) / n) >= steps) --n;  // no empty range
  return n < 2 ? 1 : (int)n;
}
static size_t operand_bytes(int64_t O, int64_t K, int N, int M, int64_t T, bool* sparse_form) {
  if (operand_form(O, K, T, N, M, sparse_form) != FORM_STREAM) return 0;
  const size_t o_pad = (size_t)((O + 255) / 256) * 256;  // whole 256-row tiles
  return *sparse_form ? o_pad * (size_t)K + o_pad * (size_t)K / 8 : o_pad * (size_t)K * 2;
}

// The part of the workspace a product cannot do without: the operand-order copy.  With no more than that the
// reduction stays in one piece.
size_t spmm_operand_workspace_bytes(int64_t O, int64_t K, int N, int M, int64_t T) {
  bool sparse_form = false;
  return operand_bytes(O, K, N, M, T, &sparse_form);
}

// Workspace of a product: the operand-order copy (if the level needs one), then the partial sums of a cut reduction.
size_t spmm_workspace_bytes(int64_t O, int64_t K, int N, int M, int64_t T) {
  bool sparse_form = false;
  const size_t operand = operand_bytes(O, K, N, M, T, &sparse_form);
  const int splits = split_count(O, K, T, sparse_form);
  if (splits < 2) return operand;
  return ((operand + 255) / 256) * 256 + (size_t)splits * (size_t)T * (size_t)O * 4;
}

// The reduce launch of layers whose reduction was cut: split_group_append lists a layer (false: table full),
// launch_split_reduce adds their partial sums up.
static bool split_group_append(SplitGroup& sg, const GemmArgs& g) {
  if (sg.count >= kSplitLayersMax) return false;
  const int64_t quads = g.T * ((g.O + 3) / 4);
  const int64_t first = sg.count ? sg.layer[sg.count - 1].block_end : 0;
  if (first + (quads + 255) / 256 > 0x7FFFFFF0) return false;
  SplitLayer& L = sg.layer[sg.count++];
  L.partial = g.partial; L.bias = g.bias; L.Y = g.Y; L.ldy = g.ldy;
  L.T = (int32_t)g.T; L.O = (int32_t)g.O; L.splits = g.splits; L.out_bf16 = g.out_bf16;
  L.block_end = (uint32_t)(first + (quads + 255) / 256);
  L.vec = (g.O % 4 == 0) && (g.ldy % 4 == 0) && aligned_to(g.Y, g.out_bf16 ? 8 : 16);
  return true;
}
static hipError_t launch_split_reduce(SplitGroup& sg, hipStream_t s) {
  if (sg.count == 0) return hipSuccess;
  hipLaunchKernelGGL(splitk_reduce_kernel, dim3(sg.layer[sg.count - 1].block_end), dim3(256), 0, s, sg);
  sg.count = 0;
  return hipGetLastError();
}

template <bool SPARSE, int WO, int WT, int OT, int TT, int STAGES>
static hipError_t launch_gemm(GemmArgs g, hipStream_t s) {
  using C = GemmCfg<SPARSE, WO, WT, OT, TT, STAGES>;
  auto kern = nm_gemm_kernel<SPARSE, WO, WT, OT, TT, STAGES>;
  static PerDeviceOnce lds_limit;
  if (hipError_t e = raise_dynamic_lds_limit(kern, C::LDS_BYTES, lds_limit); e != hipSuccess) return e;
  g.n_o_tiles = (int)((g.O + C::BO - 1) / C::BO);
  g.n_t_tiles = (int)((g.T + C::BT - 1) / C::BT);
  const int64_t n_units = (int64_t)g.n_o_tiles * g.n_t_tiles * (g.splits > 1 ? g.splits : 1);
  const int64_t grid = ((n_units + 7) / 8) * 8;
  if (grid > 0x7FFFFFFF) return hipErrorInvalidValue;
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(C::NT), C::LDS_BYTES, s, g);
  if (hipError_t e = hipGetLastError(); e != hipSuccess) return e;
  if (g.splits > 1) {
    SplitGroup sg;
    sg.count = 0;
    split_group_append(sg, g);
    return launch_split_reduce(sg, s);
  }
  return hipSuccess;
}

// Tiled kernel, many layers in one launch.  tile_group_append fills the table (false: full, launch it and retry;
// a layer with more blocks than a grid holds never fits and is launched alone).
template <int BO, int BT>
static int64_t tile_layer_blocks(const TileLayer& L) {
  const int64_t tiles = (int64_t)((L.O + BO - 1) / BO) * ((L.T + BT - 1) / BT);
  return ((tiles * (L.splits > 1 ? L.splits : 1) + 7) / 8) * 8;
}
// estimated duration of one of the layer's blocks (the model of pick_tile): the order of the launch
static double tile_layer_cost(const TileLayer& L) {
  const int n = L.splits > 1 ? L.splits : 1;
  return (double)((L.K / 64 + n - 1) / n) * (L.sparse_form ? 0.34 : 0.5);
}

template <int WO, int WT, int OT, int TT>
static bool tile_group_append(TileGroup& grp, const GemmArgs& g, bool sparse_form) {
  if (grp.count >= kTileLayersMax) return false;
  TileLayer& L = grp.layer[grp.count];
  L.A = g.A; L.sel = g.sel; L.X = g.X; L.bias = g.bias; L.Y = g.Y; L.partial = g.partial;
  L.ldy = g.ldy;
  L.O = (uint32_t)g.O; L.K = (uint32_t)g.K; L.T = (uint32_t)g.T;   // tiles_ok has bounded them
  L.ldx = (uint32_t)g.ldx; L.out_bf16 = g.out_bf16; L.vec_store = g.vec_store; L.stream_form = g.stream_form;
  L.sparse_form = sparse_form; L.splits = g.splits > 1 ? g.splits : 1;
  L.block_end = 0; L.rot = 0;
  int64_t total = tile_layer_blocks<WO * OT * 16, WT * TT * 16>(L);
  for (int i = 0; i < grp.count; ++i) total += tile_layer_blocks<WO * OT * 16, WT * TT * 16>(grp.layer[i]);
  if (total > 0x7FFFFFF0) return false;
  ++grp.count;
  return true;
}

template <int WO, int WT, int OT, int TT, int SS, int SD>
static hipError_t launch_gemm_group(TileGroup& grp, hipStream_t s) {
  using CS = GemmCfg<true, WO, WT, OT, TT, SS>;
  using CD = GemmCfg<false, WO, WT, OT, TT, SD>;
  constexpr int LDS = CS::LDS_BYTES > CD::LDS_BYTES ? CS::LDS_BYTES : CD::LDS_BYTES;
  if (grp.count == 0) return hipSuccess;
  auto kern = nm_gemm_group_kernel<WO, WT, OT, TT, SS, SD>;
  static PerDeviceOnce lds_limit;
  if (hipError_t e = raise_dynamic_lds_limit(kern, LDS, lds_limit); e != hipSuccess) return e;
  // longest blocks first (insertion sort, stable), so that the launch ends with the shortest ones
  for (int i = 1; i < grp.count; ++i) {
    const TileLayer L = grp.layer[i];
    const double cost = tile_layer_cost(L);
    int j = i;
    for (; j > 0 && tile_layer_cost(grp.layer[j - 1]) < cost; --j) grp.layer[j] = grp.layer[j - 1];
    grp.layer[j] = L;
  }
  // A layer's blocks are a whole multiple of 8, one share per XCD; the last shares are short or empty.  Each layer
  // turns its shares against the XCDs so that the estimated work per XCD stays as even as the list allows.
  uint32_t end = 0;
  double load[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int i = 0; i < grp.count; ++i) {
    TileLayer& L = grp.layer[i];
    const int64_t blocks = tile_layer_blocks<CS::BO, CS::BT>(L);
    const int64_t per_xcd = blocks / 8;
    const int64_t units = (int64_t)((L.O + CS::BO - 1) / CS::BO) * ((L.T + CS::BT - 1) / CS::BT) * L.splits;
    const double cost = tile_layer_cost(L) + 2.0;  // plus a block's start and write-out
    double share[8];
    for (int sl = 0; sl < 8; ++sl) {
      int64_t u = units - sl * per_xcd;
      u = u < 0 ? 0 : (u > per_xcd ? per_xcd : u);
      share[sl] = cost * (double)u;
    }
    int best = 0;
    double best_sq = 0;  // the turn that leaves the sum of squared loads smallest
    for (int rot = 0; rot < 8; ++rot) {
      double sq = 0;
      for (int x = 0; x < 8; ++x) {
        const double v = load[x] + share[(x + rot) & 7];
        sq += v * v;
      }
      if (rot == 0 || sq < best_sq) { best = rot; best_sq = sq; }
    }
    for (int x = 0; x < 8; ++x) load[x] += share[(x + best) & 7];
    L.rot = (uint32_t)best;
    end += (uint32_t)blocks;
    L.block_end = end;
  }
  hipLaunchKernelGGL(kern, dim3(end), dim3(CS::NT), LDS, s, grp);
  grp.count = 0;
  return hipGetLastError();
}

template <bool SPARSE, bool I8 = false>
static hipError_t launch_stream_group(const StreamGroup& grp, hipStream_t s) {
  constexpr int WO = I8 ? 4 : kStreamWO, WT = I8 ? 2 : kStreamWT;
  using C = StreamCfg<SPARSE, WO, WT, SPARSE ? 3 : 4, I8>;  // dense stages are half the size: four fit
  auto kern = nm_stream_kernel<SPARSE, WO, WT, SPARSE ? 3 : 4, I8>;
  static PerDeviceOnce lds_limit;
  if (hipError_t e = raise_dynamic_lds_limit(kern, C::LDS_BYTES, lds_limit); e != hipSuccess) return e;
  int cus = 0;
  if (hipError_t e = compute_units(&cus); e != hipSuccess) return e;
  const int n_cu = cus > 8 ? (cus / 8) * 8 : 8;
  const int64_t want = (((int64_t)grp.n_tiles + 7) / 8) * 8;
  const int64_t resident = (int64_t)n_cu * C::PER_CU;  // persistent blocks: as many as fit at once
  const unsigned grid = (unsigned)(want < resident ? want : resident);
  hipLaunchKernelGGL(kern, dim3(grid), dim3(C::NT), C::LDS_BYTES, s, grp);
  return hipGetLastError();
}

// Appends a layer to the table of a launch; false when its tiles would overflow the list.
template <bool SPARSE>
static bool group_append(StreamGroup& grp, const GemmArgs& g) {
  using C = StreamCfg<SPARSE, kStreamWO, kStreamWT, SPARSE ? 3 : 4>;
  const int64_t n_o = (g.O + C::BO - 1) / C::BO, n_t = (g.T + C::BT - 1) / C::BT;
  const int64_t end = (int64_t)grp.n_tiles + n_o * n_t;
  if (grp.count >= kStreamLayersMax || end > 0x7FFFFFF0) return false;
  StreamLayer& L = grp.layer[grp.count++];
  L.A = g.A; L.sel = g.sel; L.X = g.X; L.bias = g.bias; L.scale = nullptr; L.Y = g.Y;
  L.O = (int32_t)g.O; L.T = (int32_t)g.T; L.nk = (int32_t)(g.K / C::KSTEP);
  L.ldx = (int32_t)g.ldx; L.ldy = (int32_t)g.ldy;
  L.n_o_tiles = (int32_t)n_o;
  L.n_tiles = (int32_t)(n_o * n_t);
  L.x_scale = 1.f; L.out_kind = g.out_bf16 ? 1 : 0; L.reserved = 0;
  grp.n_tiles = (int32_t)end;
  return true;
}

template <bool SPARSE>
static hipError_t launch_stream(const GemmArgs& g, hipStream_t s) {
  StreamGroup grp;
  grp.count = 0; grp.n_tiles = 0;
  if (!group_append<SPARSE>(grp, g)) return hipErrorInvalidValue;
  return launch_stream_group<SPARSE>(grp, s);
}

// The int8 layer on the persistent kernel.  The operands are in stream order (see nm_int8.hip's pre-pass).
bool stream_i8_takes(int64_t O, int64_t K, int64_t T, int N, int M) {
  const bool sparse_form = N <= 2 && N < M;
  const int64_t kstep = sparse_form ? 128 : 64;
  // the per-tile constants alternate between two LDS slices, which needs tiles of at least three steps
  return pick_tile(O, T, K / kstep, K / 128, sparse_form ? 0.5 : 1.0) == 0 && K % kstep == 0 && K / kstep >= 3 && O <= (1 << 24) && T < (1ll << 31) && K <= (1 << 22);
}

hipError_t launch_stream_i8(const StreamI8Args& a, hipStream_t s) {
  StreamGroup grp;
  grp.count = 1;
  StreamLayer& L = grp.layer[0];
  const int64_t kstep = a.sparse_form ? 128 : 64;
  const int64_t n_o = (a.O + 255) / 256, n_t = (a.T + 255) / 256;
  if (n_o * n_t > 0x7FFFFFF0) return hipErrorInvalidValue;
  L.A = reinterpret_cast<const bf16_t*>(a.values); L.sel = a.sel; L.X = reinterpret_cast<const bf16_t*>(a.X);
  L.bias = a.bias; L.scale = a.w_scale; L.Y = a.Y;
  L.O = (int32_t)a.O; L.T = (int32_t)a.T; L.nk = (int32_t)(a.K / kstep);
  L.ldx = (int32_t)a.ldx; L.ldy = (int32_t)a.ldy;
  L.n_o_tiles = (int32_t)n_o; L.n_tiles = (int32_t)(n_o * n_t);
  L.x_scale = a.x_scale; L.out_kind = a.out_kind; L.reserved = 0;
  grp.n_tiles = L.n_tiles;
  return a.sparse_form ? launch_stream_group<true, true>(grp, s) : launch_stream_group<false, true>(grp, s);
}

template <bool SPARSE>
static hipError_t dispatch_gemm(const GemmArgs& g, int pick, hipStream_t s) {
  switch (pick) {
    case 0: return launch_stream<SPARSE>(g, s);
    case 2:
      // dense form with more tiles than compute units: two LDS stages instead of three, so that two blocks share
      // a compute unit and one's loads and write-out run under the other's matrix instructions (0.6 - 0.9 of the
      // three-stage time on such shapes; with a block per unit the deeper pipeline wins)
      if (!SPARSE && ((g.O + 127) / 128) * ((g.T + 127) / 128) > 256) return launch_gemm<SPARSE, 2, 2, 4, 4, 2>(g, s);
      return launch_gemm<SPARSE, 2, 2, 4, 4, 3>(g, s);
    default: return launch_gemm<SPARSE, 2, 2, 2, 2, 3>(g, s);
  }
}

static hipError_t launch_general(const SpmmArgs& a, hipStream_t s) {
  const int64_t n_o_tiles = (a.O + 15) / 16, n_t_tiles = (a.T + 15) / 16;
  if (n_o_tiles * n_t_tiles > 0x7FFFFFFF) return hipErrorInvalidValue;
  hipLaunchKernelGGL(spmm_general_kernel, dim3((unsigned)(n_o_tiles * n_t_tiles)), dim3(256), 0, s, a.values, a.indices,
                     a.O, a.K, a.N, a.M, a.X, a.T, a.ldx, a.bias, a.Y, a.ldy, a.out_bf16, n_o_tiles);
  return hipGetLastError();
}

// Out[t, i] = sum_r Q[t, r] * Ws[r, i] on the persistent dense kernel: the weight is written transposed into
// stream order first (a pass over the weight only), then it is an ordinary product with I out-features and a
// reduction of R.  Shapes: enough 256 x 256 tiles, R % 64 == 0, Out rows in whole aligned 16-byte pieces.
size_t dense_transposed_workspace_bytes(int64_t R, int64_t I, int64_t T) {
  if ((R % 64) || pick_tile(I, R, T, false) != 0) return 0;
  return (size_t)(((I + 255) / 256) * 256) * (size_t)R * 2;
}

hipError_t launch_dense_transposed(const bf16_t* Ws, int64_t R, int64_t I, int64_t ldw, const bf16_t* Q, int64_t T,
                                   int64_t ldq, void* Out, int64_t ldo, int out_bf16, void* workspace,
                                   size_t workspace_bytes, hipStream_t s, bool* taken) {
  *taken = false;
  const size_t need = dense_transposed_workspace_bytes(R, I, T);
  const int per_piece = out_bf16 ? 8 : 4;
  if (!need || workspace == nullptr || workspace_bytes < need || !aligned_to(workspace, 256)) return hipSuccess;
  if (!aligned_to(Q, 16) || (ldq % 8) || !aligned_to(Ws, 2) || (ldo % per_piece) || !aligned_to(Out, 16) || (I % per_piece))
    return hipSuccess;
  if (I > (1 << 24) || T >= (1ll << 31) || ldq > (1 << 22) || R > (1 << 22) || ldo > 0x7FFFFFFF) return hipSuccess;
  const int64_t i_pad = ((I + 255) / 256) * 256;
  const int64_t n = i_pad * (R / 8);
  hipLaunchKernelGGL(transpose_stream_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, Ws, R, I, ldw, i_pad,
                     reinterpret_cast<unsigned char*>(workspace));
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  GemmArgs g;
  g.A = reinterpret_cast<const bf16_t*>(workspace); g.sel = nullptr;
  g.X = Q; g.bias = nullptr; g.Y = Out;
  g.O = I; g.K = R; g.T = T; g.ldx = ldq; g.ldy = ldo;
  g.n_o_tiles = g.n_t_tiles = 0;
  g.out_bf16 = (uint8_t)out_bf16; g.vec_store = 1; g.stream_form = 1; g.splits = 1; g.partial = nullptr;
  *taken = true;
  return dispatch_gemm<false>(g, 0, s);
}

// The stream-order pre-pass of a layer into its workspace.
static hipError_t launch_stream_prepass(const SpmmArgs& a, bool sparse_form, hipStream_t s) {
  unsigned char* ws = reinterpret_cast<unsigned char*>(a.workspace);
  const int64_t o_pad = ((a.O + 255) / 256) * 256;
  if (sparse_form) {
    unsigned char* sel_s = ws + (size_t)o_pad * (size_t)a.K;
    const int64_t n = o_pad * (a.K / 32);
    const dim3 grid((unsigned)((n + 255) / 256));
    switch (a.N * 32 + a.M) {
#define X(n_, m_)                                                                                              \
  case n_ * 32 + m_:                                                                                           \
    hipLaunchKernelGGL((recode_stream_kernel<n_, m_>), grid, dim3(256), 0, s, a.values, a.indices, a.O, o_pad, a.K, \
                       ws, sel_s);                                                                             \
    break;
      X(1, 4) X(2, 4) X(1, 8) X(2, 8) X(1, 16) X(2, 16)
#undef X
      default: return hipErrorInvalidValue;
    }
  } else {
    const int64_t n = o_pad * (a.K / 8);
    hipLaunchKernelGGL(expand_stream_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, a.values, a.indices,
                       a.O, o_pad, a.K, a.N, a.M, ws);
  }
  return hipGetLastError();
}

// Operands of the matrix-core kernels for a layer whose form is known.
static void fill_gemm_args(const SpmmArgs& a, int form, bool sparse_form, GemmArgs* g) {
  g->X = a.X; g->bias = a.bias; g->Y = a.Y;
  g->O = a.O; g->K = a.K; g->T = a.T; g->ldx = a.ldx; g->ldy = a.ldy;
  g->out_bf16 = a.out_bf16;
  g->n_o_tiles = g->n_t_tiles = 0;
  g->rot = 0;
  // 16-byte pieces of Y rows: every row start and the row end fall on a piece boundary
  const int per_piece = a.out_bf16 ? 8 : 4;
  g->vec_store = (a.ldy % per_piece == 0) && aligned_to(a.Y, 16) && (a.O % per_piece == 0) &&
                 (a.bias == nullptr || aligned_to(a.bias, 16));
  g->stream_form = form == FORM_STREAM;
  {
    bool sf = false;
    const size_t operand = operand_bytes(a.O, a.K, a.N, a.M, a.T, &sf);
    int splits = split_count(a.O, a.K, a.T, sparse_form);
    // the partial sums need the full workspace; a caller that brings the operand part only gets the uncut product
    if (splits > 1 && (a.workspace == nullptr || !aligned_to(a.workspace, 256) ||
                       a.workspace_bytes < ((operand + 255) / 256) * 256 + (size_t)splits * (size_t)a.T * (size_t)a.O * 4))
      splits = 1;
    g->splits = (uint8_t)splits;
    g->partial = splits > 1 ? reinterpret_cast<float*>(reinterpret_cast<unsigned char*>(a.workspace) +
                                                       ((operand + 255) / 256) * 256)
                            : nullptr;
  }
  if (form == FORM_STREAM) {
    const int64_t o_pad = ((a.O + 255) / 256) * 256;
    unsigned char* ws = reinterpret_cast<unsigned char*>(a.workspace);
    g->A = reinterpret_cast<const bf16_t*>(ws);
    g->sel = sparse_form ? reinterpret_cast<const uint32_t*>(ws + (size_t)o_pad * (size_t)a.K) : nullptr;
  } else {
    g->A = a.values;  // 2:4: values + index words are the row-major 2:4 operand; N = M: the dense weight
    g->sel = sparse_form ? a.indices : nullptr;
  }
}

// A layer whose operand-order workspace is missing (or too small) and which the few-token kernel can multiply
// from the packed format instead.
static bool packed_path(const SpmmArgs& a) {
  if (!tiles_ok(a.K, a.X, a.ldx, a.values, a.indices, a.O, a.T)) return false;
  const size_t need = spmm_operand_workspace_bytes(a.O, a.K, a.N, a.M, a.T);
  if (!need || (a.workspace != nullptr && a.workspace_bytes >= need && aligned_to(a.workspace, 256))) return false;
  return fewtok_takes(a);
}

hipError_t launch_spmm(const SpmmArgs& a, hipStream_t s, bool* workspace_short, int phases) {
  *workspace_short = false;
  const bool prepare = phases & SPMM_PREPARE, product = phases & SPMM_PRODUCT;
  if (!tiles_ok(a.K, a.X, a.ldx, a.values, a.indices, a.O, a.T)) {
    if (!product) return hipSuccess;  // the gather kernel reads the packed layout itself
    return launch_general(a, s);
  }
  bool sparse_form = false;
  const int form = operand_form(a.O, a.K, a.T, a.N, a.M, &sparse_form);
  const size_t need = spmm_operand_workspace_bytes(a.O, a.K, a.N, a.M, a.T);
  if (need && (a.workspace == nullptr || a.workspace_bytes < need || !aligned_to(a.workspace, 256))) {
    // no workspace: few tokens can still be multiplied straight from the packed format
    if (!packed_path(a)) *workspace_short = true;
    else if (product) {
      const SpmmArgs* one = &a;
      return launch_fewtok(&one, 1, s);
    }
    return hipSuccess;
  }
  const int pick = pick_tile(a.O, a.K, a.T, sparse_form);
  GemmArgs g;
  fill_gemm_args(a, form, sparse_form, &g);
  // the persistent kernel writes Y in 16-byte pieces only; other outputs go to the gather kernel, which reads the
  // packed layout itself
  const bool gather = pick == 0 && (!g.vec_store || a.ldy > 0x7FFFFFFF);
  if (prepare && form == FORM_STREAM && !(gather && product)) {
    hipError_t e = launch_stream_prepass(a, sparse_form, s);
    if (e != hipSuccess) return e;
  }
  if (!product) return hipSuccess;
  if (gather) return launch_general(a, s);
  return sparse_form ? dispatch_gemm<true>(g, pick, s) : dispatch_gemm<false>(g, pick, s);
}

// The product of a prepared layer on the tiled kernel, as a table entry (the operands launch_spmm would hand the
// kernel): false when the layer takes another path.
static bool tiled_entry(const SpmmArgs& a, GemmArgs* g, bool* sparse_form, int* pick) {
  if (packed_path(a)) return false;
  if (!tiles_ok(a.K, a.X, a.ldx, a.values, a.indices, a.O, a.T)) return false;
  const int form = operand_form(a.O, a.K, a.T, a.N, a.M, sparse_form);
  *pick = pick_tile(a.O, a.K, a.T, *sparse_form);
  if (*pick == 0) return false;
  fill_gemm_args(a, form, *sparse_form, g);
  return true;
}

// The product of a prepared layer on the persistent kernel, as a table entry: false when this layer takes
// another path (too few tiles, a shape or alignment the kernel does not handle).
static bool stream_entry(const SpmmArgs& a, GemmArgs* g, bool* sparse_form) {
  if (packed_path(a)) return false;
  if (!tiles_ok(a.K, a.X, a.ldx, a.values, a.indices, a.O, a.T)) return false;
  const int form = operand_form(a.O, a.K, a.T, a.N, a.M, sparse_form);
  if (pick_tile(a.O, a.K, a.T, *sparse_form) != 0) return false;
  fill_gemm_args(a, form, *sparse_form, g);
  if (!g->vec_store || a.ldy > 0x7FFFFFFF) return false;
  return true;
}

bool spmm_workspace_short(const SpmmArgs& a) {
  if (packed_path(a)) return false;
  if (!tiles_ok(a.K, a.X, a.ldx, a.values, a.indices, a.O, a.T)) return false;  // the gather kernel needs none
  const size_t need = spmm_operand_workspace_bytes(a.O, a.K, a.N, a.M, a.T);
  return need && (a.workspace == nullptr || a.workspace_bytes < need || !aligned_to(a.workspace, 256));
}

// LDS stages of the dense-form 128 x 128 tiles in a shared launch: two (64 KB) instead of three (96 KB) keep the
// launch's LDS at the 2:4 form's 75 KB, so that two blocks share a compute unit (48 layers at 197 tokens: 62 us
// against 70 us with three).
constexpr int kGroupDenseStages = 2;

// Products of many prepared layers: those the persistent kernel takes share launches (one table per operand form,
// flushed when full), the small ones share one launch of the tiled kernel per tile size (both forms together),
// few-token layers without a workspace one launch of the packed-format kernel; what is left is launched alone.
hipError_t launch_spmm_batched(const SpmmArgs* layers, int count, hipStream_t s) {
  StreamGroup sparse_grp, dense_grp;
  sparse_grp.count = dense_grp.count = 0;
  sparse_grp.n_tiles = dense_grp.n_tiles = 0;
  hipError_t e = hipSuccess;
  auto flush = [&](StreamGroup& grp, bool sparse) {
    if (grp.count == 0) return hipSuccess;
    // Deepest layers first (insertion sort, stable): the blocks take the list in order, so the launch then ends
    // with the cheapest tiles and its last, partly filled round is as short as the list allows.
    for (int i = 1; i < grp.count; ++i) {
      const StreamLayer L = grp.layer[i];
      int j = i;
      for (; j > 0 && grp.layer[j - 1].nk < L.nk; --j) grp.layer[j] = grp.layer[j - 1];
      grp.layer[j] = L;
    }
    const hipError_t r = sparse ? launch_stream_group<true>(grp, s) : launch_stream_group<false>(grp, s);
    grp.count = 0; grp.n_tiles = 0;
    return r;
  };
  SplitGroup split_grp;
  split_grp.count = 0;
  TileGroup tile_grp[2];  // 128 x 128 and 64 x 64 tiles, both operand forms in each
  for (TileGroup& t : tile_grp) t.count = 0;
  auto tile_append = [&](int which, const GemmArgs& g, bool sparse_form) {
    return which == 0 ? tile_group_append<2, 2, 4, 4>(tile_grp[0], g, sparse_form)
                      : tile_group_append<2, 2, 2, 2>(tile_grp[1], g, sparse_form);
  };
  auto tile_flush = [&](int which) {
    return which == 0 ? launch_gemm_group<2, 2, 4, 4, 3, kGroupDenseStages>(tile_grp[0], s)
                      : launch_gemm_group<2, 2, 2, 2, 3, 3>(tile_grp[1], s);
  };
  // A layer alone takes 64 x 64 tiles when 128 x 128 ones would leave most compute units idle; the layers of a
  // call fill the chip together, so they take the larger tiles (half the operand traffic into the compute
  // units per output) as soon as the call holds enough of them.  A sum is accumulated in the same order under
  // either tile size, so the outputs are the same bytes.
  int64_t mid_tiles = 0;
  for (int i = 0; i < count; ++i) {
    GemmArgs g;
    bool sparse_form = false;
    int pick = 0;
    if (tiled_entry(layers[i], &g, &sparse_form, &pick))
      mid_tiles += ((layers[i].O + 127) / 128) * ((layers[i].T + 127) / 128);
  }
  const bool promote = mid_tiles >= 256;
  // few tokens and no workspace: all such layers of the call in one launch of the kernel that reads the packed format
  {
    constexpr int kChunk = 64;
    const SpmmArgs* few[kChunk];
    int n_few = 0;
    for (int i = 0; i < count; ++i) {
      if (!packed_path(layers[i])) continue;
      few[n_few++] = &layers[i];
      if (n_few == kChunk) {
        if ((e = launch_fewtok(few, n_few, s)) != hipSuccess) return e;
        n_few = 0;
      }
    }
    if (n_few && (e = launch_fewtok(few, n_few, s)) != hipSuccess) return e;
  }
  for (int i = 0; i < count; ++i) {
    GemmArgs g;
    bool sparse_form = false;
    if (packed_path(layers[i])) continue;
    if (stream_entry(layers[i], &g, &sparse_form)) {
      StreamGroup& grp = sparse_form ? sparse_grp : dense_grp;
      bool ok = sparse_form ? group_append<true>(grp, g) : group_append<false>(grp, g);
      if (!ok) {
        if ((e = flush(grp, sparse_form)) != hipSuccess) return e;
        ok = sparse_form ? group_append<true>(grp, g) : group_append<false>(grp, g);
        if (!ok) return hipErrorInvalidValue;
      }
    } else if (int pick = 0; tiled_entry(layers[i], &g, &sparse_form, &pick)) {
      // small layers: the tiled kernel, all layers of one operand form and tile size in one launch
      const int which = (pick == 2 || promote) ? 0 : 1;
      // a call that fills the chip with whole tiles has no use for cut reductions (their partial sums would only
      // add traffic and a launch): such a call's sums differ from the single calls' in rounding order only
      if (promote) { g.splits = 1; g.partial = nullptr; }
      bool listed = tile_append(which, g, sparse_form);
      if (!listed) {
        if ((e = tile_flush(which)) != hipSuccess) return e;
        listed = tile_append(which, g, sparse_form);
        if (!listed) {  // more blocks than a grid holds: alone
          bool short_ws = false;
          if ((e = launch_spmm(layers[i], s, &short_ws, SPMM_PRODUCT)) != hipSuccess) return e;
        }
      }
      // a layer whose reduction is cut into ranges: its partial sums are added up after the tile launches
      if (listed && g.splits > 1 && !split_group_append(split_grp, g)) {
        for (int w = 0; w < 2; ++w)
          if ((e = tile_flush(w)) != hipSuccess) return e;
        if ((e = launch_split_reduce(split_grp, s)) != hipSuccess) return e;
        split_group_append(split_grp, g);  // its tiles have just run; the table is empty again
      }
    } else {
      bool short_ws = false;
      if ((e = launch_spmm(layers[i], s, &short_ws, SPMM_PRODUCT)) != hipSuccess) return e;
    }
  }
  if ((e = flush(sparse_grp, true)) != hipSuccess) return e;
  if ((e = flush(dense_grp, false)) != hipSuccess) return e;
  for (int which = 0; which < 2; ++which)
    if ((e = tile_flush(which)) != hipSuccess) return e;
  return launch_split_reduce(split_grp, s);
}

}  // namespace nm
