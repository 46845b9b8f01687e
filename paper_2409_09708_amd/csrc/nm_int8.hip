// int8 form of the N:M-sparse linear layer (Section 4, Table 6: 8-bit post-training quantisation applied
// on top of the sparse networks; Section 3.1: the mask may come from any saliency):
//
//   acc[t, o] = sum_k m[o, k] * Wq[o, k] * Xq[t, k]            exact, int32
//   Y[t, o]   = fma(float(acc), x_scale * w_scale[o], bias[o])
//
// The weight arrives as a dense int8 matrix plus the mask words of its level (in the quantisation flow the
// mask is the float weight's; a symmetric quantiser keeps pruned weights at zero, and whatever a pruned
// position holds is ignored).  Two matrix-core formulations, as for bfloat16:
//   * N <= 2: every run of 4 weights keeps at most 2, the pattern of v_smfmac_i32_16x16x128_i8.  A pre-pass
//     compresses the weight to [O, K/2] values + one 2-bit selector each ([O, K/32] words).  Lane
//     (row = lane % 16, kb = lane / 16) of the W operand holds 16 compressed values covering dense
//     k = 32 kb .. 32 kb + 31 and their 16 selectors in one register; the X operand lane (col, kb) holds
//     k = 16 kb + e (e < 16) and 64 + 16 kb + (e - 16) (e >= 16).  Half of the dense multiply-accumulates.
//   * N > 2: the masked dense weight through v_mfma_i32_16x16x64_i8 (lane (row, kb): k = 16 kb .. 16 kb + 15).
// A K step is 128 wide, so the LDS geometry in bytes is that of the bfloat16 kernels at K = 64: 128-byte X rows,
// 64-byte compressed (128-byte dense) W rows, 16-byte pieces XOR-swizzled, asynchronous global -> LDS copies
// three stages deep, one barrier per step.  Large layers run the persistent kernel of the bfloat16 path
// (nm_spmm.hip, templated on these instructions; the pre-pass here writes its stream order), smaller ones the
// tiled kernel below, shapes the tiles cannot take a one-lane-per-output kernel.
#include "nm_device.h"
#include "nm_launch.h"
#include "nm_mma.h"

#include <type_traits>
#include <utility>

namespace nm {

namespace {

// Where a layer's weight comes from: the dense int8 matrix with its mask words, or (Wq == NULL) the compressed form,
// int8 values [O, K N/M] + the index stream of the bfloat16 layer (Section 1; Section 2, Fig. 2 upper part).
struct I8Weight {
  const int8_t* Wq;
  int64_t ldw;
  const uint32_t* mask;
  const int8_t* values;
  const uint32_t* indices;
  int N, M;
};

// One window of 32 consecutive weights of row o (window blk): its mask word and its 32 bytes (byte i of the window in
// bits [8 (i mod 4), +8) of bytes[i / 4]).  From the dense weight the bytes are whatever the matrix holds (the caller
// applies the mask); from the compressed form pruned positions are 0.
__device__ __forceinline__ void load_window(const I8Weight& w, int64_t o, int64_t blk, int64_t K, uint32_t& mw,
                                            uint32_t (&bytes)[8]) {
  if (w.Wq != nullptr) {
    mw = w.mask[o * (K / 32) + blk];
    const uint4* src = reinterpret_cast<const uint4*>(w.Wq + o * w.ldw + blk * 32);
    const uint4 a = src[0], b = src[1];
    bytes[0] = a.x; bytes[1] = a.y; bytes[2] = a.z; bytes[3] = a.w;
    bytes[4] = b.x; bytes[5] = b.y; bytes[6] = b.z; bytes[7] = b.w;
    return;
  }
  const int B = log2_of(w.M);
  const int64_t nf = K / w.M * w.N;
  const int64_t nw = (nf * B + 31) / 32;
  const uint32_t* row = w.indices + o * nw;
  const int groups = 32 / w.M;
  mw = 0;
#pragma unroll
  for (int i = 0; i < 8; ++i) bytes[i] = 0;
  for (int g = 0; g < groups; ++g) {
    for (int j = 0; j < w.N; ++j) {
      const int64_t f = (blk * groups + g) * w.N + j;
      const uint32_t pos = (uint32_t)(g * w.M) + stream_bits(row, nw, f * B, B);
      const uint32_t v = (uint32_t)(uint8_t)w.values[o * nf + f] << (8 * (pos & 3u));
      mw |= 1u << pos;
#pragma unroll
      for (int i = 0; i < 8; ++i) bytes[i] |= (pos >> 2) == (uint32_t)i ? v : 0u;
    }
  }
}
__device__ __forceinline__ uint32_t window_byte(const uint32_t (&bytes)[8], int i) {
  return (bytes[i >> 2] >> (8 * (i & 3))) & 0xFFu;
}

// ---------------------------------------------------------------------------------------------
// Pre-pass: one lane per 32 consecutive weights of a row (one mask word).
// Sparse form: run q (4 weights) owns slots 2q and 2q+1; its first kept weight goes to slot 2q with
// selector = its offset in the run, a second one to slot 2q+1; free slots hold 0 (any selector is harmless
// there).  A run with more than two kept weights does not fit the form: the first two are taken (only an
// illegal mask produces one).
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
compress_i8_kernel(const I8Weight src, int64_t O, int64_t K, int8_t* __restrict__ vals, uint32_t* __restrict__ sel) {
  const int64_t per_row = K / 32;
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= O * per_row) return;
  const int64_t o = id / per_row, blk = id % per_row;
  uint32_t mw, w[8];
  load_window(src, o, blk, K, mw, w);
  uint32_t out[4] = {0, 0, 0, 0}, selw = 0;
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    const uint32_t bits = (mw >> (4 * q)) & 15u;
    int slot = 0;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      if (((bits >> p) & 1u) && slot < 2) {
        const int s = 2 * q + slot;
        out[s >> 2] |= window_byte(w, 4 * q + p) << (8 * (s & 3));
        selw |= (uint32_t)p << (2 * s);
        ++slot;
      }
    }
  }
  *reinterpret_cast<uint4*>(vals + o * (K / 2) + blk * 16) = make_uint4(out[0], out[1], out[2], out[3]);
  sel[o * per_row + blk] = selw;
}

__global__ void __launch_bounds__(256)
mask_copy_i8_kernel(const I8Weight src, int64_t O, int64_t K, int8_t* __restrict__ dense) {
  const int64_t per_row = K / 32;
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= O * per_row) return;
  const int64_t o = id / per_row, blk = id % per_row;
  uint32_t mw, w[8];
  load_window(src, o, blk, K, mw, w);
  uint32_t out[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    out[i] = 0;
#pragma unroll
    for (int b = 0; b < 4; ++b)
      if ((mw >> (4 * i + b)) & 1u) out[i] |= window_byte(w, 4 * i + b) << (8 * b);
  }
  uint4* dst = reinterpret_cast<uint4*>(dense + o * K + blk * 32);
  dst[0] = make_uint4(out[0], out[1], out[2], out[3]);
  dst[1] = make_uint4(out[4], out[5], out[6], out[7]);
}

// The same two forms in the persistent kernel's stream order (large layers): rows padded with zeros to whole
// 256-row tiles; a K step is 128 wide in the 2:4 form (64 compressed bytes per row: the lane's 16 bytes are
// piece blk % 4 of step blk / 4) and 64 wide in the dense form (the lane's 32 bytes are two pieces of step blk / 2).
__global__ void __launch_bounds__(256)
compress_i8_stream_kernel(const I8Weight src, int64_t O, int64_t O_pad, int64_t K, unsigned char* __restrict__ vals_s,
                          unsigned char* __restrict__ sel_s) {
  const int64_t per_row = K / 32;
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= O_pad * per_row) return;
  const int64_t o = id / per_row, blk = id % per_row;
  uint32_t out[4] = {0, 0, 0, 0}, selw = 0;
  if (o < O) {
    uint32_t mw, w[8];
    load_window(src, o, blk, K, mw, w);
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const uint32_t bits = (mw >> (4 * q)) & 15u;
      int slot = 0;
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        if (((bits >> p) & 1u) && slot < 2) {
          const int s = 2 * q + slot;
          out[s >> 2] |= window_byte(w, 4 * q + p) << (8 * (s & 3));
          selw |= (uint32_t)p << (2 * s);
          ++slot;
        }
      }
    }
  }
  const int64_t nk = K / 128, step = blk >> 2;
  *reinterpret_cast<uint4*>(vals_s + stream_piece_offset(o, step, (int)(blk & 3), nk)) = make_uint4(out[0], out[1], out[2], out[3]);
  *reinterpret_cast<uint32_t*>(sel_s + stream_selector8_offset(o, step, (int)(blk & 3), nk)) = selw;
}

__global__ void __launch_bounds__(256)
mask_copy_i8_stream_kernel(const I8Weight src, int64_t O, int64_t O_pad, int64_t K, unsigned char* __restrict__ dense_s) {
  const int64_t per_row = K / 32;
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= O_pad * per_row) return;
  const int64_t o = id / per_row, blk = id % per_row;
  uint32_t out[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  if (o < O) {
    uint32_t mw, w[8];
    load_window(src, o, blk, K, mw, w);
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int b = 0; b < 4; ++b)
        if ((mw >> (4 * i + b)) & 1u) out[i] |= window_byte(w, 4 * i + b) << (8 * b);
  }
  const int64_t nk = K / 64, step = blk >> 1;
  const int c0 = (int)(blk & 1) * 2;
  *reinterpret_cast<uint4*>(dense_s + stream_piece_offset(o, step, c0, nk)) = make_uint4(out[0], out[1], out[2], out[3]);
  *reinterpret_cast<uint4*>(dense_s + stream_piece_offset(o, step, c0 + 1, nk)) = make_uint4(out[4], out[5], out[6], out[7]);
}

// ---------------------------------------------------------------------------------------------
// Tiled matrix-core product
// ---------------------------------------------------------------------------------------------
struct I8Args {
  const int8_t* A;      // SPARSE: compressed values [O, K/2]; dense: masked weight [O, K]
  const uint32_t* sel;  // SPARSE: selector words [O, K/32]
  const int8_t* X;
  const float* w_scale;  // [O] or NULL (= 1)
  const float* bias;     // [O] or NULL
  float x_scale;
  void* Y;
  int64_t O, K, T, ldx, ldy;
  int n_o_tiles, n_t_tiles;
  int out_kind;   // NM_OUT_F32 / NM_OUT_BF16 / NM_OUT_I32 (raw accumulators)
  int vec_store;  // Y rows split into whole aligned 16-byte pieces
};

template <bool SPARSE, int WO, int WT, int OT, int TT, int STAGES_>
struct I8Cfg {
  static constexpr int STAGES = STAGES_;
  static constexpr int NW = WO * WT;
  static constexpr int NT = NW * 64;
  static constexpr int BO = WO * OT * 16;
  static constexpr int BT = WT * TT * 16;
  static constexpr int KC = 128;                        // dense k per stage
  static constexpr int H = SPARSE ? 1 : 2;              // sub-steps per stage (one K = 128 sparse or two K = 64 dense instructions per tile pair)
  static constexpr int A_ROWB = SPARSE ? 64 : 128;      // bytes of one W row per stage
  static constexpr int X_BYTES = BT * 128;
  static constexpr int A_BYTES = BO * A_ROWB;
  static constexpr int S_BYTES = SPARSE ? BO * 16 : 0;  // four selector words per row per stage
  static constexpr int STAGE = X_BYTES + A_BYTES + S_BYTES;
  static constexpr int LDS_BYTES = STAGES * STAGE;
  static constexpr int X_LOADS = X_BYTES / 1024;        // wave-wide 16-byte loads per stage
  static constexpr int A_LOADS = A_BYTES / 1024;
  static constexpr int S_LOADS = SPARSE ? (S_BYTES + 1023) / 1024 : 0;  // 64 rows of selectors per load
  static constexpr int X_PW = (X_LOADS + NW - 1) / NW;  // per wave (surplus waves repeat a load)
  static constexpr int A_PW = (A_LOADS + NW - 1) / NW;
  static constexpr int S_PW = SPARSE ? (S_LOADS + NW - 1) / NW : 0;
  static constexpr int LPW = X_PW + A_PW + S_PW;
  static_assert((STAGES == 2 || STAGES == 3) && STAGES * LPW < 64 && LDS_BYTES <= 160 * 1024, "stages");
  static_assert(!SPARSE || S_BYTES % 1024 == 0, "whole selector loads");
};

template <bool SPARSE, int WO, int WT, int OT, int TT, int STAGES>
__global__ void __launch_bounds__(WO * WT * 64)
nm_i8_gemm_kernel(const I8Args a) {
  using C = I8Cfg<SPARSE, WO, WT, OT, TT, STAGES>;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;

  // XCD-aware tile order: every XCD (own L2) takes a contiguous run of tiles, o fastest
  const int n_tiles = a.n_o_tiles * a.n_t_tiles;
  const int per_xcd = (n_tiles + 7) >> 3;
  const int tile = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
  if (tile >= n_tiles) return;
  const int64_t o0 = (int64_t)(tile % a.n_o_tiles) * C::BO;
  const int64_t t0 = (int64_t)(tile / a.n_o_tiles) * C::BT;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wo = wave % WO;
  const int wt = wave / WO;
  const int r16 = lane & 15;
  const int kb = lane >> 4;

  // ---- per-lane source offsets and per-wave LDS destinations of this wave's loads (fixed over K); rows past
  // the edge re-read the last valid row (their outputs are never stored)
  const int64_t a_ld = SPARSE ? (a.K >> 1) : a.K;  // bytes per row of A
  uint32_t x_voff[C::X_PW], a_voff[C::A_PW], s_voff[C::S_PW > 0 ? C::S_PW : 1];
  uint32_t x_dst[C::X_PW], a_dst[C::A_PW], s_dst[C::S_PW > 0 ? C::S_PW : 1];
  const int64_t t_last = a.T - 1 - t0, o_last = a.O - 1 - o0;
#pragma unroll
  for (int i = 0; i < C::X_PW; ++i) {
    const int j = (wave + i * C::NW) % C::X_LOADS;
    int64_t row = 8 * j + (lane >> 3);
    const int c = (lane & 7) ^ (int)(row & 7);
    if (row > t_last) row = t_last;
    x_voff[i] = (uint32_t)(row * a.ldx + c * 16);
    x_dst[i] = (uint32_t)(j * 1024);
  }
#pragma unroll
  for (int i = 0; i < C::A_PW; ++i) {
    const int j = (wave + i * C::NW) % C::A_LOADS;
    int64_t row;
    int c;
    if (SPARSE) { row = 16 * j + (lane >> 2); c = (lane & 3) ^ (int)((row >> 1) & 3); }
    else { row = 8 * j + (lane >> 3); c = (lane & 7) ^ (int)(row & 7); }
    if (row > o_last) row = o_last;
    a_voff[i] = (uint32_t)(row * a_ld + c * 16);
    a_dst[i] = (uint32_t)(C::X_BYTES + j * 1024);
  }
  if (SPARSE) {
#pragma unroll
    for (int i = 0; i < C::S_PW; ++i) {
      const int j = (wave + i * C::NW) % C::S_LOADS;
      int64_t row = 64 * j + lane;
      if (row > o_last) row = o_last;
      s_voff[i] = (uint32_t)(row * (a.K >> 3));  // K/32 words of 4 bytes per row
      s_dst[i] = (uint32_t)(C::X_BYTES + C::A_BYTES + j * 1024);
    }
  }
  const int8_t* x_base = a.X + t0 * a.ldx;
  const int8_t* a_base = a.A + o0 * a_ld;
  const unsigned char* s_base = SPARSE ? reinterpret_cast<const unsigned char*>(a.sel) + o0 * (a.K >> 3) : nullptr;

  auto issue_one = [&](auto d_tag, int ks, int buf) {
    constexpr int d = decltype(d_tag)::value;
    const uint32_t lds = __builtin_amdgcn_readfirstlane(lds0 + (uint32_t)buf * C::STAGE);
    if constexpr (d < C::X_PW) {
      dma16(make_uniform(x_base + (int64_t)ks * 128), x_voff[d], lds + x_dst[d]);
    } else if constexpr (d < C::X_PW + C::A_PW) {
      dma16(make_uniform(a_base + (int64_t)ks * (SPARSE ? 64 : 128)), a_voff[d - C::X_PW], lds + a_dst[d - C::X_PW]);
    } else {
      dma16(make_uniform(s_base + (int64_t)ks * 16), s_voff[d - C::X_PW - C::A_PW], lds + s_dst[d - C::X_PW - C::A_PW]);
    }
  };
  auto issue_stage = [&](int ks, int buf) {
    [&]<int... D>(std::integer_sequence<int, D...>) {
      (issue_one(std::integral_constant<int, D>{}, ks, buf), ...);
    }(std::make_integer_sequence<int, C::LPW>{});
  };

  i32x4_t acc[OT][TT];
#pragma unroll
  for (int i = 0; i < OT; ++i)
#pragma unroll
    for (int j = 0; j < TT; ++j) acc[i][j] = i32x4_t{0, 0, 0, 0};

  // fragment read offsets inside a stage (the XOR undoes the swizzle applied by the loads)
  const int x_sw = r16 & 7;
  const int x_row = (wt * TT * 16 + r16) * 128;
  const int a_row = C::X_BYTES + (wo * OT * 16 + r16) * C::A_ROWB;
  const int a_sw = SPARSE ? ((r16 >> 1) & 3) : (r16 & 7);
  const int s_row = C::X_BYTES + C::A_BYTES + (wo * OT * 16 + r16) * 16 + kb * 4;

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
        af[i] = *reinterpret_cast<const u32x4_t*>(base + a_row + i * 16 * C::A_ROWB + ((kb ^ a_sw) * 16));
        sel[i] = *reinterpret_cast<const int*>(base + s_row + i * 16 * 16);
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
      for (int i = 0; i < OT; ++i)
        af[i] = *reinterpret_cast<const u32x4_t*>(base + a_row + i * 16 * C::A_ROWB + (((h * 4 + kb) ^ a_sw) * 16));
#pragma unroll
      for (int j = 0; j < TT; ++j)
        bd[j] = *reinterpret_cast<const u32x4_t*>(base + x_row + j * 16 * 128 + (((h * 4 + kb) ^ x_sw) * 16));
    }
  };
  constexpr int MMA = OT * TT;
  constexpr int EVERY = MMA / C::LPW > 0 ? MMA / C::LPW : 1;
  auto multiply = [&](bool load, int lks, int lbuf) {
    [&]<int... Q>(std::integer_sequence<int, Q...>) {
      ([&] {
        constexpr int j = Q / OT, i = Q % OT;
        if (SPARSE)
          acc[i][j] = __builtin_amdgcn_smfmac_i32_16x16x128_i8(__builtin_bit_cast(i32x4_t, af[i]),
                                                               __builtin_bit_cast(i32x8_t, bs[j]), acc[i][j], sel[i], 0, 0);
        else
          acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(__builtin_bit_cast(i32x4_t, af[i]),
                                                            __builtin_bit_cast(i32x4_t, bd[j]), acc[i][j], 0, 0, 0);
        if constexpr (Q % EVERY == EVERY - 1 && Q / EVERY < C::LPW) {
          if (load) issue_one(std::integral_constant<int, Q / EVERY>{}, lks, lbuf);
          __builtin_amdgcn_sched_barrier(0);
        }
      }(), ...);
    }(std::make_integer_sequence<int, MMA>{});
  };

  const int nk = (int)(a.K / C::KC);
#pragma unroll
  for (int s = 0; s < STAGES - 1; ++s)
    if (s < nk) issue_stage(s, s);

  // One barrier per stage; the buffer multiplied in the previous step is refilled right after the barrier,
  // two stages ahead.
  {
    int buf = 0;
    for (int ks = 0; ks < nk; ++ks) {
      if (STAGES == 3 && ks + 1 < nk) wait_loads_outstanding<C::LPW>();  // one younger stage may still be in flight
      else wait_loads_outstanding<0>();
      __builtin_amdgcn_s_barrier();
      int nbuf = buf + STAGES - 1;
      if (nbuf >= STAGES) nbuf -= STAGES;
#pragma unroll
      for (int h = 0; h < H; ++h) {
        read_frags(buf, h);
        multiply(h == 0 && ks + STAGES - 1 < nk, ks + STAGES - 1, nbuf);
      }
      if (++buf == STAGES) buf = 0;
    }
  }

  // ---- write-out.  A lane holds out-features o .. o+3 (accumulator element e -> row 4 kb + e of the 16-row
  // block) of token r16.  The accumulators are rescaled (or kept as integers), then, for aligned outputs,
  // every wave transposes 16 tokens at a time through its own LDS slice so that the global stores are 16 bytes
  // per lane and whole row segments of the wave tile are written contiguously.
  // from here on the accumulators hold the 32-bit output patterns: float, or the integers themselves
#pragma unroll
  for (int i = 0; i < OT; ++i) {
    if (a.out_kind == 2) break;
    const int64_t o = o0 + (wo * OT + i) * 16 + kb * 4;
    float sc[4], bi[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const bool in = o + e < a.O;
      sc[e] = a.x_scale * ((a.w_scale && in) ? a.w_scale[o + e] : 1.f);
      bi[e] = (a.bias && in) ? a.bias[o + e] : 0.f;
    }
#pragma unroll
    for (int j = 0; j < TT; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[i][j][e] = (int)__float_as_uint(fmaf((float)acc[i][j][e], sc[e], bi[e]));
  }
  __builtin_amdgcn_s_barrier();  // every wave is done with the operand stages
  auto get = [&](int i, int j) { return __builtin_bit_cast(u32x4_t, acc[i][j]); };
  const int64_t row0 = t0 + wt * TT * 16, col0 = o0 + wo * OT * 16;
  static_assert(C::NW * wave_tile_slice_bytes<OT, 4>() <= C::LDS_BYTES, "write-out slices");
  if (a.vec_store) {
    if (a.out_kind == 1)
      write_wave_tile_pieces<OT, TT, 2>(smem + wave * wave_tile_slice_bytes<OT, 2>(), lane, get, a.Y, a.ldy, row0, col0, a.T, a.O);
    else
      write_wave_tile_pieces<OT, TT, 4>(smem + wave * wave_tile_slice_bytes<OT, 4>(), lane, get, a.Y, a.ldy, row0, col0, a.T, a.O);
  } else {
    write_wave_tile_elements<OT, TT>(lane, get, a.Y, a.ldy, row0, col0, a.T, a.O, a.out_kind == 1);
  }
}

// Any shape and alignment: one lane per output, reading the dense weight and the mask words (or the compressed
// form: decode the position, select the activation, multiply, add) directly.
__global__ void __launch_bounds__(256)
i8_general_kernel(const I8Weight w, int64_t O, int64_t K, const int8_t* __restrict__ X, int64_t T, int64_t ldx,
                  float x_scale, const float* __restrict__ w_scale, const float* __restrict__ bias, void* __restrict__ Y,
                  int64_t ldy, int out_kind) {
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= T * O) return;
  const int64_t t = id / O, o = id % O;
  int acc = 0;
  if (w.Wq != nullptr) {
    const int64_t mw = (K + 31) / 32;
    for (int64_t k = 0; k < K; ++k)
      if ((w.mask[o * mw + (k >> 5)] >> (k & 31)) & 1u) acc += (int)w.Wq[o * w.ldw + k] * (int)X[t * ldx + k];
  } else {
    const int B = log2_of(w.M);
    const int64_t nf = K / w.M * w.N;
    const int64_t nw = (nf * B + 31) / 32;
    const uint32_t* row = w.indices + o * nw;
    for (int64_t f = 0; f < nf; ++f) {
      const int64_t k = (f / w.N) * w.M + stream_bits(row, nw, f * B, B);
      acc += (int)w.values[o * nf + f] * (int)X[t * ldx + k];
    }
  }
  if (out_kind == 2) {
    reinterpret_cast<int*>(Y)[t * ldy + o] = acc;
    return;
  }
  const float y = fmaf((float)acc, x_scale * (w_scale ? w_scale[o] : 1.f), bias ? bias[o] : 0.f);
  if (out_kind == 1) reinterpret_cast<bf16_t*>(Y)[t * ldy + o] = (bf16_t)f32_to_bf16_rne(y);
  else reinterpret_cast<float*>(Y)[t * ldy + o] = y;
}

// ---------------------------------------------------------------------------------------------
// Compressed form of the int8 weight: the kept values of every group in ascending position and the index stream
// of the bfloat16 layer.  A caller's mask is made usable as in the bfloat16 packing (the N lowest set positions;
// missing ones completed with the lowest unset positions, stored as 0).
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t group_mask_bits(const uint32_t* __restrict__ mask, int64_t K, int64_t o, int64_t g, int M) {
  const int64_t k0 = g * M;
  return (mask[o * ((K + 31) / 32) + (k0 >> 5)] >> (k0 & 31)) & ((1u << M) - 1u);
}

__global__ void __launch_bounds__(256)
pack_i8_values_kernel(const int8_t* __restrict__ Wq, int64_t ldw, const uint32_t* __restrict__ mask, int64_t O, int64_t K,
                      int N, int M, int8_t* __restrict__ values) {
  const int64_t G = K / M;
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= O * G) return;
  const int64_t o = id / G, g = id % G;
  uint32_t filled;
  const uint32_t km = legalize_mask(group_mask_bits(mask, K, o, g, M), N, M, &filled);
  int j = 0;
  for (int i = 0; i < M; ++i)
    if ((km >> i) & 1u) {
      values[o * (G * N) + g * N + j] = ((filled >> i) & 1u) ? (int8_t)0 : Wq[o * ldw + g * M + i];
      ++j;
    }
}

// one lane per index word: the fields that overlap it, from the mask words of their groups
__global__ void __launch_bounds__(256)
pack_i8_index_kernel(const uint32_t* __restrict__ mask, int64_t O, int64_t K, int N, int M, uint32_t* __restrict__ indices) {
  const int b = log2_of(M);
  const int64_t nf = K / M * N;
  const int64_t nw = (nf * b + 31) / 32;
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= O * nw) return;
  const int64_t o = id / nw, w = id % nw;
  const int64_t bit0 = w * 32;
  const int64_t f_lo = bit0 / b;
  int64_t f_hi = (bit0 + 31) / b;
  if (f_hi > nf - 1) f_hi = nf - 1;
  uint32_t word = 0, km = 0, filled;
  int64_t g_cached = -1;
  for (int64_t f = f_lo; f <= f_hi; ++f) {
    const int64_t g = f / N;
    if (g != g_cached) { km = legalize_mask(group_mask_bits(mask, K, o, g, M), N, M, &filled); g_cached = g; }
    int want = (int)(f % N);
    uint64_t p = 0;
    for (int i = 0; i < M; ++i)
      if ((km >> i) & 1u) { if (want == 0) { p = (uint64_t)i; break; } --want; }
    const int64_t off = f * b - bit0;  // negative for a field that began in the previous word
    word |= off >= 0 ? (uint32_t)(p << off) : (uint32_t)(p >> (-off));
  }
  indices[o * nw + w] = word;
}

__global__ void __launch_bounds__(256)
unpack_i8_kernel(const int8_t* __restrict__ values, const uint32_t* __restrict__ indices, int64_t O, int64_t K, int N, int M,
                 int8_t* __restrict__ Wd, int64_t ldw) {
  const int b = log2_of(M);
  const int64_t G = K / M;
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= O * G) return;
  const int64_t o = id / G, g = id % G;
  const int64_t nf = G * N;
  const int64_t nw = (nf * b + 31) / 32;
  int8_t* dst = Wd + o * ldw + g * M;
  for (int i = 0; i < M; ++i) dst[i] = 0;
  for (int j = 0; j < N; ++j) {
    const int64_t f = g * N + j;
    dst[stream_bits(indices + o * nw, nw, f * b, b)] = values[o * nf + f];
  }
}

inline bool aligned_to(const void* p, uintptr_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

template <bool SPARSE, int WO, int WT, int OT, int TT, int STAGES>
hipError_t launch_i8_gemm(I8Args g, hipStream_t s) {
  using C = I8Cfg<SPARSE, WO, WT, OT, TT, STAGES>;
  auto kern = nm_i8_gemm_kernel<SPARSE, WO, WT, OT, TT, STAGES>;
  static PerDeviceOnce lds_limit;
  if (hipError_t e = raise_dynamic_lds_limit(kern, C::LDS_BYTES, lds_limit); e != hipSuccess) return e;
  g.n_o_tiles = (int)((g.O + C::BO - 1) / C::BO);
  g.n_t_tiles = (int)((g.T + C::BT - 1) / C::BT);
  const int64_t n_tiles = (int64_t)g.n_o_tiles * g.n_t_tiles;
  const int64_t grid = ((n_tiles + 7) / 8) * 8;
  if (grid > 0x7FFFFFFF) return hipErrorInvalidValue;
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(C::NT), C::LDS_BYTES, s, g);
  return hipGetLastError();
}

template <bool SPARSE>
hipError_t dispatch_i8(const I8Args& g, hipStream_t s) {
  const int64_t tiles_big = ((g.O + 255) / 256) * ((g.T + 255) / 256);
  const int64_t tiles_mid = ((g.O + 127) / 128) * ((g.T + 127) / 128);
  const int pick = tiles_big >= 256 ? 3 : (tiles_mid >= 256 ? 2 : 1);
  if (pick == 3) return launch_i8_gemm<SPARSE, 4, 2, 4, 8, SPARSE ? 3 : 2>(g, s);
  if (pick == 2) return launch_i8_gemm<SPARSE, 2, 2, 4, 4, 3>(g, s);
  return launch_i8_gemm<SPARSE, 2, 2, 2, 2, 3>(g, s);
}

}  // namespace

size_t i8_workspace_bytes(int64_t O, int64_t K, int N, int M, int64_t T) {
  if (K % 128) return 0;  // the general kernel reads the weight and the mask itself
  const bool sparse_form = N <= 2 && N < M;
  const int64_t rows = stream_i8_takes(O, K, T, N, M) ? ((O + 255) / 256) * 256 : O;  // stream order: whole tiles
  return sparse_form ? (size_t)(rows * K / 2) + (size_t)(rows * K / 8) : (size_t)(rows * K);
}

hipError_t launch_pack_i8(const int8_t* Wq, int64_t O, int64_t K, int64_t ldw, int N, int M, const uint32_t* mask,
                          int8_t* values, uint32_t* indices, hipStream_t s) {
  const int64_t ng = O * (K / M);
  hipLaunchKernelGGL(pack_i8_values_kernel, dim3((unsigned)((ng + 255) / 256)), dim3(256), 0, s, Wq, ldw, mask, O, K, N, M,
                     values);
  const int64_t nw = O * index_words_per_row(K, N, M);
  hipLaunchKernelGGL(pack_i8_index_kernel, dim3((unsigned)((nw + 255) / 256)), dim3(256), 0, s, mask, O, K, N, M, indices);
  return hipGetLastError();
}

hipError_t launch_unpack_i8(const int8_t* values, const uint32_t* indices, int64_t O, int64_t K, int N, int M, int8_t* Wd,
                            int64_t ldw, hipStream_t s) {
  const int64_t ng = O * (K / M);
  hipLaunchKernelGGL(unpack_i8_kernel, dim3((unsigned)((ng + 255) / 256)), dim3(256), 0, s, values, indices, O, K, N, M, Wd,
                     ldw);
  return hipGetLastError();
}

hipError_t launch_linear_i8(const I8LinearArgs& a, hipStream_t s, bool* workspace_short, int phases) {
  *workspace_short = false;
  const bool prepare = phases & SPMM_PREPARE, product = phases & SPMM_PRODUCT;
  const bool packed = a.Wq == nullptr;
  const I8Weight src{a.Wq, a.ldw, a.mask, a.values, a.indices, a.N, a.M};
  const bool tiles = (a.K % 128 == 0) && a.O <= (1 << 24) && a.K <= (1 << 24) && a.T <= (1ll << 31);
  const bool operands_ok = !product || (aligned_to(a.X, 16) && (a.ldx % 16 == 0) && a.ldx <= (1 << 24));
  // the same answer in both phases; the compressed form is read element by element (no alignment needed)
  const bool weight_ok = packed || (aligned_to(a.Wq, 16) && (a.ldw % 16 == 0));
  auto general = [&]() {
    if (a.T * a.O > 0x7FFFFFFFll * 256) return hipErrorInvalidValue;
    hipLaunchKernelGGL(i8_general_kernel, dim3((unsigned)((a.T * a.O + 255) / 256)), dim3(256), 0, s, src, a.O, a.K, a.X, a.T,
                       a.ldx, a.x_scale, a.w_scale, a.bias, a.Y, a.ldy, a.out_kind);
    return hipGetLastError();
  };
  if (!tiles || !operands_ok || !weight_ok) {
    if (!product) return hipSuccess;
    return general();
  }
  const size_t need = i8_workspace_bytes(a.O, a.K, a.N, a.M, a.T);
  if (a.workspace == nullptr || a.workspace_bytes < need || !aligned_to(a.workspace, 256)) {
    *workspace_short = true;
    return hipSuccess;
  }
  const bool sparse_form = a.N <= 2 && a.N < a.M;
  unsigned char* ws = reinterpret_cast<unsigned char*>(a.workspace);
  if (stream_i8_takes(a.O, a.K, a.T, a.N, a.M)) {
    // large layers: the persistent kernel, operands in its stream order.  It writes Y in 16-byte pieces and
    // fetches scales and bias in 16-byte pieces; a call whose output or constants are not aligned for that runs
    // the general kernel (it reads the weight itself).
    const int64_t o_pad = ((a.O + 255) / 256) * 256;
    unsigned char* sel_s = ws + (size_t)(o_pad * a.K / 2);
    if (prepare) {
      const int64_t n = o_pad * (a.K / 32);
      const dim3 grid((unsigned)((n + 255) / 256));
      if (sparse_form)
        hipLaunchKernelGGL(compress_i8_stream_kernel, grid, dim3(256), 0, s, src, a.O, o_pad, a.K, ws, sel_s);
      else
        hipLaunchKernelGGL(mask_copy_i8_stream_kernel, grid, dim3(256), 0, s, src, a.O, o_pad, a.K, ws);
      hipError_t e = hipGetLastError();
      if (e != hipSuccess) return e;
    }
    if (!product) return hipSuccess;
    const int per_piece = a.out_kind == 1 ? 8 : 4;
    const bool vec = (a.ldy % per_piece == 0) && aligned_to(a.Y, 16) && (a.O % per_piece == 0) && a.ldy <= 0x7FFFFFFF &&
                     aligned_to(a.w_scale, 16) && aligned_to(a.bias, 16) && (a.O % 4 == 0);
    if (!vec) return general();
    StreamI8Args g;
    g.values = reinterpret_cast<const int8_t*>(ws); g.sel = sparse_form ? reinterpret_cast<const uint32_t*>(sel_s) : nullptr;
    g.sparse_form = sparse_form; g.X = a.X; g.w_scale = a.w_scale; g.bias = a.bias; g.x_scale = a.x_scale;
    g.Y = a.Y; g.O = a.O; g.K = a.K; g.T = a.T; g.ldx = a.ldx; g.ldy = a.ldy; g.out_kind = a.out_kind;
    return launch_stream_i8(g, s);
  }
  int8_t* vals = reinterpret_cast<int8_t*>(ws);
  uint32_t* sel = reinterpret_cast<uint32_t*>(ws + (size_t)(a.O * a.K / 2));
  if (prepare) {
    const int64_t n = a.O * (a.K / 32);
    const dim3 grid((unsigned)((n + 255) / 256));
    if (sparse_form) hipLaunchKernelGGL(compress_i8_kernel, grid, dim3(256), 0, s, src, a.O, a.K, vals, sel);
    else hipLaunchKernelGGL(mask_copy_i8_kernel, grid, dim3(256), 0, s, src, a.O, a.K, vals);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  if (!product) return hipSuccess;
  I8Args g;
  g.A = vals; g.sel = sparse_form ? sel : nullptr; g.X = a.X;
  g.w_scale = a.w_scale; g.bias = a.bias; g.x_scale = a.x_scale;
  g.Y = a.Y; g.O = a.O; g.K = a.K; g.T = a.T; g.ldx = a.ldx; g.ldy = a.ldy;
  g.n_o_tiles = g.n_t_tiles = 0;
  g.out_kind = a.out_kind;
  const int per_piece = a.out_kind == 1 ? 8 : 4;
  g.vec_store = (a.ldy % per_piece == 0) && aligned_to(a.Y, 16) && (a.O % per_piece == 0);
  return sparse_form ? dispatch_i8<true>(g, s) : dispatch_i8<false>(g, s);
}

}  // namespace nm
