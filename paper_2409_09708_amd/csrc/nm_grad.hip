// Training products of one sparse linear layer (Section 3.2: the gradient of the loss is taken with
// respect to the sparse weights of the chosen configuration; Section 3.1, weight-update figure: the
// sparse matrix of the applied level is what is trained inside the shared weight).  With the mask of
// the step held fixed and Y = X (W (.) m)^T:
//
//   dX[t, k] = sum_o dY[t, o] * (W (.) m)[o, k]            reduction over the out-features
//   dW[o, k] = sum_t dY[t, o] * X[t, k]   ((.) m[o, k])     reduction over the tokens
//
// Both are dense products (the weight is N:M along k, which is an OUTPUT index of dX, so no term of
// the reduction can be skipped), and in both the reduction index is the ROW index of an operand as
// it lies in memory: W (.) m is [O, K], dY is [T, O], X is [T, K].  The matrix instruction wants, per
// lane, 8 consecutive reduction indices of one row.  Instead of transposing operands in HBM, a tile
// travels global -> LDS as it lies (rows = reduction index) and the fragments are read with the
// transposing LDS read of gfx950 (ds_read_b64_tr_b16): in each group of 16 lanes, lanes 4e .. 4e+3
// name the 16 elements of "row" e (4 each), and lane i receives element i of rows 0 .. 3, i.e. four
// consecutive reduction indices of column i.
//
// One kernel serves both products:  C[i, j] = sum_r P[r, i] * Q(j, r), stored as Out[j, i]:
//   dX: P = W (.) m [r = o, i = k], Q = dY as [j = t, r = o] (reduction contiguous), Out = dX [t, k]
//   dW: P = X       [r = t, i = k], Q = dY as [r = t, j = o] (reduction = row),       Out = dW [o, k]
// The token reduction of dW is long and its output small (a few dozen 128 x 256 tiles), so it is cut
// into `splits` ranges; every block leaves an fp32 partial tile and a second kernel adds the partial
// tiles in split order (the result does not depend on scheduling), applies the mask and rounds.
#include "nm_device.h"
#include "nm_launch.h"
#include "nm_mma.h"

#include <type_traits>
#include <utility>

namespace nm {

namespace {

typedef short i16x4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) i16x4_t* lds_i16x4_ptr;

struct TGemmArgs {
  const bf16_t* P;  // [R, I], ld ldp
  const bf16_t* Q;  // Q_STRIDED: [R, J], else [J, R]; ld ldq
  int64_t I, J, R, ldp, ldq;
  void* out;        // Out[J, I], ld ldo (when partial is NULL)
  int64_t ldo;
  int out_bf16;
  int vec_store;    // Out rows split into whole aligned 16-byte pieces
  int n_i_tiles, n_j_tiles;
  int splits;       // ranges the reduction is cut into (>= 1)
  float* partial;   // not NULL: fp32 partial tiles [split][tile][accumulator][thread] (16 bytes per thread)
                    // instead of Out
};

struct TCfg {
  // 4 waves (2 x 2), each 64 (i) x 128 (j) outputs: a wave reads 12 fragments per 32 matrix instructions (the
  // LDS read rate is what bounds these kernels; 64 x 64 per wave needs 8 per 16).  Two blocks share a compute
  // unit (72 KiB of LDS each), so one block's barrier and write-out overlap the other's arithmetic.
  static constexpr int WI = 2, WJ = 2, IT = 4, JT = 8;
  static constexpr int NW = WI * WJ, NT = NW * 64;
  static constexpr int BI = WI * IT * 16, BJ = WJ * JT * 16;  // 128 x 256 outputs per block
  static constexpr int RS = 32;                                // reduction indices per stage: one instruction deep
  static constexpr int STAGES = 3;
  static constexpr int P_ROWB = BI * 2, Q_ROWB = BJ * 2;       // bytes of a row of a reduction-major tile
  static constexpr int P_BYTES = RS * BI * 2, Q_BYTES = RS * BJ * 2;
  static constexpr int STAGE = P_BYTES + Q_BYTES;
  static constexpr int LDS_BYTES = STAGES * STAGE;
  static constexpr int P_PW = P_BYTES / 1024 / NW, Q_PW = Q_BYTES / 1024 / NW;  // wave-wide loads per wave
  static constexpr int LPW = P_PW + Q_PW;
  static constexpr int MMA = IT * JT;
  static_assert(P_PW * NW * 1024 == P_BYTES && Q_PW * NW * 1024 == Q_BYTES && STAGES * LPW < 64, "load split");
  static_assert(2 * LDS_BYTES <= 160 * 1024, "two blocks per compute unit");
};

// Transposing fragment read from a tile stored as [RS rows (reduction)][ROWB / 2 columns], the 16-byte pieces
// of row r at slot (piece ^ 2 (r & 3) ^ 8 ((r >> 3) & 1)): the 16 lanes of a group touch four rows, and the
// first term puts their 32-byte runs on different banks; two groups are served together and their rows lie 8
// apart, the second term sends them to different halves of the 64 banks.  Lane (c16 = lane % 16, kb = lane / 16) receives the reduction indices
// 8 kb .. 8 kb + 7 of column 16 * block + c16.
template <int ROWB>
__device__ __forceinline__ u32x4_t read_transposed(const unsigned char* tile, int block, int c16, int kb) {
  const int sub = c16 >> 2;  // row inside the group of four; also (row & 3)
  const int off = (8 * kb + sub) * ROWB + (((2 * (block ^ sub) + ((c16 & 3) >> 1)) ^ (8 * (kb & 1))) << 4) + (c16 & 1) * 8;
  const i16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4_ptr)(tile + off));
  const i16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4_ptr)(tile + off + 4 * ROWB));
  typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
  const u32x2_t l = __builtin_bit_cast(u32x2_t, lo), h = __builtin_bit_cast(u32x2_t, hi);
  return u32x4_t{l[0], l[1], h[0], h[1]};
}

// Where lane `lane` of the n-th wave-wide load (1 KiB of consecutive LDS) of a reduction-major tile reads:
// row of the stage and 16-byte piece of that row (before the edge clamp).
template <int ROWB>
__device__ __forceinline__ void strided_load_place(int n, int lane, int* row, int* piece) {
  constexpr int PER_ROW = ROWB / 16, ROWS = 1024 / ROWB;
  *row = n * ROWS + lane / PER_ROW;
  *piece = (lane % PER_ROW) ^ (2 * (*row & 3)) ^ (8 * ((*row >> 3) & 1));
}

template <bool Q_STRIDED>
__global__ void __launch_bounds__(TCfg::NT, 2)
nm_tgemm_kernel(const TGemmArgs a) {
  using C = TCfg;
  constexpr int IT = C::IT, JT = C::JT, STAGES = C::STAGES;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem;

  // Block -> (tile, split).  Consecutive block ids land on different XCDs (8, each with its own L2); every
  // XCD takes a contiguous run of (split, tile) pairs, tiles fastest and i fastest among the tiles, so the
  // blocks that share an L2 share rows of Q, and each range of rows of a split reduction is fetched into one
  // L2 (two where a split straddles a boundary).
  const int n_tiles = a.n_i_tiles * a.n_j_tiles;
  const int64_t n_blocks = (int64_t)n_tiles * a.splits;
  const int64_t per_xcd = (n_blocks + 7) >> 3;
  const int64_t virt = (int64_t)(blockIdx.x & 7) * per_xcd + (int64_t)(blockIdx.x >> 3);
  if (virt >= n_blocks) return;
  const int split = (int)(virt / n_tiles);
  const int tile = (int)(virt % n_tiles);
  const int64_t i0 = (int64_t)(tile % a.n_i_tiles) * C::BI;
  const int64_t j0 = (int64_t)(tile / a.n_i_tiles) * C::BJ;

  // this block's reduction steps
  const int64_t steps_all = (a.R + C::RS - 1) / C::RS;
  int64_t step_first = 0, nk = steps_all;
  if (a.splits > 1) {
    const int64_t share = steps_all / a.splits, extra = steps_all % a.splits;
    step_first = split * share + (split < extra ? split : extra);
    nk = share + (split < extra ? 1 : 0);
  }
  const int64_t r_first = step_first * C::RS;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wi = wave % C::WI;
  const int wj = wave / C::WI;
  const int c16 = lane & 15;
  const int kb = lane >> 4;

  // ---- this wave's loads of a stage.  Columns of a reduction-major tile past the edge re-read the last whole
  // piece of the row (those outputs are never stored).  Rows past R are clamped to stay inside the operand
  // and zeroed in LDS before use.
  int p_row[C::P_PW], q_row[C::Q_PW];       // row inside the stage (reduction-major) or inside the tile
  uint32_t p_col[C::P_PW], q_col[C::Q_PW];  // byte offset inside the row
  uint32_t p_dst[C::P_PW], q_dst[C::Q_PW];
  const int64_t p_last_piece = (a.I - i0) / 8 - 1;
#pragma unroll
  for (int d = 0; d < C::P_PW; ++d) {
    const int n = wave + d * C::NW;
    int piece;
    strided_load_place<C::P_ROWB>(n, lane, &p_row[d], &piece);
    if (piece > p_last_piece) piece = (int)p_last_piece;
    p_col[d] = (uint32_t)(piece * 16);
    p_dst[d] = (uint32_t)(n * 1024);
  }
  const int64_t q_last_piece = (a.J - j0) / 8 - 1, q_last_row = a.J - 1 - j0;
#pragma unroll
  for (int d = 0; d < C::Q_PW; ++d) {
    const int n = wave + d * C::NW;
    if (Q_STRIDED) {
      int piece;
      strided_load_place<C::Q_ROWB>(n, lane, &q_row[d], &piece);
      if (piece > q_last_piece) piece = (int)q_last_piece;
      q_col[d] = (uint32_t)(piece * 16);
    } else {
      // [BJ rows j][32 reduction indices]: 64 bytes per row, load n covers rows 16n .. 16n+15, lane ->
      // (row 16n + lane / 4, slot lane % 4), the slot holds piece slot ^ ((row >> 1) & 3)
      int64_t row = 16 * n + (lane >> 2);
      const int piece = (lane & 3) ^ (int)((row >> 1) & 3);
      if (row > q_last_row) row = q_last_row;
      q_row[d] = (int)row;
      q_col[d] = (uint32_t)(piece * 16);
    }
    q_dst[d] = (uint32_t)(C::P_BYTES + n * 1024);
  }
  const bf16_t* p_base = a.P + i0;
  // lane byte offsets of the loads of a stage with all its rows (the common case; a ragged last stage clamps)
  uint32_t p_voff[C::P_PW], q_voff[C::Q_PW];
#pragma unroll
  for (int d = 0; d < C::P_PW; ++d) p_voff[d] = (uint32_t)p_row[d] * (uint32_t)(a.ldp * 2) + p_col[d];
#pragma unroll
  for (int d = 0; d < C::Q_PW; ++d) q_voff[d] = (uint32_t)q_row[d] * (uint32_t)(a.ldq * 2) + q_col[d];
  const bf16_t* q_base = Q_STRIDED ? a.Q + j0 : a.Q + j0 * a.ldq;
  const uint32_t ldp2 = (uint32_t)(a.ldp * 2), ldq2 = (uint32_t)(a.ldq * 2);

  // A stage's sources: the (wave-uniform) operand addresses at its first reduction index and the rows it has
  struct StageSrc { uniform_ptr_t p, q; int rows; };
  auto stage_src = [&](int64_t r) {
    StageSrc src;
    src.p = make_uniform(p_base + r * a.ldp);
    src.q = make_uniform(Q_STRIDED ? q_base + r * a.ldq : q_base + r);
    src.rows = (int)((a.R - r) < C::RS ? (a.R - r) : C::RS);  // >= 1
    return src;
  };
  // the d-th load of a stage into LDS buffer buf
  auto issue_one = [&](auto d_tag, const StageSrc& src, int buf) {
    constexpr int d = decltype(d_tag)::value;
    const uint32_t lds = __builtin_amdgcn_readfirstlane(lds0 + (uint32_t)buf * C::STAGE);
    const bool ragged = src.rows < C::RS;  // wave-uniform; only the last stage of the reduction
    if constexpr (d < C::P_PW) {
      uint32_t voff = p_voff[d];
      if (ragged && p_row[d] >= src.rows) voff = (uint32_t)(src.rows - 1) * ldp2 + p_col[d];
      dma16(src.p, voff, lds + p_dst[d]);
    } else if constexpr (Q_STRIDED) {
      uint32_t voff = q_voff[d - C::P_PW];
      if (ragged && q_row[d - C::P_PW] >= src.rows) voff = (uint32_t)(src.rows - 1) * ldq2 + q_col[d - C::P_PW];
      dma16(src.q, voff, lds + q_dst[d - C::P_PW]);
    } else {
      dma16(src.q, q_voff[d - C::P_PW], lds + q_dst[d - C::P_PW]);
    }
  };
  auto issue_stage = [&](int64_t r, int buf) {
    const StageSrc src = stage_src(r);
    [&]<int... D>(std::integer_sequence<int, D...>) {
      (issue_one(std::integral_constant<int, D>{}, src, buf), ...);
    }(std::make_integer_sequence<int, C::LPW>{});
  };

  f32x4_t acc[IT][JT];
#pragma unroll
  for (int i = 0; i < IT; ++i)
#pragma unroll
    for (int j = 0; j < JT; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  u32x4_t pf[IT], qf[JT];
  auto read_frags = [&](int buf) {
    const unsigned char* base = smem + buf * C::STAGE;
#pragma unroll
    for (int i = 0; i < IT; ++i) pf[i] = read_transposed<C::P_ROWB>(base, wi * IT + i, c16, kb);
#pragma unroll
    for (int j = 0; j < JT; ++j) {
      if (Q_STRIDED) {
        qf[j] = read_transposed<C::Q_ROWB>(base + C::P_BYTES, wj * JT + j, c16, kb);
      } else {
        const int row = (wj * JT + j) * 16 + c16;
        qf[j] = *reinterpret_cast<const u32x4_t*>(base + C::P_BYTES + row * 64 + ((kb ^ ((c16 >> 1) & 3)) << 4));
      }
    }
  };
  // 32 matrix instructions; the wave's loads of a later stage are issued between them
  auto multiply = [&](bool load, int64_t lr, int lbuf) {
    const StageSrc src = stage_src(load ? lr : r_first);
    [&]<int... Q>(std::integer_sequence<int, Q...>) {
      ([&] {
        constexpr int j = Q / IT, i = Q % IT;
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, pf[i]),
                                                            __builtin_bit_cast(bf16x8_t, qf[j]), acc[i][j], 0, 0, 0);
        if constexpr (Q % 4 == 3 && Q / 4 < C::LPW) {
          if (load) issue_one(std::integral_constant<int, Q / 4>{}, src, lbuf);
          __builtin_amdgcn_sched_barrier(0);
        }
      }(), ...);
    }(std::make_integer_sequence<int, C::MMA>{});
  };
  auto wait_stage = [&](int younger) {
    [&]<int... Y>(std::integer_sequence<int, Y...>) {
      ((younger == Y ? wait_loads_outstanding<Y * C::LPW>() : void()), ...);
    }(std::make_integer_sequence<int, STAGES - 1>{});
  };

#pragma unroll
  for (int s = 0; s < STAGES - 1; ++s)
    if (s < nk) issue_stage(r_first + (int64_t)s * C::RS, s);

  // One barrier per stage; the buffer multiplied in the previous step is refilled right after the barrier,
  // STAGES - 1 stages ahead.
  {
    int buf = 0;
    int64_t ks = 0;
    // Steady state, free of conditions: while the stage to be fetched exists and has all its rows (then so has
    // the one being multiplied), the waits are fixed, no row is clamped or cleared, and the operand addresses
    // advance by additions.  A wave issues in order, so every scalar and vector instruction saved here is issue
    // time its matrix instructions get.  The last STAGES - 1 steps (and a ragged last stage of the reduction)
    // take the general form below.
    int64_t n_fast = nk - (STAGES - 1);
    if (n_fast > 0 && a.R - (r_first + (nk - 1) * C::RS) < C::RS) --n_fast;
    if (n_fast > 0) {
      const int64_t r_load = r_first + (int64_t)(STAGES - 1) * C::RS;
      const unsigned char* fp = reinterpret_cast<const unsigned char*>(p_base + r_load * a.ldp);
      const unsigned char* fq = reinterpret_cast<const unsigned char*>(Q_STRIDED ? q_base + r_load * a.ldq : q_base + r_load);
      const int64_t p_step = (int64_t)C::RS * a.ldp * 2, q_step = Q_STRIDED ? (int64_t)C::RS * a.ldq * 2 : (int64_t)C::RS * 2;
      uint32_t lds_load = lds0 + (uint32_t)((STAGES - 1) * C::STAGE);  // LDS address of the buffer to be refilled
      for (; ks < n_fast; ++ks) {
        wait_loads_outstanding<(STAGES - 2) * C::LPW>();
        __builtin_amdgcn_s_barrier();
        read_frags(buf);
        const uniform_ptr_t up = make_uniform(fp), uq = make_uniform(fq);
        const uint32_t lds = __builtin_amdgcn_readfirstlane(lds_load);
        [&]<int... Q>(std::integer_sequence<int, Q...>) {
          ([&] {
            constexpr int j = Q / IT, i = Q % IT;
            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, pf[i]),
                                                                __builtin_bit_cast(bf16x8_t, qf[j]), acc[i][j], 0, 0, 0);
            if constexpr (Q % 4 == 3 && Q / 4 < C::LPW) {
              constexpr int d = Q / 4;
              if constexpr (d < C::P_PW) dma16(up, p_voff[d], lds + p_dst[d]);
              else dma16(uq, q_voff[d - C::P_PW], lds + q_dst[d - C::P_PW]);
              __builtin_amdgcn_sched_barrier(0);
            }
          }(), ...);
        }(std::make_integer_sequence<int, C::MMA>{});
        fp += p_step;
        fq += q_step;
        lds_load += (uint32_t)C::STAGE;
        if (lds_load == lds0 + (uint32_t)(STAGES * C::STAGE)) lds_load = lds0;
        if (++buf == STAGES) buf = 0;
      }
    }
    for (; ks < nk; ++ks) {
      const int64_t ahead = nk - 1 - ks;  // stages after this one; the loads of at most STAGES - 2 of them are out
      wait_stage(ahead < STAGES - 2 ? (int)ahead : STAGES - 2);
      const int64_t r = r_first + ks * C::RS;
      if (a.R - r < C::RS) {
        // ragged last stage of the reduction: this wave's own loads have landed; it clears the rows past R
        // it fetched (reduction-major tiles only; the other form requires R % 32 == 0)
        const int rows_left = (int)(a.R - r);
        unsigned char* base = smem + buf * C::STAGE;
#pragma unroll
        for (int d = 0; d < C::P_PW; ++d)
          if (p_row[d] >= rows_left) *reinterpret_cast<u32x4_t*>(base + p_dst[d] + lane * 16) = u32x4_t{0, 0, 0, 0};
        if (Q_STRIDED) {
#pragma unroll
          for (int d = 0; d < C::Q_PW; ++d)
            if (q_row[d] >= rows_left) *reinterpret_cast<u32x4_t*>(base + q_dst[d] + lane * 16) = u32x4_t{0, 0, 0, 0};
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      }
      __builtin_amdgcn_s_barrier();
      int nbuf = buf + STAGES - 1;
      if (nbuf >= STAGES) nbuf -= STAGES;
      read_frags(buf);
      multiply(ks + STAGES - 1 < nk, r + (int64_t)(STAGES - 1) * C::RS, nbuf);
      if (++buf == STAGES) buf = 0;
    }
  }

  // ---- split reduction: the partial tile, 16 bytes per lane and accumulator, fully coalesced
  if (a.partial) {
    f32x4_t* mine = reinterpret_cast<f32x4_t*>(a.partial) + ((size_t)split * n_tiles + tile) * (C::MMA * C::NT) + tid;
#pragma unroll
    for (int i = 0; i < IT; ++i)
#pragma unroll
      for (int j = 0; j < JT; ++j) mine[(i * JT + j) * C::NT] = acc[i][j];
    return;
  }

  // ---- write-out.  A lane holds columns i .. i+3 (accumulator element e -> row 4 kb + e of the 16-row block)
  // of output row j = c16, i.e. 8 or 16 contiguous bytes of an Out row.  For aligned outputs every wave
  // transposes 16 output rows at a time through its own LDS slice, so that the global stores are 16 bytes
  // per lane and whole row segments of the wave tile are written contiguously.
  __builtin_amdgcn_s_barrier();  // every wave is done with the operand stages
  auto get = [&](int i, int j) { return __builtin_bit_cast(u32x4_t, acc[i][j]); };
  const int64_t row0 = j0 + wj * JT * 16, col0 = i0 + wi * IT * 16;
  static_assert(C::NW * wave_tile_slice_bytes<IT, 4>() <= C::LDS_BYTES, "write-out slices");
  if (a.vec_store) {
    if (a.out_bf16)
      write_wave_tile_pieces<IT, JT, 2>(smem + wave * wave_tile_slice_bytes<IT, 2>(), lane, get, a.out, a.ldo, row0, col0, a.J, a.I);
    else
      write_wave_tile_pieces<IT, JT, 4>(smem + wave * wave_tile_slice_bytes<IT, 4>(), lane, get, a.out, a.ldo, row0, col0, a.J, a.I);
  } else {
    write_wave_tile_elements<IT, JT>(lane, get, a.out, a.ldo, row0, col0, a.J, a.I, a.out_bf16 != 0);
  }
}

// Sum of the partial tiles in split order, the mask of the step (bit k % 32 of word k / 32 of row o; NULL =
// every weight receives its gradient) and the rounding.  One lane per accumulator of the tile kernel.
__global__ void __launch_bounds__(256)
grad_reduce_kernel(const float* __restrict__ partial, int splits, int n_tiles, int n_i_tiles, int64_t I, int64_t J,
                   const uint32_t* __restrict__ mask, void* __restrict__ out, int64_t ldo, int out_bf16) {
  using C = TCfg;
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= (int64_t)n_tiles * C::MMA * C::NT) return;
  const int tid = (int)(id % C::NT);
  const int q = (int)((id / C::NT) % C::MMA);
  const int tile = (int)(id / (C::NT * C::MMA));
  const f32x4_t* src = reinterpret_cast<const f32x4_t*>(partial) + id;
  const size_t stride = (size_t)n_tiles * (C::MMA * C::NT);
  f32x4_t sum = src[0];
  for (int s = 1; s < splits; ++s) sum += src[(size_t)s * stride];
  const int lane = tid & 63, wave = tid >> 6;
  const int wi = wave % C::WI, wj = wave / C::WI;
  const int i = q / C::JT, j = q % C::JT;
  const int64_t ii = (int64_t)(tile % n_i_tiles) * C::BI + (wi * C::IT + i) * 16 + (lane >> 4) * 4;
  const int64_t jj = (int64_t)(tile / n_i_tiles) * C::BJ + (wj * C::JT + j) * 16 + (lane & 15);
  if (jj >= J || ii >= I) return;
  if (mask) {
    const uint32_t w = mask[jj * ((I + 31) / 32) + (ii >> 5)] >> (ii & 31);  // I % 4 == 0: the four bits share a word
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (!((w >> e) & 1u)) sum[e] = 0.f;
  }
  if (out_bf16) {
    bf16_t* dst = reinterpret_cast<bf16_t*>(out) + jj * ldo + ii;
    if (ii + 3 < I && ((uintptr_t)dst & 7) == 0) {
      *reinterpret_cast<uint2*>(dst) = make_uint2(pack_bf16x2(sum[0], sum[1]), pack_bf16x2(sum[2], sum[3]));
    } else {
      for (int e = 0; e < 4 && ii + e < I; ++e) dst[e] = (bf16_t)f32_to_bf16_rne(sum[e]);
    }
  } else {
    float* dst = reinterpret_cast<float*>(out) + jj * ldo + ii;
    if (ii + 3 < I && ((uintptr_t)dst & 15) == 0) {
      *reinterpret_cast<f32x4_t*>(dst) = sum;
    } else {
      for (int e = 0; e < 4 && ii + e < I; ++e) dst[e] = sum[e];
    }
  }
}

// Any shape and alignment: one lane per output, a plain loop over the reduction.
__global__ void __launch_bounds__(256)
backward_input_general_kernel(const bf16_t* __restrict__ Ws, int64_t O, int64_t K, int64_t ldw,
                              const bf16_t* __restrict__ dY, int64_t T, int64_t ldy, void* __restrict__ dX, int64_t ldx,
                              int out_bf16) {
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= T * K) return;
  const int64_t t = id / K, k = id % K;
  float acc = 0.f;
  for (int64_t o = 0; o < O; ++o) acc = fmaf(bf16_to_f32(dY[t * ldy + o]), bf16_to_f32(Ws[o * ldw + k]), acc);
  if (out_bf16) reinterpret_cast<bf16_t*>(dX)[t * ldx + k] = (bf16_t)f32_to_bf16_rne(acc);
  else reinterpret_cast<float*>(dX)[t * ldx + k] = acc;
}

__global__ void __launch_bounds__(256)
backward_weight_general_kernel(const bf16_t* __restrict__ dY, int64_t T, int64_t O, int64_t ldy,
                               const bf16_t* __restrict__ X, int64_t K, int64_t ldx, const uint32_t* __restrict__ mask,
                               void* __restrict__ dW, int64_t lddw, int out_bf16) {
  const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (id >= O * K) return;
  const int64_t o = id / K, k = id % K;
  float acc = 0.f;
  if (!mask || ((mask[o * ((K + 31) / 32) + (k >> 5)] >> (k & 31)) & 1u))
    for (int64_t t = 0; t < T; ++t) acc = fmaf(bf16_to_f32(dY[t * ldy + o]), bf16_to_f32(X[t * ldx + k]), acc);
  if (out_bf16) reinterpret_cast<bf16_t*>(dW)[o * lddw + k] = (bf16_t)f32_to_bf16_rne(acc);
  else reinterpret_cast<float*>(dW)[o * lddw + k] = acc;
}

inline bool aligned_to(const void* p, uintptr_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

template <bool Q_STRIDED>
hipError_t launch_tgemm(TGemmArgs g, hipStream_t s) {
  using C = TCfg;
  auto kern = nm_tgemm_kernel<Q_STRIDED>;
  static PerDeviceOnce lds_limit;
  if (hipError_t e = raise_dynamic_lds_limit(kern, C::LDS_BYTES, lds_limit); e != hipSuccess) return e;
  const int64_t n_tiles = (int64_t)g.n_i_tiles * g.n_j_tiles;
  const int64_t grid = ((n_tiles * g.splits + 7) / 8) * 8;
  if (grid > 0x7FFFFFFF) return hipErrorInvalidValue;
  hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(C::NT), C::LDS_BYTES, s, g);
  return hipGetLastError();
}

// Ranges of the token reduction of dW.  Two blocks fit a compute unit, 512 at once on a 256-unit chip; the
// smallest count that fills at least 90 % of a whole number of such rounds is taken (else the fullest), with
// at least four steps per range where the reduction is long enough.
struct WeightGradPlan {
  bool tiles;  // the matrix-core kernel takes this shape
  int n_i_tiles, n_j_tiles, splits;
};
WeightGradPlan weight_grad_plan(int64_t O, int64_t K, int64_t T) {
  WeightGradPlan p{false, 0, 0, 0};
  if ((O % 8) || (K % 8) || O > (1 << 24) || K > (1 << 22) || T > (1ll << 31)) return p;
  const int64_t ni = (K + TCfg::BI - 1) / TCfg::BI, nj = (O + TCfg::BJ - 1) / TCfg::BJ;
  if (ni * nj > (1 << 20)) return p;
  p.tiles = true;
  p.n_i_tiles = (int)ni;
  p.n_j_tiles = (int)nj;
  const int64_t steps = (T + TCfg::RS - 1) / TCfg::RS, tiles = ni * nj;
  int best = 1;
  double best_fill = 0.0;
  for (int s = 1; s <= 64; ++s) {
    if (s > 1 && steps / s < 4) break;
    const int64_t blocks = tiles * s, rounds = (blocks + 511) / 512;
    const double fill = (double)blocks / (double)(rounds * 512);
    if (fill > best_fill + 1e-9) { best = s; best_fill = fill; }
    if (fill >= 0.9) break;
  }
  p.splits = best;
  return p;
}

}  // namespace

size_t backward_input_workspace_bytes(int64_t O, int64_t K, int64_t T) {
  return dense_transposed_workspace_bytes(O, K, T);
}

hipError_t launch_backward_input(const bf16_t* Ws, int64_t O, int64_t K, int64_t ldw, const bf16_t* dY, int64_t T,
                                 int64_t ldy, void* dX, int64_t ldx, int out_bf16, void* workspace,
                                 size_t workspace_bytes, hipStream_t s, bool* workspace_short) {
  *workspace_short = false;
  // Large layers: dX = dY * Ws is the forward product of a layer whose weight is Ws^T, so once the weight has
  // been written transposed into stream order (a pass over the weight only) the persistent dense kernel of the
  // forward path computes it.
  const size_t need = backward_input_workspace_bytes(O, K, T);
  if (need) {
    if (workspace == nullptr || workspace_bytes < need || !aligned_to(workspace, 256)) {
      *workspace_short = true;
      return hipSuccess;
    }
    bool taken = false;
    hipError_t e = launch_dense_transposed(Ws, O, K, ldw, dY, T, ldy, dX, ldx, out_bf16, workspace, workspace_bytes, s,
                                           &taken);
    if (e != hipSuccess || taken) return e;
  }
  const bool tiles = (O % 32 == 0) && (K % 8 == 0) && (ldw % 8 == 0) && (ldy % 8 == 0) && aligned_to(Ws, 16) &&
                     aligned_to(dY, 16) && K <= (1 << 24) && T <= (1ll << 31) && ldw <= (1 << 22) && ldy <= (1 << 22);
  if (!tiles) {
    if (T * K > 0x7FFFFFFFll * 256) return hipErrorInvalidValue;
    hipLaunchKernelGGL(backward_input_general_kernel, dim3((unsigned)((T * K + 255) / 256)), dim3(256), 0, s, Ws, O, K, ldw,
                       dY, T, ldy, dX, ldx, out_bf16);
    return hipGetLastError();
  }
  TGemmArgs g;
  g.P = Ws; g.Q = dY; g.I = K; g.J = T; g.R = O; g.ldp = ldw; g.ldq = ldy;
  g.out = dX; g.ldo = ldx; g.out_bf16 = out_bf16;
  const int per_piece = out_bf16 ? 8 : 4;
  g.vec_store = (ldx % per_piece == 0) && aligned_to(dX, 16);  // K % 8 == 0 holds here
  g.n_i_tiles = (int)((K + TCfg::BI - 1) / TCfg::BI);
  g.n_j_tiles = (int)((T + TCfg::BJ - 1) / TCfg::BJ);
  g.splits = 1; g.partial = nullptr;
  return launch_tgemm<false>(g, s);
}

size_t backward_weight_workspace_bytes(int64_t O, int64_t K, int64_t T) {
  const WeightGradPlan p = weight_grad_plan(O, K, T);
  if (!p.tiles) return 0;
  return (size_t)p.splits * (size_t)p.n_i_tiles * (size_t)p.n_j_tiles * (size_t)(TCfg::BI * TCfg::BJ) * sizeof(float);
}

hipError_t launch_backward_weight(const bf16_t* dY, int64_t T, int64_t O, int64_t ldy, const bf16_t* X, int64_t K,
                                  int64_t ldx, const uint32_t* mask, void* dW, int64_t lddw, int out_bf16, void* workspace,
                                  size_t workspace_bytes, hipStream_t s, bool* workspace_short) {
  *workspace_short = false;
  const WeightGradPlan p = weight_grad_plan(O, K, T);
  const bool tiles = p.tiles && (ldy % 8 == 0) && (ldx % 8 == 0) && aligned_to(dY, 16) && aligned_to(X, 16) &&
                     ldx <= (1 << 22) && ldy <= (1 << 22);
  if (!tiles) {
    if (O * K > 0x7FFFFFFFll * 256) return hipErrorInvalidValue;
    hipLaunchKernelGGL(backward_weight_general_kernel, dim3((unsigned)((O * K + 255) / 256)), dim3(256), 0, s, dY, T, O, ldy,
                       X, K, ldx, mask, dW, lddw, out_bf16);
    return hipGetLastError();
  }
  const size_t need = backward_weight_workspace_bytes(O, K, T);
  if (workspace == nullptr || workspace_bytes < need || !aligned_to(workspace, 256)) {
    *workspace_short = true;
    return hipSuccess;
  }
  TGemmArgs g;
  g.P = X; g.Q = dY; g.I = K; g.J = O; g.R = T; g.ldp = ldx; g.ldq = ldy;
  g.out = nullptr; g.ldo = 0; g.out_bf16 = 0; g.vec_store = 0;
  g.n_i_tiles = p.n_i_tiles; g.n_j_tiles = p.n_j_tiles;
  g.splits = p.splits; g.partial = reinterpret_cast<float*>(workspace);
  hipError_t e = launch_tgemm<true>(g, s);
  if (e != hipSuccess) return e;
  const int64_t n = (int64_t)p.n_i_tiles * p.n_j_tiles * TCfg::MMA * TCfg::NT;
  hipLaunchKernelGGL(grad_reduce_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, g.partial, p.splits,
                     p.n_i_tiles * p.n_j_tiles, p.n_i_tiles, K, O, mask, dW, lddw, out_bf16);
  return hipGetLastError();
}

}  // namespace nm
