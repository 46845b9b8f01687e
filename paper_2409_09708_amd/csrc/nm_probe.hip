// Measurement aids: the two rates the product and packing kernels are priced against, measured on the device at
// hand instead of taken from a data sheet.  Neither is part of the layer.
//
//  * matrix rate: a loop of nothing but matrix instructions on register operands (finite pseudo-random bf16
//    patterns; constant operands would let the clock run higher than real data does), 32 independent
//    accumulator blocks per wave, two waves per SIMD, every compute unit busy.
//  * copy rate: a plain streaming copy, 16 bytes per lane, eight blocks per compute unit.  Its known traffic also
//    scales the profiler's byte counters.
#include "nm_device.h"
#include "nm_launch.h"
#include "nm_mma.h"

namespace nm {

namespace {

__device__ __forceinline__ uint32_t mix(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}
// two bf16 of magnitude in [0.5, 2) with random sign and fraction
__device__ __forceinline__ uint32_t finite_pair(uint32_t h) { return (h & 0x80FF80FFu) | 0x3F003F00u; }

template <int KIND>  // 0: v_smfmac_f32_16x16x64_bf16, 1: v_mfma_f32_16x16x32_bf16
__global__ void __launch_bounds__(256, 2) matrix_rate_kernel(int iters, float* sink) {
  constexpr int OT = 4, TT = 8;
  const uint32_t seed = mix(blockIdx.x * 256u + threadIdx.x + 1u);
  u32x4_t a[OT];
  u32x8_t b[TT];
  int sel[OT];
#pragma unroll
  for (int i = 0; i < OT; ++i) {
#pragma unroll
    for (int e = 0; e < 4; ++e) a[i][e] = finite_pair(mix(seed + 17u * i + e));
    // legal selector pairs (first < second inside every run of four)
    sel[i] = (int)0x4E4E4E4Eu;
  }
#pragma unroll
  for (int j = 0; j < TT; ++j)
#pragma unroll
    for (int e = 0; e < 8; ++e) b[j][e] = finite_pair(mix(seed + 1000u + 31u * j + e));
  f32x4_t acc[OT][TT];
#pragma unroll
  for (int i = 0; i < OT; ++i)
#pragma unroll
    for (int j = 0; j < TT; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < TT; ++j)
#pragma unroll
      for (int i = 0; i < OT; ++i) {
        if constexpr (KIND == 0)
          acc[i][j] = __builtin_amdgcn_smfmac_f32_16x16x64_bf16(__builtin_bit_cast(bf16x8_t, a[i]),
                                                                __builtin_bit_cast(bf16x16_t, b[j]), acc[i][j], sel[i], 0, 0);
        else
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
              __builtin_bit_cast(bf16x8_t, a[i]),
              __builtin_bit_cast(bf16x8_t, u32x4_t{b[j][0], b[j][1], b[j][2], b[j][3]}), acc[i][j], 0, 0, 0);
      }
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < OT; ++i)
#pragma unroll
    for (int j = 0; j < TT; ++j) s += acc[i][j][0] + acc[i][j][1] + acc[i][j][2] + acc[i][j][3];
  sink[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

// every block copies one contiguous share, four 16-byte pieces per lane in flight, loads and stores with the
// non-temporal hint (nothing is reused): of the forms tried (grid-strided or block-contiguous, with and without the
// hint, 2 to 32 blocks per compute unit) this one was the fastest that is also steady from run to run
__global__ void __launch_bounds__(256) copy_kernel(const u32x4_t* __restrict__ src, u32x4_t* __restrict__ dst, size_t n) {
  const size_t per = (n + gridDim.x - 1) / gridDim.x;
  const size_t b0 = (size_t)blockIdx.x * per, b1 = b0 + per < n ? b0 + per : n;
  size_t i = b0 + threadIdx.x;
  for (; i + 3 * 256 < b1; i += 4 * 256) {
    u32x4_t v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = __builtin_nontemporal_load(src + i + u * 256);
#pragma unroll
    for (int u = 0; u < 4; ++u) __builtin_nontemporal_store(v[u], dst + i + u * 256);
  }
  for (; i < b1; i += 256) dst[i] = src[i];
}

}  // namespace

hipError_t launch_probe_matrix(int kind, int iters, float* sink, int64_t* flops, hipStream_t s) {
  int cus = 0;
  if (hipError_t e = compute_units(&cus); e != hipSuccess) return e;
  // two blocks of four waves per compute unit: two waves per SIMD
  const unsigned grid = (unsigned)(cus * 2 < kMaxProbeBlocks ? cus * 2 : kMaxProbeBlocks);
  if (kind == 0) hipLaunchKernelGGL(matrix_rate_kernel<0>, dim3(grid), dim3(256), 0, s, iters, sink);
  else hipLaunchKernelGGL(matrix_rate_kernel<1>, dim3(grid), dim3(256), 0, s, iters, sink);
  // dense-equivalent operations: 2 * 16 * 16 * K per instruction, K = 64 (2:4 form) or 32
  *flops = (int64_t)grid * 4 * iters * 32 * (2ll * 16 * 16 * (kind == 0 ? 64 : 32));
  return hipGetLastError();
}

size_t probe_sink_bytes() { return (size_t)kMaxProbeBlocks * 256 * sizeof(float); }

hipError_t launch_probe_copy(const void* src, void* dst, size_t bytes, hipStream_t s) {
  int cus = 0;
  if (hipError_t e = compute_units(&cus); e != hipSuccess) return e;
  hipLaunchKernelGGL(copy_kernel, dim3((unsigned)cus * 8), dim3(256), 0, s, reinterpret_cast<const u32x4_t*>(src),
                     reinterpret_cast<u32x4_t*>(dst), bytes / 16);
  return hipGetLastError();
}

}  // namespace nm
