// Host-side launch interface between the C ABI layer and the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace nm {

typedef uint16_t bf16_t;

// One-time setup of a kernel on the current device.  Function attributes and the compute-unit count belong to a
// device, and a process may drive several (one current at a time), so the "done" marks are kept per device.
// A race between threads only repeats an idempotent call.
constexpr int kMaxDevices = 64;
struct PerDeviceOnce {
  bool done[kMaxDevices] = {};
};
inline hipError_t current_device_slot(int* dev) {
  hipError_t e = hipGetDevice(dev);
  if (e != hipSuccess) return e;
  return (*dev >= 0 && *dev < kMaxDevices) ? hipSuccess : hipErrorInvalidDevice;
}
template <typename Kernel>
inline hipError_t raise_dynamic_lds_limit(Kernel kern, int bytes, PerDeviceOnce& once) {
  int dev = 0;
  hipError_t e = current_device_slot(&dev);
  if (e != hipSuccess) return e;
  if (once.done[dev]) return hipSuccess;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e != hipSuccess) return e;
  once.done[dev] = true;
  return hipSuccess;
}
// Compute units of the current device (cached per device).
inline hipError_t compute_units(int* n) {
  static int cached[kMaxDevices] = {};
  int dev = 0;
  hipError_t e = current_device_slot(&dev);
  if (e != hipSuccess) return e;
  if (!cached[dev]) {
    int cus = 0;
    if ((e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return e;
    cached[dev] = cus > 0 ? cus : 1;
  }
  *n = cached[dev];
  return hipSuccess;
}

struct PackDesc {
  const bf16_t* W;
  bf16_t* values;
  uint32_t* indices;
  int64_t O, K;
  int32_t N, M;
};
struct PackRankedDesc {
  const bf16_t* W;
  const uint8_t* rank;
  bf16_t* values;
  uint32_t* indices;
  int64_t O, K;
  int32_t N, M;
};

// nm_pack.hip
hipError_t launch_prune(const bf16_t* W, int64_t O, int64_t K, int64_t ldw, int N, int M, uint32_t* mask,
                        bf16_t* w_masked, hipStream_t s);
hipError_t launch_pack(const bf16_t* W, int64_t O, int64_t K, int64_t ldw, int N, int M, const uint32_t* mask,
                       bf16_t* values, uint32_t* indices, hipStream_t s);
hipError_t launch_pack_batched(const PackDesc* descs, int count, hipStream_t s);
// pack + operand-order workspace of the product at T tokens, for many layers
struct LayerDesc {
  const bf16_t* W;
  bf16_t* values;
  uint32_t* indices;
  int64_t O, K;
  int32_t N, M;
  int64_t T;
  void* workspace;
  size_t workspace_bytes;
};
hipError_t launch_pack_prepare_batched(const LayerDesc* descs, int count, hipStream_t s, bool* workspace_short);
hipError_t launch_unpack(const bf16_t* values, const uint32_t* indices, int64_t O, int64_t K, int N, int M,
                         bf16_t* Wd, int64_t ldw, hipStream_t s);
hipError_t launch_pack_ranked_batched(const PackRankedDesc* descs, int count, hipStream_t s);
hipError_t launch_pack_ranked(const bf16_t* W, const uint8_t* rank, int64_t O, int64_t K, int64_t ldw, int N, int M,
                              bf16_t* values, uint32_t* indices, hipStream_t s);
hipError_t launch_mask_check(const uint32_t* mask, int64_t O, int64_t K, int N, int M, uint32_t* bad, hipStream_t s);

// nm_rank.hip
hipError_t launch_rank(const bf16_t* W, int64_t O, int64_t K, int64_t ldw, int M, uint8_t* rank, hipStream_t s);
struct RankDesc {
  const bf16_t* W;
  uint8_t* rank;
  int64_t O, K;
  int32_t M, reserved;
};
hipError_t launch_rank_batched(const RankDesc* descs, int count, hipStream_t s);
hipError_t launch_score_mask(const float* score, int64_t O, int64_t K, int64_t lds, int N, int M, uint32_t* mask,
                             hipStream_t s);
hipError_t launch_rank_mask(const uint8_t* rank, int64_t O, int64_t K, int N, uint32_t* mask, hipStream_t s);

// nm_spmm.hip
struct SpmmArgs {
  const bf16_t* values;
  const uint32_t* indices;
  int64_t O, K;
  int N, M;
  const bf16_t* X;
  int64_t T, ldx;
  const float* bias;  // nullable
  void* Y;
  int64_t ldy;
  int out_bf16;
  void* workspace;
  size_t workspace_bytes;
};
size_t spmm_workspace_bytes(int64_t O, int64_t K, int N, int M, int64_t T);
size_t spmm_operand_workspace_bytes(int64_t O, int64_t K, int N, int M, int64_t T);  // the part that is required
bool spmm_stream_order(int64_t O, int64_t K, int64_t T, int N, int M, bool* sparse_form);
// phases: SPMM_PREPARE rewrites the packed weight into matrix-core operand order in the workspace,
// SPMM_PRODUCT multiplies (expects a prepared workspace); both = the whole call.
// returns hipSuccess or the launch error; *workspace_short is set when the workspace is required but
// missing, misaligned or too small (nothing is launched then)
enum { SPMM_PREPARE = 1, SPMM_PRODUCT = 2 };
hipError_t launch_spmm(const SpmmArgs& a, hipStream_t s, bool* workspace_short, int phases);
// the products (SPMM_PRODUCT) of many prepared layers, sharing launches where the shapes allow
// (the caller has checked the workspaces with spmm_workspace_short)
bool spmm_workspace_short(const SpmmArgs& a);
hipError_t launch_spmm_batched(const SpmmArgs* layers, int count, hipStream_t s);

// nm_fewtok.hip: products at few tokens straight from the packed format (no workspace)
bool fewtok_shape(int64_t O, int64_t K, int N, int M, int64_t T);
bool fewtok_takes(const SpmmArgs& a);
hipError_t launch_fewtok(const SpmmArgs* const* layers, int count, hipStream_t s);

// Out[t, i] = sum_r Q[t, r] * Ws[r, i] on the persistent dense product kernel (weight transposed into stream
// order in the workspace first); *taken stays false, and nothing is launched, when the shape, the alignment or
// the workspace do not allow it.
size_t dense_transposed_workspace_bytes(int64_t R, int64_t I, int64_t T);
hipError_t launch_dense_transposed(const bf16_t* Ws, int64_t R, int64_t I, int64_t ldw, const bf16_t* Q, int64_t T,
                                   int64_t ldq, void* Out, int64_t ldo, int out_bf16, void* workspace,
                                   size_t workspace_bytes, hipStream_t s, bool* taken);

// nm_grad.hip: training products of a layer.  Ws is the masked dense weight [O, K].
size_t backward_input_workspace_bytes(int64_t O, int64_t K, int64_t T);
hipError_t launch_backward_input(const bf16_t* Ws, int64_t O, int64_t K, int64_t ldw, const bf16_t* dY, int64_t T,
                                 int64_t ldy, void* dX, int64_t ldx, int out_bf16, void* workspace,
                                 size_t workspace_bytes, hipStream_t s, bool* workspace_short);
size_t backward_weight_workspace_bytes(int64_t O, int64_t K, int64_t T);
// *workspace_short is set when the workspace is required but missing, misaligned or too small
hipError_t launch_backward_weight(const bf16_t* dY, int64_t T, int64_t O, int64_t ldy, const bf16_t* X, int64_t K,
                                  int64_t ldx, const uint32_t* mask, void* dW, int64_t lddw, int out_bf16, void* workspace,
                                  size_t workspace_bytes, hipStream_t s, bool* workspace_short);

// nm_spmm.hip: the int8 layer on the persistent kernel (operands in stream order, O padded to 256 rows)
struct StreamI8Args {
  const int8_t* values;  // stream-order compressed values (2:4 form) or masked dense weight
  const uint32_t* sel;   // stream-order selector words (2:4 form)
  bool sparse_form;
  const int8_t* X;
  const float* w_scale;  // nullable; 16-byte aligned
  const float* bias;     // nullable; 16-byte aligned
  float x_scale;
  void* Y;
  int64_t O, K, T, ldx, ldy;
  int out_kind;
};
bool stream_i8_takes(int64_t O, int64_t K, int64_t T, int N, int M);
hipError_t launch_stream_i8(const StreamI8Args& a, hipStream_t s);

// nm_probe.hip: measurement aids (matrix-instruction rate, streaming copy rate)
constexpr int kMaxProbeBlocks = 2048;
size_t probe_sink_bytes();
hipError_t launch_probe_matrix(int kind, int iters, float* sink, int64_t* ops, hipStream_t s);
hipError_t launch_probe_copy(const void* src, void* dst, size_t bytes, hipStream_t s);

// nm_int8.hip: the int8 layer.  Phases as for launch_spmm.
struct I8LinearArgs {
  const int8_t* Wq;      // dense int8 weight [O, K], ld ldw; NULL = the weight comes compressed (values, indices)
  int64_t ldw;
  const uint32_t* mask;  // mask words [O, ceil(K/32)]
  const int8_t* values;  // compressed form: kept values [O, K N/M] ...
  const uint32_t* indices;  // ... and the index stream of the bfloat16 layer
  int64_t O, K;
  int N, M;
  const int8_t* X;
  int64_t T, ldx;
  float x_scale;
  const float* w_scale;  // nullable
  const float* bias;     // nullable
  void* Y;
  int64_t ldy;
  int out_kind;          // 0 float, 1 bfloat16, 2 int32 accumulators
  void* workspace;
  size_t workspace_bytes;
};
size_t i8_workspace_bytes(int64_t O, int64_t K, int N, int M, int64_t T);
hipError_t launch_linear_i8(const I8LinearArgs& a, hipStream_t s, bool* workspace_short, int phases);
// compressed form of the int8 weight under a mask, and back
hipError_t launch_pack_i8(const int8_t* Wq, int64_t O, int64_t K, int64_t ldw, int N, int M, const uint32_t* mask,
                          int8_t* values, uint32_t* indices, hipStream_t s);
hipError_t launch_unpack_i8(const int8_t* values, const uint32_t* indices, int64_t O, int64_t K, int N, int M, int8_t* Wd,
                            int64_t ldw, hipStream_t s);

}  // namespace nm
