// C ABI of the N:M-sparse linear layer: argument validation on the host, then kernel launches on
// the caller's stream.  Declarations and the contract of every call are in include/nm_sparse.h.
#include "nm_sparse.h"

#include "nm_device.h"
#include "nm_launch.h"

#include <atomic>

namespace {

thread_local int32_t g_last_hip_error = 0;

// Scratch of nm_linear_forward_static: device memory that exists as long as the library is loaded, one copy on
// every device the library runs on.  In host code the array's name is only a handle; the memory's address on the
// current device comes from hipGetSymbolAddress (asked once per device) and is what the kernels receive.
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
__device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
std::atomic<unsigned char*> g_scratch_ptr[nm::kMaxDevices];

hipError_t static_scratch(unsigned char** ptr) {
  int dev = 0;
  hipError_t e = nm::current_device_slot(&dev);
  if (e != hipSuccess) return e;
  unsigned char* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (p == nullptr) {
    void* addr = nullptr;
    if ((e = hipGetSymbolAddress(&addr, HIP_SYMBOL(scratch))) != hipSuccess) return e;
    if (addr == nullptr) return hipErrorInvalidSymbol;
    p = static_cast<unsigned char*>(addr);
    g_scratch_ptr[dev].store(p, std::memory_order_release);
  }
  *ptr = p;
  return hipSuccess;
}

inline int32_t device_status(hipError_t e) {
  if (e == hipSuccess) return NM_OK;
  g_last_hip_error = (int32_t)e;
  return NM_ERR_DEVICE;
}

inline bool level_ok(int32_t N, int32_t M) { return (M == 4 || M == 8 || M == 16) && N >= 1 && N <= M; }

inline bool aligned(const void* p, uintptr_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

// shape of a weight: level first (so that an illegal M never reaches a modulo), then sizes
inline int32_t check_weight(int64_t O, int64_t K, int32_t N, int32_t M) {
  if (!level_ok(N, M)) return NM_ERR_LEVEL;
  if (O <= 0 || K <= 0 || (K % M) != 0) return NM_ERR_SHAPE;
  if (O > (int64_t)1 << 31 || K > (int64_t)1 << 31) return NM_ERR_SHAPE;
  if (O * K > (int64_t)1 << 40) return NM_ERR_SHAPE;  // every launcher's grid (at most one block per 1024 weights) fits 2^31 - 1
  return NM_OK;
}

}  // namespace

extern "C" {

const char* nm_status_string(int32_t status) {
  switch (status) {
    case NM_OK: return "ok";
    case NM_ERR_NULL: return "a required pointer is NULL";
    case NM_ERR_SHAPE: return "illegal shape (sizes must be positive, K a multiple of M, leading dimensions >= row length)";
    case NM_ERR_LEVEL: return "illegal N:M level (M in {4, 8, 16}, 1 <= N <= M)";
    case NM_ERR_ALIGN: return "a pointer is not aligned as documented";
    case NM_ERR_DTYPE: return "unknown output type";
    case NM_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case NM_ERR_DEVICE: return "a HIP call failed (see nm_last_hip_error)";
    case NM_ERR_EXHAUSTED: return "random numbers exhausted before a configuration fell into the interval";
    default: return "unknown status";
  }
}

int32_t nm_last_hip_error(void) { return g_last_hip_error; }

size_t nm_values_bytes(int64_t O, int64_t K, int32_t N, int32_t M) {
  if (check_weight(O, K, N, M) != NM_OK) return 0;
  return (size_t)O * (size_t)nm::values_per_row(K, N, M) * sizeof(nm_bf16);
}

size_t nm_index_bytes(int64_t O, int64_t K, int32_t N, int32_t M) {
  if (check_weight(O, K, N, M) != NM_OK) return 0;
  return (size_t)O * (size_t)nm::index_words_per_row(K, N, M) * sizeof(uint32_t);
}

size_t nm_mask_bytes(int64_t O, int64_t K) {
  if (O <= 0 || K <= 0) return 0;
  return (size_t)O * (size_t)nm::mask_words_per_row(K) * sizeof(uint32_t);
}

size_t nm_spmm_workspace_bytes(int64_t O, int64_t K, int32_t N, int32_t M, int64_t T) {
  if (check_weight(O, K, N, M) != NM_OK || T <= 0) return 0;
  return nm::spmm_workspace_bytes(O, K, N, M, T);
}

int32_t nm_prune(const nm_bf16* W, int64_t O, int64_t K, int64_t ldw, int32_t N, int32_t M, uint32_t* mask,
                 nm_bf16* W_masked, void* stream) {
  if (!W || !mask) return NM_ERR_NULL;
  if (int32_t s = check_weight(O, K, N, M)) return s;
  if (ldw < K) return NM_ERR_SHAPE;
  if (!aligned(W, 2) || !aligned(mask, 4) || !aligned(W_masked, 2)) return NM_ERR_ALIGN;
  return device_status(nm::launch_prune(W, O, K, ldw, N, M, mask, W_masked, (hipStream_t)stream));
}

int32_t nm_pack(const nm_bf16* W, int64_t O, int64_t K, int64_t ldw, int32_t N, int32_t M, const uint32_t* mask,
                nm_bf16* values, uint32_t* indices, void* stream) {
  if (!W || !values || !indices) return NM_ERR_NULL;
  if (int32_t s = check_weight(O, K, N, M)) return s;
  if (ldw < K) return NM_ERR_SHAPE;
  if (!aligned(W, 2) || !aligned(values, 2) || !aligned(indices, 4) || !aligned(mask, 4)) return NM_ERR_ALIGN;
  return device_status(nm::launch_pack(W, O, K, ldw, N, M, mask, values, indices, (hipStream_t)stream));
}

int32_t nm_pack_batched(const nm_pack_desc* descs, int32_t count, void* stream) {
  if (!descs) return NM_ERR_NULL;
  if (count <= 0) return NM_ERR_SHAPE;
  static_assert(sizeof(nm_pack_desc) == sizeof(nm::PackDesc), "descriptor layouts must match");
  for (int32_t i = 0; i < count; ++i) {
    const nm_pack_desc& d = descs[i];
    if (!d.W || !d.values || !d.indices) return NM_ERR_NULL;
    if (int32_t s = check_weight(d.O, d.K, d.N, d.M)) return s;
    if (!aligned(d.W, 2) || !aligned(d.values, 2) || !aligned(d.indices, 4)) return NM_ERR_ALIGN;
  }
  return device_status(nm::launch_pack_batched(reinterpret_cast<const nm::PackDesc*>(descs), count, (hipStream_t)stream));
}

int32_t nm_pack_prepare_batched(const nm_layer_desc* descs, int32_t count, void* stream) {
  if (!descs) return NM_ERR_NULL;
  if (count <= 0) return NM_ERR_SHAPE;
  static_assert(sizeof(nm_layer_desc) == sizeof(nm::LayerDesc), "descriptor layouts must match");
  for (int32_t i = 0; i < count; ++i) {
    const nm_layer_desc& d = descs[i];
    if (!d.W || !d.values || !d.indices) return NM_ERR_NULL;
    if (int32_t s = check_weight(d.O, d.K, d.N, d.M)) return s;
    if (d.T <= 0 || d.T > (int64_t)1 << 31) return NM_ERR_SHAPE;
    if (!aligned(d.W, 2) || !aligned(d.values, 2) || !aligned(d.indices, 4)) return NM_ERR_ALIGN;
  }
  bool workspace_short = false;
  hipError_t e = nm::launch_pack_prepare_batched(reinterpret_cast<const nm::LayerDesc*>(descs), count,
                                                 (hipStream_t)stream, &workspace_short);
  if (workspace_short) return NM_ERR_WORKSPACE;
  return device_status(e);
}

int32_t nm_unpack(const nm_bf16* values, const uint32_t* indices, int64_t O, int64_t K, int32_t N, int32_t M,
                  nm_bf16* W_dense, int64_t ldw, void* stream) {
  if (!values || !indices || !W_dense) return NM_ERR_NULL;
  if (int32_t s = check_weight(O, K, N, M)) return s;
  if (ldw < K) return NM_ERR_SHAPE;
  if (!aligned(values, 2) || !aligned(indices, 4) || !aligned(W_dense, 2)) return NM_ERR_ALIGN;
  return device_status(nm::launch_unpack(values, indices, O, K, N, M, W_dense, ldw, (hipStream_t)stream));
}

size_t nm_rank_bytes(int64_t O, int64_t K) {
  if (O <= 0 || K <= 0 || (K % 4) != 0) return 0;
  return (size_t)O * (size_t)K / 2;
}

int32_t nm_rank(const nm_bf16* W, int64_t O, int64_t K, int64_t ldw, int32_t M, uint8_t* rank, void* stream) {
  if (!W || !rank) return NM_ERR_NULL;
  if (int32_t s = check_weight(O, K, M, M)) return s;
  if (ldw < K) return NM_ERR_SHAPE;
  if (!aligned(W, 2)) return NM_ERR_ALIGN;
  return device_status(nm::launch_rank(W, O, K, ldw, M, rank, (hipStream_t)stream));
}

int32_t nm_rank_batched(const nm_rank_desc* descs, int32_t count, void* stream) {
  if (!descs) return NM_ERR_NULL;
  if (count <= 0) return NM_ERR_SHAPE;
  static_assert(sizeof(nm_rank_desc) == sizeof(nm::RankDesc), "descriptor layouts must match");
  for (int32_t i = 0; i < count; ++i) {
    const nm_rank_desc& d = descs[i];
    if (!d.W || !d.rank) return NM_ERR_NULL;
    if (int32_t s = check_weight(d.O, d.K, d.M, d.M)) return s;
    if (!aligned(d.W, 2)) return NM_ERR_ALIGN;
  }
  return device_status(nm::launch_rank_batched(reinterpret_cast<const nm::RankDesc*>(descs), count, (hipStream_t)stream));
}

int32_t nm_rank_mask(const uint8_t* rank, int64_t O, int64_t K, int32_t N, int32_t M, uint32_t* mask, void* stream) {
  if (!rank || !mask) return NM_ERR_NULL;
  if (int32_t s = check_weight(O, K, N, M)) return s;
  if (!aligned(mask, 4)) return NM_ERR_ALIGN;
  return device_status(nm::launch_rank_mask(rank, O, K, N, mask, (hipStream_t)stream));
}

int32_t nm_pack_ranked(const nm_bf16* W, const uint8_t* rank, int64_t O, int64_t K, int64_t ldw, int32_t N, int32_t M,
                       nm_bf16* values, uint32_t* indices, void* stream) {
  if (!W || !rank || !values || !indices) return NM_ERR_NULL;
  if (int32_t s = check_weight(O, K, N, M)) return s;
  if (ldw < K) return NM_ERR_SHAPE;
  if (!aligned(W, 2) || !aligned(values, 2) || !aligned(indices, 4)) return NM_ERR_ALIGN;
  return device_status(nm::launch_pack_ranked(W, rank, O, K, ldw, N, M, values, indices, (hipStream_t)stream));
}

int32_t nm_pack_ranked_batched(const nm_pack_ranked_desc* descs, int32_t count, void* stream) {
  if (!descs) return NM_ERR_NULL;
  if (count <= 0) return NM_ERR_SHAPE;
  static_assert(sizeof(nm_pack_ranked_desc) == sizeof(nm::PackRankedDesc), "descriptor layouts must match");
  for (int32_t i = 0; i < count; ++i) {
    const nm_pack_ranked_desc& d = descs[i];
    if (!d.W || !d.rank || !d.values || !d.indices) return NM_ERR_NULL;
    if (int32_t s = check_weight(d.O, d.K, d.N, d.M)) return s;
    if (!aligned(d.W, 2) || !aligned(d.values, 2) || !aligned(d.indices, 4)) return NM_ERR_ALIGN;
  }
  return device_status(nm::launch_pack_ranked_batched(reinterpret_cast<const nm::PackRankedDesc*>(descs), count,
                                                      (hipStream_t)stream));
}

int32_t nm_mask_check(const uint32_t* mask, int64_t O, int64_t K, int32_t N, int32_t M, uint32_t* bad_groups,
                      void* stream) {
  if (!mask || !bad_groups) return NM_ERR_NULL;
  if (int32_t s = check_weight(O, K, N, M)) return s;
  if (!aligned(mask, 4) || !aligned(bad_groups, 4)) return NM_ERR_ALIGN;
  return device_status(nm::launch_mask_check(mask, O, K, N, M, bad_groups, (hipStream_t)stream));
}

}  // extern "C"

namespace {

// validation shared by the product calls; fills the launch arguments
int32_t spmm_check(const nm_bf16* values, const uint32_t* indices, int64_t O, int64_t K, int32_t N, int32_t M,
                   const nm_bf16* X, int64_t T, int64_t ldx, const float* bias, void* Y, int64_t ldy, int32_t out_dtype,
                   void* workspace, size_t workspace_bytes, bool product, nm::SpmmArgs* a) {
  if (!values || !indices || (product && (!X || !Y))) return NM_ERR_NULL;
  if (int32_t s = check_weight(O, K, N, M)) return s;
  if (T <= 0 || T > (int64_t)1 << 31) return NM_ERR_SHAPE;
  if (product && (ldx < K || ldy < O)) return NM_ERR_SHAPE;
  if (out_dtype != NM_OUT_F32 && out_dtype != NM_OUT_BF16) return NM_ERR_DTYPE;
  if (!aligned(values, 2) || !aligned(indices, 4) || !aligned(X, 2) || !aligned(bias, 4) ||
      !aligned(Y, out_dtype == NM_OUT_F32 ? 4 : 2))
    return NM_ERR_ALIGN;
  a->values = values; a->indices = indices; a->O = O; a->K = K; a->N = N; a->M = M;
  a->X = X; a->T = T; a->ldx = product ? ldx : K; a->bias = bias; a->Y = Y; a->ldy = ldy;
  a->out_bf16 = (out_dtype == NM_OUT_BF16);
  a->workspace = workspace; a->workspace_bytes = workspace_bytes;
  return NM_OK;
}

int32_t spmm_entry(const nm_bf16* values, const uint32_t* indices, int64_t O, int64_t K, int32_t N, int32_t M,
                   const nm_bf16* X, int64_t T, int64_t ldx, const float* bias, void* Y, int64_t ldy, int32_t out_dtype,
                   void* workspace, size_t workspace_bytes, void* stream, int phases) {
  nm::SpmmArgs a;
  if (int32_t st = spmm_check(values, indices, O, K, N, M, X, T, ldx, bias, Y, ldy, out_dtype, workspace, workspace_bytes,
                              phases & nm::SPMM_PRODUCT, &a))
    return st;
  bool workspace_short = false;
  hipError_t e = nm::launch_spmm(a, (hipStream_t)stream, &workspace_short, phases);
  if (workspace_short) return NM_ERR_WORKSPACE;
  return device_status(e);
}

// the int8 layer from the dense weight + mask (values == NULL) or from the compressed form (Wq == NULL)
int32_t i8_entry(const int8_t* Wq, int64_t O, int64_t K, int64_t ldw, const uint32_t* mask, const int8_t* values,
                 const uint32_t* indices, int32_t N, int32_t M, const int8_t* Xq, int64_t T, int64_t ldx, float x_scale,
                 const float* w_scale, const float* bias, void* Y, int64_t ldy, int32_t out_dtype, void* workspace,
                 size_t workspace_bytes, void* stream, int phases) {
  const bool product = phases & nm::SPMM_PRODUCT;
  const bool packed = values != nullptr || indices != nullptr;
  if (packed ? (!values || !indices) : (!Wq || !mask)) return NM_ERR_NULL;
  if (product && (!Xq || !Y)) return NM_ERR_NULL;
  if (int32_t s = check_weight(O, K, N, M)) return s;
  if (T <= 0 || T > (int64_t)1 << 31 || (!packed && ldw < K)) return NM_ERR_SHAPE;
  if (product && (ldx < K || ldy < O)) return NM_ERR_SHAPE;
  if (out_dtype != NM_OUT_F32 && out_dtype != NM_OUT_BF16 && out_dtype != NM_OUT_I32) return NM_ERR_DTYPE;
  if (!aligned(mask, 4) || !aligned(indices, 4) || !aligned(w_scale, 4) || !aligned(bias, 4) ||
      !aligned(Y, out_dtype == NM_OUT_BF16 ? 2 : 4))
    return NM_ERR_ALIGN;
  nm::I8LinearArgs a;
  a.Wq = packed ? nullptr : Wq; a.ldw = ldw; a.mask = mask; a.values = values; a.indices = indices;
  a.O = O; a.K = K; a.N = N; a.M = M;
  a.X = Xq; a.T = T; a.ldx = ldx; a.x_scale = x_scale; a.w_scale = w_scale; a.bias = bias;
  a.Y = Y; a.ldy = ldy; a.out_kind = out_dtype;
  a.workspace = workspace; a.workspace_bytes = workspace_bytes;
  bool workspace_short = false;
  hipError_t e = nm::launch_linear_i8(a, (hipStream_t)stream, &workspace_short, phases);
  if (workspace_short) return NM_ERR_WORKSPACE;
  return device_status(e);
}

}  // namespace

extern "C" {

int32_t nm_linear_forward(const nm_bf16* values, const uint32_t* indices, int64_t O, int64_t K, int32_t N, int32_t M,
                          const nm_bf16* X, int64_t T, int64_t ldx, const float* bias, void* Y, int64_t ldy,
                          int32_t out_dtype, void* workspace, size_t workspace_bytes, void* stream) {
  return spmm_entry(values, indices, O, K, N, M, X, T, ldx, bias, Y, ldy, out_dtype, workspace, workspace_bytes, stream,
                    nm::SPMM_PREPARE | nm::SPMM_PRODUCT);
}

int32_t nm_spmm(const nm_bf16* values, const uint32_t* indices, int64_t O, int64_t K, int32_t N, int32_t M,
                const nm_bf16* X, int64_t T, int64_t ldx, void* Y, int64_t ldy, int32_t out_dtype, void* workspace,
                size_t workspace_bytes, void* stream) {
  return spmm_entry(values, indices, O, K, N, M, X, T, ldx, nullptr, Y, ldy, out_dtype, workspace, workspace_bytes,
                    stream, nm::SPMM_PREPARE | nm::SPMM_PRODUCT);
}

int32_t nm_spmm_prepare(const nm_bf16* values, const uint32_t* indices, int64_t O, int64_t K, int32_t N, int32_t M,
                        int64_t T, void* workspace, size_t workspace_bytes, void* stream) {
  return spmm_entry(values, indices, O, K, N, M, nullptr, T, K, nullptr, nullptr, O, NM_OUT_F32, workspace,
                    workspace_bytes, stream, nm::SPMM_PREPARE);
}

int32_t nm_linear_forward_prepared(const nm_bf16* values, const uint32_t* indices, int64_t O, int64_t K, int32_t N,
                                   int32_t M, const nm_bf16* X, int64_t T, int64_t ldx, const float* bias, void* Y,
                                   int64_t ldy, int32_t out_dtype, const void* workspace, size_t workspace_bytes,
                                   void* stream) {
  return spmm_entry(values, indices, O, K, N, M, X, T, ldx, bias, Y, ldy, out_dtype, const_cast<void*>(workspace),
                    workspace_bytes, stream, nm::SPMM_PRODUCT);
}

size_t nm_static_scratch_bytes(void) { return kStaticScratchBytes; }

int32_t nm_linear_forward_static(const nm_bf16* values, const uint32_t* indices, int64_t O, int64_t K, int32_t N,
                                 int32_t M, const nm_bf16* X, int64_t T, int64_t ldx, const float* bias, void* Y,
                                 int64_t ldy, int32_t out_dtype, void* stream) {
  nm::SpmmArgs a;
  if (int32_t st = spmm_check(values, indices, O, K, N, M, X, T, ldx, bias, Y, ldy, out_dtype, nullptr, 0, true, &a))
    return st;
  if (nm::spmm_operand_workspace_bytes(O, K, N, M, T) > kStaticScratchBytes) return NM_ERR_WORKSPACE;
  unsigned char* ws = nullptr;
  if (int32_t st = device_status(static_scratch(&ws))) return st;
  a.workspace = ws;
  a.workspace_bytes = kStaticScratchBytes;
  bool workspace_short = false;
  hipError_t e = nm::launch_spmm(a, (hipStream_t)stream, &workspace_short, nm::SPMM_PREPARE | nm::SPMM_PRODUCT);
  if (workspace_short) return NM_ERR_WORKSPACE;
  return device_status(e);
}

size_t nm_backward_weight_workspace_bytes(int64_t O, int64_t K, int64_t T) {
  if (O <= 0 || K <= 0 || T <= 0) return 0;
  return nm::backward_weight_workspace_bytes(O, K, T);
}

size_t nm_backward_input_workspace_bytes(int64_t O, int64_t K, int64_t T) {
  if (O <= 0 || K <= 0 || T <= 0) return 0;
  return nm::backward_input_workspace_bytes(O, K, T);
}

int32_t nm_linear_backward_input(const nm_bf16* Ws, int64_t O, int64_t K, int64_t ldw, const nm_bf16* dY, int64_t T,
                                 int64_t ldy, void* dX, int64_t ldx, int32_t out_dtype, void* workspace,
                                 size_t workspace_bytes, void* stream) {
  if (!Ws || !dY || !dX) return NM_ERR_NULL;
  if (O <= 0 || K <= 0 || T <= 0 || O > (int64_t)1 << 31 || K > (int64_t)1 << 31 || T > (int64_t)1 << 31)
    return NM_ERR_SHAPE;
  if (ldw < K || ldy < O || ldx < K) return NM_ERR_SHAPE;
  if (out_dtype != NM_OUT_F32 && out_dtype != NM_OUT_BF16) return NM_ERR_DTYPE;
  if (!aligned(Ws, 2) || !aligned(dY, 2) || !aligned(dX, out_dtype == NM_OUT_F32 ? 4 : 2)) return NM_ERR_ALIGN;
  bool workspace_short = false;
  hipError_t e = nm::launch_backward_input(Ws, O, K, ldw, dY, T, ldy, dX, ldx, out_dtype == NM_OUT_BF16, workspace,
                                           workspace_bytes, (hipStream_t)stream, &workspace_short);
  if (workspace_short) return NM_ERR_WORKSPACE;
  return device_status(e);
}

int32_t nm_linear_backward_weight(const nm_bf16* dY, int64_t T, int64_t O, int64_t ldy, const nm_bf16* X, int64_t K,
                                  int64_t ldx, const uint32_t* mask, void* dW, int64_t lddw, int32_t out_dtype,
                                  void* workspace, size_t workspace_bytes, void* stream) {
  if (!dY || !X || !dW) return NM_ERR_NULL;
  if (O <= 0 || K <= 0 || T <= 0 || O > (int64_t)1 << 31 || K > (int64_t)1 << 31 || T > (int64_t)1 << 31)
    return NM_ERR_SHAPE;
  if (ldy < O || ldx < K || lddw < K) return NM_ERR_SHAPE;
  if (out_dtype != NM_OUT_F32 && out_dtype != NM_OUT_BF16) return NM_ERR_DTYPE;
  if (!aligned(dY, 2) || !aligned(X, 2) || !aligned(mask, 4) || !aligned(dW, out_dtype == NM_OUT_F32 ? 4 : 2))
    return NM_ERR_ALIGN;
  bool workspace_short = false;
  hipError_t e = nm::launch_backward_weight(dY, T, O, ldy, X, K, ldx, mask, dW, lddw, out_dtype == NM_OUT_BF16, workspace,
                                            workspace_bytes, (hipStream_t)stream, &workspace_short);
  if (workspace_short) return NM_ERR_WORKSPACE;
  return device_status(e);
}

size_t nm_i8_workspace_bytes(int64_t O, int64_t K, int32_t N, int32_t M, int64_t T) {
  if (check_weight(O, K, N, M) != NM_OK || T <= 0) return 0;
  return nm::i8_workspace_bytes(O, K, N, M, T);
}

int32_t nm_linear_forward_i8(const int8_t* Wq, int64_t O, int64_t K, int64_t ldw, const uint32_t* mask, int32_t N,
                             int32_t M, const int8_t* Xq, int64_t T, int64_t ldx, float x_scale, const float* w_scale,
                             const float* bias, void* Y, int64_t ldy, int32_t out_dtype, void* workspace,
                             size_t workspace_bytes, void* stream) {
  return i8_entry(Wq, O, K, ldw, mask, nullptr, nullptr, N, M, Xq, T, ldx, x_scale, w_scale, bias, Y, ldy, out_dtype, workspace,
                  workspace_bytes, stream, nm::SPMM_PREPARE | nm::SPMM_PRODUCT);
}

int32_t nm_i8_prepare(const int8_t* Wq, int64_t O, int64_t K, int64_t ldw, const uint32_t* mask, int32_t N, int32_t M,
                      int64_t T, void* workspace, size_t workspace_bytes, void* stream) {
  return i8_entry(Wq, O, K, ldw, mask, nullptr, nullptr, N, M, nullptr, T, K, 1.f, nullptr, nullptr, nullptr, O, NM_OUT_F32,
                  workspace, workspace_bytes, stream, nm::SPMM_PREPARE);
}

int32_t nm_linear_forward_i8_prepared(const int8_t* Wq, int64_t O, int64_t K, int64_t ldw, const uint32_t* mask,
                                      int32_t N, int32_t M, const int8_t* Xq, int64_t T, int64_t ldx, float x_scale,
                                      const float* w_scale, const float* bias, void* Y, int64_t ldy, int32_t out_dtype,
                                      void* workspace, size_t workspace_bytes, void* stream) {
  return i8_entry(Wq, O, K, ldw, mask, nullptr, nullptr, N, M, Xq, T, ldx, x_scale, w_scale, bias, Y, ldy, out_dtype, workspace,
                  workspace_bytes, stream, nm::SPMM_PRODUCT);
}

size_t nm_values_i8_bytes(int64_t O, int64_t K, int32_t N, int32_t M) {
  if (check_weight(O, K, N, M) != NM_OK) return 0;
  return (size_t)O * (size_t)nm::values_per_row(K, N, M);
}

int32_t nm_pack_i8(const int8_t* Wq, int64_t O, int64_t K, int64_t ldw, int32_t N, int32_t M, const uint32_t* mask,
                   int8_t* values, uint32_t* indices, void* stream) {
  if (!Wq || !mask || !values || !indices) return NM_ERR_NULL;
  if (int32_t s = check_weight(O, K, N, M)) return s;
  if (ldw < K) return NM_ERR_SHAPE;
  if (!aligned(mask, 4) || !aligned(indices, 4)) return NM_ERR_ALIGN;
  return device_status(nm::launch_pack_i8(Wq, O, K, ldw, N, M, mask, values, indices, (hipStream_t)stream));
}

int32_t nm_unpack_i8(const int8_t* values, const uint32_t* indices, int64_t O, int64_t K, int32_t N, int32_t M,
                     int8_t* Wq_dense, int64_t ldw, void* stream) {
  if (!values || !indices || !Wq_dense) return NM_ERR_NULL;
  if (int32_t s = check_weight(O, K, N, M)) return s;
  if (ldw < K) return NM_ERR_SHAPE;
  if (!aligned(indices, 4)) return NM_ERR_ALIGN;
  return device_status(nm::launch_unpack_i8(values, indices, O, K, N, M, Wq_dense, ldw, (hipStream_t)stream));
}

int32_t nm_linear_forward_i8_packed(const int8_t* values, const uint32_t* indices, int64_t O, int64_t K, int32_t N,
                                    int32_t M, const int8_t* Xq, int64_t T, int64_t ldx, float x_scale,
                                    const float* w_scale, const float* bias, void* Y, int64_t ldy, int32_t out_dtype,
                                    void* workspace, size_t workspace_bytes, void* stream) {
  if (!values || !indices) return NM_ERR_NULL;
  return i8_entry(nullptr, O, K, K, nullptr, values, indices, N, M, Xq, T, ldx, x_scale, w_scale, bias, Y, ldy, out_dtype,
                  workspace, workspace_bytes, stream, nm::SPMM_PREPARE | nm::SPMM_PRODUCT);
}

int32_t nm_i8_prepare_packed(const int8_t* values, const uint32_t* indices, int64_t O, int64_t K, int32_t N, int32_t M,
                             int64_t T, void* workspace, size_t workspace_bytes, void* stream) {
  if (!values || !indices) return NM_ERR_NULL;
  return i8_entry(nullptr, O, K, K, nullptr, values, indices, N, M, nullptr, T, K, 1.f, nullptr, nullptr, nullptr, O,
                  NM_OUT_F32, workspace, workspace_bytes, stream, nm::SPMM_PREPARE);
}

int32_t nm_linear_forward_i8_packed_prepared(const int8_t* values, const uint32_t* indices, int64_t O, int64_t K,
                                             int32_t N, int32_t M, const int8_t* Xq, int64_t T, int64_t ldx,
                                             float x_scale, const float* w_scale, const float* bias, void* Y,
                                             int64_t ldy, int32_t out_dtype, void* workspace, size_t workspace_bytes,
                                             void* stream) {
  if (!values || !indices) return NM_ERR_NULL;
  return i8_entry(nullptr, O, K, K, nullptr, values, indices, N, M, Xq, T, ldx, x_scale, w_scale, bias, Y, ldy, out_dtype,
                  workspace, workspace_bytes, stream, nm::SPMM_PRODUCT);
}

int32_t nm_prune_scored(const float* score, int64_t O, int64_t K, int64_t lds, int32_t N, int32_t M, uint32_t* mask,
                        void* stream) {
  if (!score || !mask) return NM_ERR_NULL;
  if (int32_t s = check_weight(O, K, N, M)) return s;
  if (lds < K) return NM_ERR_SHAPE;
  if (!aligned(score, 4) || !aligned(mask, 4)) return NM_ERR_ALIGN;
  return device_status(nm::launch_score_mask(score, O, K, lds, N, M, mask, (hipStream_t)stream));
}

size_t nm_probe_sink_bytes(void) { return nm::probe_sink_bytes(); }

int32_t nm_probe_matrix_rate(int32_t kind, int32_t iters, void* sink, int64_t* ops, void* stream) {
  if (!sink || !ops) return NM_ERR_NULL;
  if (kind != 0 && kind != 1) return NM_ERR_DTYPE;
  if (iters <= 0) return NM_ERR_SHAPE;
  if (!aligned(sink, 4)) return NM_ERR_ALIGN;
  return device_status(nm::launch_probe_matrix(kind, iters, static_cast<float*>(sink), ops, (hipStream_t)stream));
}

int32_t nm_probe_copy(const void* src, void* dst, size_t bytes, void* stream) {
  if (!src || !dst) return NM_ERR_NULL;
  if (bytes == 0 || (bytes % 16) != 0) return NM_ERR_SHAPE;
  if (!aligned(src, 16) || !aligned(dst, 16)) return NM_ERR_ALIGN;
  return device_status(nm::launch_probe_copy(src, dst, bytes, (hipStream_t)stream));
}

int32_t nm_linear_forward_prepared_batched(const nm_forward_desc* descs, int32_t count, void* stream) {
  if (!descs) return NM_ERR_NULL;
  if (count <= 0) return NM_ERR_SHAPE;
  constexpr int kChunk = 64;  // descriptors converted at a time (no allocation)
  nm::SpmmArgs layers[kChunk];
  auto convert = [&](int32_t i, nm::SpmmArgs* a) {
    const nm_forward_desc& d = descs[i];
    return spmm_check(d.values, d.indices, d.O, d.K, d.N, d.M, d.X, d.T, d.ldx, d.bias, d.Y, d.ldy, d.out_dtype,
                      d.workspace, d.workspace_bytes, true, a);
  };
  for (int32_t i = 0; i < count; ++i) {  // every argument error is reported before anything is launched
    if (int32_t st = convert(i, &layers[0])) return st;
    if (nm::spmm_workspace_short(layers[0])) return NM_ERR_WORKSPACE;
  }
  for (int32_t first = 0; first < count; first += kChunk) {
    const int n = count - first < kChunk ? count - first : kChunk;
    for (int i = 0; i < n; ++i) convert(first + i, &layers[i]);
    if (int32_t st = device_status(nm::launch_spmm_batched(layers, n, (hipStream_t)stream))) return st;
  }
  return NM_OK;
}

}  // extern "C"
