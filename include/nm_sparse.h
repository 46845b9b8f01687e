/*
 * nm_sparse.h -- C ABI of the N:M-sparse linear layer for AMD MI355X (gfx950).
 *
 * The library implements the deployment primitive that layer-wise N:M sparsity for
 * vision transformers assumes (Section 3, "Problem Formulation": an accelerator that
 * supports several N:M levels, one level chosen per linear layer):
 *
 *   prune  -- Section 3.1, "Dynamic Masking", Eq. (1): in every group of M consecutive
 *             weights keep the N of largest saliency; saliency = weight magnitude.
 *   pack   -- Section 1 and Section 2 (Fig. 2, upper part): store the kept values and,
 *             for each, a log2(M)-bit index of its position inside its group.
 *   spmm   -- Section 2 (Fig. 2, lower part): decode the indices, select the matching
 *             activations, multiply-accumulate; the result is the exact product with
 *             the masked weight, with N/M of the dense multiply-accumulates.
 *
 * Conventions
 *   W  [O, K]  weight, row-major, leading dimension ldw (elements); O = out features,
 *              K = in features = reduction dimension.  Groups of M are aligned
 *              (k in [g*M, g*M+M)) and run along K.
 *   X  [T, K]  activations, row-major, leading dimension ldx.  T = tokens.
 *   Y  [T, O]  Y = X * (W (.) mask)^T (+ bias), row-major, leading dimension ldy.
 *   All weights and activations are bfloat16 carried as raw 16-bit patterns (nm_bf16);
 *   products are accumulated in fp32.
 *   Legal levels: M in {4, 8, 16}, 1 <= N <= M.  K must be a multiple of M.
 *
 * Selection rule (exactly N kept per group): order the members of a group by
 * (magnitude descending, position ascending) and keep the first N.  Magnitude is compared
 * on the stored bfloat16 value: key = bit pattern & 0x7FFF (so -0 ties +0, Inf beats every
 * finite value and NaN patterns carry the largest keys).
 *
 * Packed layout (the only layout that crosses this boundary)
 *   values   nm_bf16 [O, K*N/M], row-major, no padding: values[o, g*N + j] is the j-th
 *            kept weight of group g of row o, kept weights in ascending position.
 *   indices  uint32  [O, ceil(K*N/M*b/32)], b = log2(M): per row an LSB-first bit stream;
 *            field f = g*N + j occupies bits [f*b, f*b+b) of the row and holds the
 *            position (0..M-1) of values[o, f] inside its group; the row is padded with
 *            zero bits to a 32-bit boundary.  3-bit fields (M = 8) may straddle words.
 *   mask     uint32  [O, ceil(K/32)]: bit (k mod 32) of word floor(k/32) of row o is
 *            the mask value of W[o, k]; padding bits are zero.
 *
 * Ownership and execution
 *   Every data pointer is a DEVICE pointer owned by the caller unless it is marked
 *   "host".  The library allocates no device memory.  Its only state: the last HIP
 *   error code of the calling thread, and per device (a process may use several, the
 *   current one at call time is used) a few marks of one-time setup: the dynamic-LDS limit
 *   raised per kernel, the compute-unit count, the address of the static scratch.  No
 *   environment variable is read.  `stream` is a hipStream_t passed as void* (NULL = the null
 *   stream).  Calls validate their arguments on the host, enqueue their kernels on
 *   `stream` and return without synchronising.  Argument errors are reported before
 *   anything is launched, so they can be exercised without a GPU.  A call enqueues
 *   kernels only (no copies, fills or allocations), so it may be issued on a stream that
 *   is being captured into a graph; host descriptor arrays are read before it returns.
 *   The first launch of a kernel in a process also raises that kernel's dynamic-LDS limit
 *   (hipFuncSetAttribute): issue a call once eagerly before recording it.
 *   No function throws, aborts or prints.
 */
#ifndef NM_SPARSE_H
#define NM_SPARSE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef uint16_t nm_bf16; /* bfloat16 bit pattern */

/* Status codes (return value of every int32_t function). */
enum {
  NM_OK = 0,
  NM_ERR_NULL = 1,      /* a required pointer is NULL */
  NM_ERR_SHAPE = 2,     /* O, K or T <= 0; K % M != 0; a leading dimension smaller than the row; count <= 0;
                           O, K or T above 2^31 or O * K above 2^40 */
  NM_ERR_LEVEL = 3,     /* M not in {4, 8, 16} or N outside [1, M] */
  NM_ERR_ALIGN = 4,     /* a pointer is not aligned as documented */
  NM_ERR_DTYPE = 5,     /* out_dtype is not one the call offers */
  NM_ERR_WORKSPACE = 6, /* workspace is NULL or smaller than nm_spmm_workspace_bytes() and the shape needs one */
  NM_ERR_DEVICE = 7,    /* a HIP call failed; see nm_last_hip_error() */
  NM_ERR_EXHAUSTED = 8  /* nm_sample_config ran out of random numbers before a configuration fell into the interval */
};

enum { NM_OUT_F32 = 0, NM_OUT_BF16 = 1, NM_OUT_I32 = 2 /* int8 calls only: the raw integer sums */ };

/* Text for a status code (static storage, never NULL). */
const char* nm_status_string(int32_t status);

/* hipError_t of the most recent failed HIP call made by this library on the calling thread
 * (0 if none). */
int32_t nm_last_hip_error(void);

/* Buffer sizes in bytes for the layouts above; 0 if the level or shape is illegal. */
size_t nm_values_bytes(int64_t O, int64_t K, int32_t N, int32_t M);
size_t nm_index_bytes(int64_t O, int64_t K, int32_t N, int32_t M);
size_t nm_mask_bytes(int64_t O, int64_t K);

/* Scratch needed by nm_spmm / nm_linear_forward for this layer and token count (bytes,
 * possibly 0).  The product kernels consume the weight in matrix-core operand order, which
 * depends on the kernel the token count selects; whenever the packed layout is not already
 * that order the call first rewrites the packed weight into the scratch (large layers: always).
 * 0 if the level or shape is illegal. */
size_t nm_spmm_workspace_bytes(int64_t O, int64_t K, int32_t N, int32_t M, int64_t T);

/*
 * nm_prune -- Eq. (1) with magnitude saliency (Section 3.1).
 *   W         in   [O, K], ld ldw, 2-byte aligned
 *   mask      out  [O, ceil(K/32)] words, 4-byte aligned; exactly N bits set per group
 *   W_masked  out  optional (NULL to skip): [O, K] with ld ldw; W where mask = 1, +0
 *                  elsewhere.  May be the same pointer as W (in-place pruning).
 */
int32_t nm_prune(const nm_bf16* W, int64_t O, int64_t K, int64_t ldw, int32_t N, int32_t M,
                 uint32_t* mask, nm_bf16* W_masked, void* stream);

/*
 * nm_pack -- compress W to the packed layout (Fig. 2, upper part).
 *   mask == NULL : select by magnitude as nm_prune does, fused with packing (the hot path).
 *   mask != NULL : use the caller's mask (any saliency, e.g. a Taylor score, Section 3.1).
 *                  Per group the N lowest set positions are kept; a group with fewer than N
 *                  set bits is completed with its lowest unset positions, stored with value
 *                  +0.  Use nm_mask_check to find out whether a mask has exactly N per group.
 *   values   out  nm_values_bytes(O,K,N,M) bytes, 2-byte aligned (16-byte alignment lets the
 *                  fast kernels run)
 *   indices  out  nm_index_bytes(O,K,N,M) bytes, 4-byte aligned; every word is written,
 *                  padding bits zero
 * nm_pack(W, mask = NULL) and nm_prune followed by nm_pack(W, mask) write identical bytes.
 */
int32_t nm_pack(const nm_bf16* W, int64_t O, int64_t K, int64_t ldw, int32_t N, int32_t M,
                const uint32_t* mask, nm_bf16* values, uint32_t* indices, void* stream);

/* One nm_pack(mask = NULL) per descriptor, in a single launch (a model's layers are
 * compressed together: Section 3, configuration alpha = (s^1 ... s^L)). */
typedef struct nm_pack_desc {
  const nm_bf16* W; /* device, [O, K] contiguous (ldw = K) */
  nm_bf16* values;  /* device, out */
  uint32_t* indices; /* device, out */
  int64_t O, K;
  int32_t N, M;
} nm_pack_desc;

/* descs is a HOST array of `count` descriptors; it is read before the call returns. */
int32_t nm_pack_batched(const nm_pack_desc* descs, int32_t count, void* stream);

/*
 * nm_unpack -- inverse of nm_pack: W_dense[o, g*M + idx] = value, +0 elsewhere.
 *   W_dense  out  [O, K] with ld ldw; every element of the O x K block is written.
 */
int32_t nm_unpack(const nm_bf16* values, const uint32_t* indices, int64_t O, int64_t K,
                  int32_t N, int32_t M, nm_bf16* W_dense, int64_t ldw, void* stream);

/*
 * nm_mask_check -- counts the groups of `mask` whose population count differs from N.
 *   bad_groups  out  one uint32 on the device; overwritten with the count (saturating).
 */
int32_t nm_mask_check(const uint32_t* mask, int64_t O, int64_t K, int32_t N, int32_t M,
                      uint32_t* bad_groups, void* stream);

/*
 * Nested levels from one stored rank per weight -- Section 3, "Subset-Superset Relationship": under one
 * pruning criterion the weights kept at a sparser level are among those kept at a denser level of the same
 * M.  The rank of a weight inside its group, in the order of the selection rule above (magnitude
 * descending, position ascending; 0 = kept first), therefore holds every level at once: the mask of N:M is
 * rank < N.  A supernet that derives a layer's sparse weight each time a level is sampled (Section 3.1,
 * "Dynamic Masking") ranks a weight once per update and takes any level from the ranks.
 *   rank layout  uint8 [O, K/2], row-major, no padding: weight k of row o in bits [4 (k mod 2), +4) of byte
 *                o*K/2 + k/2; nm_rank_bytes(O, K) bytes (0 if the shape is illegal).
 *   nm_rank         W [O, K] (ld ldw) -> ranks for groups of M.  A 16-byte aligned W with ldw = K and a
 *                   16-byte aligned rank buffer run the fast kernel; any other case a slower one.
 *   nm_rank_mask    mask words of level N:M (layout of nm_prune's mask): bit = rank < N.  For ranks written
 *                   by nm_rank(W, M) the words equal those of nm_prune(W, N, M).
 *   nm_pack_ranked  nm_pack with the selection read from the ranks; for ranks written by nm_rank(W, M) it
 *                   writes the bytes nm_pack(W, mask = NULL) writes.  Ranks that are not a permutation per
 *                   group are treated like a caller's mask with the wrong count (see nm_pack).
 */
size_t nm_rank_bytes(int64_t O, int64_t K);
int32_t nm_rank(const nm_bf16* W, int64_t O, int64_t K, int64_t ldw, int32_t M, uint8_t* rank, void* stream);
/* One nm_rank per descriptor (W contiguous, ldw = K), in a single launch where the shapes allow: a supernet
 * ranks all its layers after a weight update.  descs is a HOST array, read before the call returns. */
typedef struct nm_rank_desc {
  const nm_bf16* W; /* device, [O, K] contiguous */
  uint8_t* rank;    /* device, out */
  int64_t O, K;
  int32_t M, reserved;
} nm_rank_desc;
int32_t nm_rank_batched(const nm_rank_desc* descs, int32_t count, void* stream);
int32_t nm_rank_mask(const uint8_t* rank, int64_t O, int64_t K, int32_t N, int32_t M, uint32_t* mask,
                     void* stream);
int32_t nm_pack_ranked(const nm_bf16* W, const uint8_t* rank, int64_t O, int64_t K, int64_t ldw, int32_t N,
                       int32_t M, nm_bf16* values, uint32_t* indices, void* stream);
/* One nm_pack_ranked per descriptor (W contiguous, ldw = K), in a single launch where the shapes and levels
 * allow: after the ranks of a supernet's layers are written, a sampled configuration (one level per layer,
 * Section 3.1) is packed from them in one go.  descs is a HOST array, read before the call returns. */
typedef struct nm_pack_ranked_desc {
  const nm_bf16* W;    /* device, [O, K] contiguous */
  const uint8_t* rank; /* device, nm_rank_bytes(O, K) bytes written by nm_rank(W, M) */
  nm_bf16* values;     /* device, out */
  uint32_t* indices;   /* device, out */
  int64_t O, K;
  int32_t N, M;
} nm_pack_ranked_desc;
int32_t nm_pack_ranked_batched(const nm_pack_ranked_desc* descs, int32_t count, void* stream);

/*
 * nm_spmm -- Y = X * W_s^T from the packed weight (Fig. 2, lower part):
 *   Y[t, o] = sum_g sum_{j<N} X[t, g*M + idx[o,g,j]] * val[o,g,j], fp32 accumulation.
 *   values, indices  in   packed layout of an [O, K] weight at level N:M
 *   X                in   [T, K], ld ldx
 *   Y                out  [T, O], ld ldy (elements of the output type); float if
 *                         out_dtype = NM_OUT_F32, bfloat16 (round to nearest even) if
 *                         NM_OUT_BF16
 *   workspace        scratch of at least nm_spmm_workspace_bytes(O,K,N,M,T) bytes, 256-byte
 *                    aligned; may be NULL when that size is 0.  Its contents are undefined
 *                    after the call; concurrent calls need distinct workspaces.
 *                    A layer with few output tiles and a long reduction (one image through a wide layer: T = 197,
 *                    K = 3072) is cut into 2 .. 8 ranges along K; their fp32 partial sums live behind the
 *                    operand-order copy in the workspace (nm_spmm_workspace_bytes counts them) and a second launch
 *                    adds them in range order.  A workspace that holds the operand-order copy only gives the uncut
 *                    product (same result up to rounding order).
 *                    Without a workspace (NULL, or too small), a product of T <= 208 tokens at a level of
 *                    {1:4, 1:8, 2:8, 4:8, 1:16, 2:16, 4:16} with K % 64 == 0 and O % 4 == 0 still runs: a
 *                    kernel reads the packed format itself (Fig. 2: values + positions, decoded on the fly;
 *                    slower than the workspace path, nothing to prepare).  Every other shape reports
 *                    NM_ERR_WORKSPACE.
 * The matrix-core kernels need K % 64 == 0, 16-byte aligned X, values and Y and ldx, ldy
 * multiples of 8; other shapes run a slower general kernel with the same results.  Rows of X and Y
 * that start on 128-byte boundaries (ldx, ldy multiples of 64) are fastest.
 */
int32_t nm_spmm(const nm_bf16* values, const uint32_t* indices, int64_t O, int64_t K,
                int32_t N, int32_t M, const nm_bf16* X, int64_t T, int64_t ldx,
                void* Y, int64_t ldy, int32_t out_dtype,
                void* workspace, size_t workspace_bytes, void* stream);

/*
 * nm_linear_forward -- one sparse linear layer at its own level (Section 3.1: the level
 * chosen for a layer is applied when that layer is computed): nm_spmm plus an optional
 * fp32 bias[O] (NULL = none) added to the fp32 accumulator before the output is rounded.
 */
int32_t nm_linear_forward(const nm_bf16* values, const uint32_t* indices, int64_t O, int64_t K,
                          int32_t N, int32_t M, const nm_bf16* X, int64_t T, int64_t ldx,
                          const float* bias, void* Y, int64_t ldy, int32_t out_dtype,
                          void* workspace, size_t workspace_bytes, void* stream);

/*
 * nm_linear_forward_static -- nm_linear_forward for callers that cannot allocate device memory and so cannot
 * bring a workspace: code under HIP graph capture, tight serving loops, harnesses that forbid allocation.  The
 * scratch is a fixed array of nm_static_scratch_bytes() bytes (8 MiB) inside the library's device image; every
 * device the library runs on holds its own copy until the process ends.  The call allocates and frees nothing.
 *   Arguments and results as nm_linear_forward (same kernels, same bytes written to Y).
 *   NM_ERR_WORKSPACE  the layer's operand-order copy needs more scratch than the array holds; nothing is launched.
 *                     (A layer whose cut reduction, see nm_spmm, does not fit beside that copy, i.e.
 *                     nm_spmm_workspace_bytes(O, K, N, M, T) > nm_static_scratch_bytes(), is multiplied uncut: the
 *                     result of nm_linear_forward up to rounding order.)
 * All calls on one device share that device's array: two such calls whose kernels may overlap (different streams,
 * or threads) race on it; calls on one stream are ordered and safe.  The array keeps the last call's contents;
 * every call rewrites the part it reads, so nothing needs clearing.
 */
size_t nm_static_scratch_bytes(void);
int32_t nm_linear_forward_static(const nm_bf16* values, const uint32_t* indices, int64_t O, int64_t K,
                                 int32_t N, int32_t M, const nm_bf16* X, int64_t T, int64_t ldx,
                                 const float* bias, void* Y, int64_t ldy, int32_t out_dtype, void* stream);

/*
 * The two halves of nm_linear_forward, for callers whose weights stay fixed across many calls (a
 * deployed layer keeps its level and weights: Section 3, the configuration alpha is chosen once):
 *   nm_spmm_prepare             rewrites the packed weight into matrix-core operand order in the
 *                               workspace (nothing to do, and no workspace needed, when
 *                               nm_spmm_workspace_bytes() is 0).  T is the token count the product
 *                               calls will use (it selects the same kernels).
 *   nm_linear_forward_prepared  the product alone, reading a workspace that nm_spmm_prepare filled
 *                               for the same (values, indices, O, K, N, M, T); the workspace is
 *                               not modified, so it can serve any number of calls.
 * nm_linear_forward(args) == nm_spmm_prepare(args) followed by nm_linear_forward_prepared(args).
 */
int32_t nm_spmm_prepare(const nm_bf16* values, const uint32_t* indices, int64_t O, int64_t K,
                        int32_t N, int32_t M, int64_t T,
                        void* workspace, size_t workspace_bytes, void* stream);

int32_t nm_linear_forward_prepared(const nm_bf16* values, const uint32_t* indices, int64_t O,
                                   int64_t K, int32_t N, int32_t M, const nm_bf16* X, int64_t T,
                                   int64_t ldx, const float* bias, void* Y, int64_t ldy,
                                   int32_t out_dtype, const void* workspace,
                                   size_t workspace_bytes, void* stream);

/*
 * nm_linear_forward_prepared_batched -- nm_linear_forward_prepared for every descriptor, in as few launches as
 * the shapes allow: large layers of the same operand form (N <= 2, or N > 2) share one launch of the persistent
 * product kernel, whose blocks walk the tiles of all of them as one list.  For the independent products of a
 * stack of layers (each with its own input; Section 3: one level per layer) this removes the partial last round
 * of tiles every single launch ends with.  Small layers (a few tokens: batch-1 inference) likewise share launches
 * of the tiled kernel, which no one of them could fill.  Results are bit-identical to the single calls, with one
 * exception: a layer whose reduction a single call cuts into ranges (few tiles, long K; see nm_spmm) is not cut
 * inside a call that fills the chip anyway, and its sums then differ in rounding order.
 *   descs  HOST array of `count` descriptors, read before the call returns.  Fields as the arguments of
 *          nm_linear_forward_prepared; the outputs must not overlap each other or any input.
 * Errors as for nm_linear_forward_prepared (the first offending descriptor decides); nothing is launched on an
 * argument error or a short workspace.
 */
typedef struct nm_forward_desc {
  const nm_bf16* values;    /* device, packed layer (values, indices) at level N:M */
  const uint32_t* indices;
  int64_t O, K;
  int32_t N, M;
  const nm_bf16* X;         /* device, [T, K], ld ldx */
  int64_t T, ldx;
  const float* bias;        /* device, [O] or NULL */
  void* Y;                  /* device, out, [T, O], ld ldy */
  int64_t ldy;
  int32_t out_dtype, reserved;
  void* workspace;          /* filled by nm_spmm_prepare / nm_pack_prepare_batched for this layer and T */
  size_t workspace_bytes;
} nm_forward_desc;
int32_t nm_linear_forward_prepared_batched(const nm_forward_desc* descs, int32_t count, void* stream);

/*
 * Training products of one sparse layer (Section 3.2: in every step the gradient of the loss is taken with
 * respect to the sparse weights of the chosen configuration; Section 3.1, the weight-update figure: the sparse
 * matrix of the applied level is trained inside the shared weight).  With Y = X * (W (.) m)^T and the mask m of
 * the step held fixed:
 *
 *   nm_linear_backward_input    dX[t, k] = sum_o dY[t, o] * Ws[o, k], fp32 accumulation.
 *       Ws   in   the masked dense weight W (.) m, [O, K], ld ldw (what nm_prune writes to W_masked and what
 *                 nm_unpack restores from the packed form)
 *       dY   in   [T, O], ld ldy            dX   out  [T, K], ld ldx, float or bfloat16 (out_dtype)
 *       workspace scratch of nm_backward_input_workspace_bytes(O, K, T) bytes, 256-byte aligned (large layers:
 *                 the weight is first written transposed in matrix-core operand order, then the product is
 *                 the forward one); NULL allowed when that size is 0.  Contents undefined afterwards.
 *   nm_linear_backward_weight   dW[o, k] = m[o, k] * sum_t dY[t, o] * X[t, k], fp32 accumulation.
 *       dY   in   [T, O], ld ldy            X    in   [T, K], ld ldx
 *       mask in   mask words of the step as nm_prune writes them ([O, ceil(K/32)]); pruned positions receive
 *                 +0.  NULL = no mask: every shared weight receives the gradient of its position.
 *       dW   out  [O, K], ld lddw, float or bfloat16 (out_dtype)
 *       workspace scratch of nm_backward_weight_workspace_bytes(O, K, T) bytes, 256-byte aligned (the token
 *                 reduction is cut into ranges whose partial sums are added in a fixed order, so results
 *                 repeat bit for bit); NULL allowed when that size is 0.  Contents undefined afterwards;
 *                 concurrent calls need distinct workspaces.
 * The matrix-core kernels need 16-byte aligned operands, leading dimensions that are multiples of 8, K % 8 == 0
 * and O % 32 == 0 (dX) or O % 8 == 0 (dW); other shapes run a slower general kernel with the same results.
 * Errors: NM_ERR_NULL, NM_ERR_SHAPE (sizes <= 0, a leading dimension smaller than its row), NM_ERR_DTYPE,
 * NM_ERR_ALIGN (element alignment), NM_ERR_WORKSPACE, NM_ERR_DEVICE.
 */
size_t nm_backward_input_workspace_bytes(int64_t O, int64_t K, int64_t T);
size_t nm_backward_weight_workspace_bytes(int64_t O, int64_t K, int64_t T);
int32_t nm_linear_backward_input(const nm_bf16* Ws, int64_t O, int64_t K, int64_t ldw, const nm_bf16* dY,
                                 int64_t T, int64_t ldy, void* dX, int64_t ldx, int32_t out_dtype,
                                 void* workspace, size_t workspace_bytes, void* stream);
int32_t nm_linear_backward_weight(const nm_bf16* dY, int64_t T, int64_t O, int64_t ldy, const nm_bf16* X,
                                  int64_t K, int64_t ldx, const uint32_t* mask, void* dW, int64_t lddw,
                                  int32_t out_dtype, void* workspace, size_t workspace_bytes, void* stream);

/*
 * nm_prune_scored -- Eq. (1) with a saliency supplied by the caller (Section 3.1: rho can be the weight magnitude,
 * a Taylor score, ...): in every aligned group of M the N positions with the largest score are kept.
 *   score  in   float [O, K], ld lds, 4-byte aligned.  Equal scores go to the lower index; -0 equals +0; a NaN
 *               ranks above every number.
 *   mask   out  [O, ceil(K/32)] words as nm_prune writes them; feed them to nm_pack(mask), nm_mask_check,
 *               nm_linear_backward_weight or the int8 calls.
 * With score = |W| it writes the mask nm_prune writes.
 */
int32_t nm_prune_scored(const float* score, int64_t O, int64_t K, int64_t lds, int32_t N, int32_t M,
                        uint32_t* mask, void* stream);

/*
 * int8 form of the layer (Section 4, the post-training-quantisation experiment of Table 6: 8-bit quantisation on
 * top of the sparse networks; Section 3.1: any saliency may produce the mask):
 *
 *   acc[t, o] = sum_k m[o, k] * Wq[o, k] * Xq[t, k]                 exact int32 sum
 *   Y[t, o]   = fma(float(acc[t, o]), x_scale * w_scale[o], bias[o])   (fp32; or acc itself for NM_OUT_I32)
 *
 *   Wq       in   dense int8 weight [O, K], ld ldw.  Only positions whose mask bit is set are used; what the
 *                 others hold is ignored (a symmetric quantiser leaves pruned weights at 0 anyway).
 *   mask     in   mask words [O, ceil(K/32)] of level N:M as nm_prune writes them for the float weight, or from
 *                 any other saliency; it must be legal for the level (nm_mask_check == 0), otherwise kept
 *                 weights beyond two per run of four may be dropped at levels with N <= 2.
 *   Xq       in   int8 [T, K], ld ldx
 *   x_scale, w_scale ([O], NULL = 1), bias ([O], NULL = 0)  fp32 rescaling, not used for NM_OUT_I32
 *   Y        out  [T, O], ld ldy: float, bfloat16 (round to nearest even) or int32
 *   workspace scratch of nm_i8_workspace_bytes(O, K, N, M, T) bytes, 256-byte aligned (NULL allowed when 0): the
 *             weight compressed to matrix-core operand order (values + 2-bit selectors at N <= 2, masked dense
 *             otherwise), in the order of the kernel the token count T selects (large layers: the persistent
 *             kernel's stream order, rows padded to whole 256-row tiles).
 * nm_linear_forward_i8 = nm_i8_prepare (weight only, once per weight and token count) +
 * nm_linear_forward_i8_prepared (the product; the workspace is only read).  The matrix-core kernels need K % 128 == 0, 16-byte aligned Wq and Xq
 * and ldw, ldx multiples of 16; other shapes run a general kernel on Wq and mask with the same results.
 * K * 127 * 128 must stay below 2^31 (K <= 132096) for the integer sum not to wrap.
 * Errors as for nm_linear_forward.
 */
size_t nm_i8_workspace_bytes(int64_t O, int64_t K, int32_t N, int32_t M, int64_t T);
int32_t nm_linear_forward_i8(const int8_t* Wq, int64_t O, int64_t K, int64_t ldw, const uint32_t* mask, int32_t N,
                             int32_t M, const int8_t* Xq, int64_t T, int64_t ldx, float x_scale,
                             const float* w_scale, const float* bias, void* Y, int64_t ldy, int32_t out_dtype,
                             void* workspace, size_t workspace_bytes, void* stream);
int32_t nm_i8_prepare(const int8_t* Wq, int64_t O, int64_t K, int64_t ldw, const uint32_t* mask, int32_t N,
                      int32_t M, int64_t T, void* workspace, size_t workspace_bytes, void* stream);
int32_t nm_linear_forward_i8_prepared(const int8_t* Wq, int64_t O, int64_t K, int64_t ldw, const uint32_t* mask,
                                      int32_t N, int32_t M, const int8_t* Xq, int64_t T, int64_t ldx, float x_scale,
                                      const float* w_scale, const float* bias, void* Y, int64_t ldy,
                                      int32_t out_dtype, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Compressed form of the int8 layer (Section 1 and Section 2, Fig. 2 upper part, for the quantised sparse weight of
 * Section 4's Table 6): the kept int8 values of every group in ascending position, int8 [O, K*N/M]
 * (nm_values_i8_bytes), and for each its log2(M)-bit position in the index stream of the bfloat16 layer
 * (nm_index_bytes; the positions depend on the mask alone).  Half the bytes of the bfloat16 values, and
 * N/M * (1 + log2(M)/8) bytes per weight instead of the 1 + 1/8 of dense weight + mask words.
 *   nm_pack_i8      Wq [O, K] (ld ldw) under `mask` (mask words as nm_prune writes them; a mask without exactly N
 *                   bits in a group is made usable as in nm_pack: the N lowest set positions, missing ones completed
 *                   with the lowest unset positions stored as 0) -> values, indices.
 *   nm_unpack_i8    the inverse: Wq_dense[o, g*M + position] = value, 0 elsewhere; every element of the O x K block
 *                   is written.
 *   nm_linear_forward_i8_packed, nm_i8_prepare_packed, nm_linear_forward_i8_packed_prepared
 *                   nm_linear_forward_i8, nm_i8_prepare and nm_linear_forward_i8_prepared with the weight given in
 *                   this form; same workspace (nm_i8_workspace_bytes), same bytes in it, same results.  The matrix-core
 *                   kernels need K % 128 == 0, a 16-byte aligned Xq and ldx a multiple of 16; other shapes run a
 *                   general kernel on the compressed form.
 * Errors: NM_ERR_NULL, NM_ERR_LEVEL, NM_ERR_SHAPE, NM_ERR_ALIGN (mask, indices: 4 bytes), NM_ERR_DTYPE,
 * NM_ERR_WORKSPACE, NM_ERR_DEVICE; nothing is launched on an argument error.
 */
size_t nm_values_i8_bytes(int64_t O, int64_t K, int32_t N, int32_t M);
int32_t nm_pack_i8(const int8_t* Wq, int64_t O, int64_t K, int64_t ldw, int32_t N, int32_t M, const uint32_t* mask,
                   int8_t* values, uint32_t* indices, void* stream);
int32_t nm_unpack_i8(const int8_t* values, const uint32_t* indices, int64_t O, int64_t K, int32_t N, int32_t M,
                     int8_t* Wq_dense, int64_t ldw, void* stream);
int32_t nm_linear_forward_i8_packed(const int8_t* values, const uint32_t* indices, int64_t O, int64_t K, int32_t N,
                                    int32_t M, const int8_t* Xq, int64_t T, int64_t ldx, float x_scale,
                                    const float* w_scale, const float* bias, void* Y, int64_t ldy, int32_t out_dtype,
                                    void* workspace, size_t workspace_bytes, void* stream);
int32_t nm_i8_prepare_packed(const int8_t* values, const uint32_t* indices, int64_t O, int64_t K, int32_t N, int32_t M,
                             int64_t T, void* workspace, size_t workspace_bytes, void* stream);
int32_t nm_linear_forward_i8_packed_prepared(const int8_t* values, const uint32_t* indices, int64_t O, int64_t K,
                                             int32_t N, int32_t M, const int8_t* Xq, int64_t T, int64_t ldx,
                                             float x_scale, const float* w_scale, const float* bias, void* Y,
                                             int64_t ldy, int32_t out_dtype, void* workspace, size_t workspace_bytes,
                                             void* stream);

/*
 * nm_pack_prepare_batched -- for every descriptor nm_pack(mask = NULL) followed by nm_spmm_prepare, in as few
 * launches as the shapes allow: a model's layers are compressed and made ready for their products together
 * (Section 3, configuration alpha = (s^1 ... s^L); Section 3.1: the sparse weights are derived from the shared
 * ones each time a configuration is chosen).  It writes exactly the bytes the two calls write.
 *   descs  HOST array of `count` descriptors, read before the call returns.  W is [O, K] contiguous;
 *          workspace holds nm_spmm_workspace_bytes(O, K, N, M, T) bytes, 256-byte aligned, one per layer
 *          (NULL allowed where that size is 0); T is the token count of the product calls that follow
 *          (nm_linear_forward_prepared with the same values, indices, workspace and T).
 * Errors as for nm_pack and nm_spmm_prepare; NM_ERR_WORKSPACE before anything is launched.
 */
typedef struct nm_layer_desc {
  const nm_bf16* W;  /* device, [O, K] contiguous */
  nm_bf16* values;   /* device, out */
  uint32_t* indices; /* device, out */
  int64_t O, K;
  int32_t N, M;
  int64_t T;
  void* workspace;   /* device, out */
  size_t workspace_bytes;
} nm_layer_desc;

int32_t nm_pack_prepare_batched(const nm_layer_desc* descs, int32_t count, void* stream);

/*
 * Measurement aids -- no part of the layer and of no passage of the paper: the two rates the kernels above are
 * priced against, measured on the device at hand rather than taken from a data sheet.
 *   nm_probe_matrix_rate  a loop of nothing but matrix instructions on register operands, every compute unit
 *                         busy with two waves per SIMD.  kind 0: the 2:4 sparse bfloat16 instruction
 *                         (v_smfmac_f32_16x16x64_bf16), kind 1: the dense one (v_mfma_f32_16x16x32_bf16); each
 *                         wave issues iters * 32 of them.
 *       sink  device, out: nm_probe_sink_bytes() bytes, 4-byte aligned (keeps the sums alive; contents arbitrary)
 *       ops   HOST, out: dense-equivalent operations the launch performs (2 * 16 * 16 * K per instruction);
 *             divide by the launch's measured duration.
 *   nm_probe_copy         dst[0 .. bytes) = src[0 .. bytes): a plain streaming copy, 16 bytes per lane; bytes a
 *                         multiple of 16, both pointers 16-byte aligned, no overlap.  Reads and writes `bytes`
 *                         once each, which also calibrates a profiler's byte counters.
 * Errors: NM_ERR_NULL, NM_ERR_DTYPE (kind), NM_ERR_SHAPE (iters <= 0, bytes), NM_ERR_ALIGN, NM_ERR_DEVICE.
 */
size_t nm_probe_sink_bytes(void);
int32_t nm_probe_matrix_rate(int32_t kind, int32_t iters, void* sink, int64_t* ops, void* stream);
int32_t nm_probe_copy(const void* src, void* dst, size_t bytes, void* stream);

/*
 * Host-only helpers of the configuration search (no GPU work, HOST pointers throughout).
 *
 * nm_config_cost -- Section 3.2 ("Prioritizing Sparser Subnets"; the appendix on settings: the cost F is the
 * network's FLOPs): F(alpha) = fixed_cost + sum_l layer_macs[l] * N[l] / M[l], a linear layer at N:M performing
 * N/M of its dense multiply-accumulates (Section 2).  Returns -1 on a NULL pointer, L <= 0, an illegal level or
 * a negative layer cost.  With DeiT-B's layers it gives the 17.6G (dense) and 9.2G (uniform 2:4) of Table 1.
 *
 * nm_sample_config -- the two-step sampling algorithm (Section 3.2, "Sampling Strategy"): (1) one of the
 * n_edges - 1 cost intervals [edges[i], edges[i+1]) uniformly (the last one includes its upper end, since
 * configurations with F = C_upper are admitted); (2) a configuration drawn layer by layer from the current
 * choice probabilities, repeated until its cost falls into the interval (i.e. from the probabilities
 * conditioned on the interval).  The random numbers are the caller's: `uniforms` holds n_uniforms numbers in
 * [0, 1), consumed in order (one for the interval, then L per attempt); a layer's choice is the first whose
 * cumulative probability exceeds its uniform.
 *   choice_N, choice_M  the S levels to choose from;  probs  [L, S] row-major, each row summing to 1
 *   choice  out [L]: index into the S levels;  interval  out;  used  out: uniforms consumed
 * Returns NM_OK, NM_ERR_NULL / NM_ERR_SHAPE / NM_ERR_LEVEL for bad arguments (edges must increase strictly), or
 * NM_ERR_EXHAUSTED when the uniforms run out first (choice then holds the last attempt).
 */
double nm_config_cost(const double* layer_macs, const int32_t* N, const int32_t* M, int32_t L, double fixed_cost);
int32_t nm_sample_config(const double* layer_macs, int32_t L, double fixed_cost, const int32_t* choice_N,
                         const int32_t* choice_M, int32_t S, const double* probs, const double* edges,
                         int32_t n_edges, const double* uniforms, int64_t n_uniforms, int32_t* choice,
                         int32_t* interval, int64_t* used);

#ifdef __cplusplus
}
#endif
#endif /* NM_SPARSE_H */
