"""CPU checker for the N:M-sparse linear layer.  TEST INFRASTRUCTURE ONLY.

This file is the yardstick the HIP library is compared with.  It is plain
numpy (fp64 for all floating point), slow on purpose, and shares no code with
the HIP path; nothing in the product imports it.  Only the tests, the smoke
check and the benchmark's CPU-baseline leg may call it.

What it computes, and where the paper defines it:

* `nm_mask`      -- Section 3.1, "Dynamic Masking", Eq. (1): in every group of M
                   consecutive weights keep the N with the largest saliency,
                   saliency = weight magnitude (the paper's default).
* `nm_mask_from_scores` -- the same selection with the saliency given as numbers (Section
                   3.1 names the Taylor score as an alternative to the magnitude).
* `apply_mask`   -- Section 3.1: a weight whose mask value is 0 is set to zero.
* `nm_pack` / `nm_unpack` -- Section 1 and Section 2 (Fig. 2, upper part): the
                   compressed form stores the kept values and, for each, a
                   log2(M)-bit index of its position in its group.
* `nm_linear`    -- Section 2 (Fig. 2, lower part): the sparse product equals
                   the ordinary matrix product with the masked weight.  It is
                   written here as exactly that: a dense fp64 GEMM.

* `nm_rank`      -- Section 3, "Subset-Superset Relationship": under one pruning
                   criterion the weights kept at a sparser level are a subset
                   of those kept at a denser one.  So one number per weight,
                   its rank inside its group in the order (saliency
                   descending, position ascending), holds every level at once:
                   the mask of N:M is rank < N.  `rank_nibbles` is its stored
                   form (4 bits per weight).

* `nm_linear_backward` -- Section 3.2, the supernet training loop: the chosen
                   configuration's sparse weights W(alpha) take part in the
                   forward pass and the gradient of the loss is taken with
                   respect to them; Section 3.1 (the weight-update figure): the
                   sparse matrix of the applied level is what is trained, inside
                   the shared weight.  For one layer Y = X (W (.) m)^T with the
                   mask held fixed this is the chain rule: dX = dY (W (.) m),
                   dW = (dY^T X) (.) m.  The unmasked product dY^T X (every
                   shared weight receives the gradient of its position) is the
                   other common choice and is offered as `masked_grad=False`.

Readings where the paper is silent or garbled (all listed in the design notes):
zeta of Eq. (1) is the N-th LARGEST score; exactly N are kept, equal scores go
to the lower index; groups are aligned and run along the input (reduction)
dimension of a row-major [O, K] weight; saliency is compared on the stored
bfloat16 value (key = bit pattern without the sign bit); kept values are stored
in ascending position; index fields form an LSB-first bit stream per row,
padded to a 32-bit word.

All matrices are carried as bfloat16 bit patterns (numpy uint16).
"""
from __future__ import annotations

import math
from typing import Optional, Tuple

import numpy as np

LEGAL_M = (4, 8, 16)


def check_level(N: int, M: int) -> None:
    if M not in LEGAL_M or not (1 <= N <= M):
        raise ValueError(f"illegal level {N}:{M}")


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact value of each bfloat16 bit pattern, as float64."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def saliency_key(w_bits: np.ndarray) -> np.ndarray:
    """rho(w) = |w| (Section 3.1), as an integer that orders like |w|.

    For bfloat16 (sign, 8 exponent bits, 7 fraction bits) dropping the sign bit
    leaves an unsigned integer that increases with the magnitude; +0 and -0 get
    the same key.
    """
    return (np.ascontiguousarray(w_bits, dtype=np.uint16) & np.uint16(0x7FFF)).astype(np.int32)


def nm_mask(w_bits: np.ndarray, N: int, M: int) -> np.ndarray:
    """Eq. (1): boolean mask [O, K], exactly N ones in each aligned group of M along K.

    Order the M members of a group by (saliency descending, position ascending);
    the first N are kept.
    """
    check_level(N, M)
    O, K = w_bits.shape
    if K % M:
        raise ValueError("K must be a multiple of M")
    key = saliency_key(w_bits).reshape(O, K // M, M)
    order = np.argsort(-key, axis=-1, kind="stable")  # stable: equal keys stay in position order
    mask = np.zeros((O, K // M, M), dtype=bool)
    np.put_along_axis(mask, order[..., :N], True, axis=-1)
    return mask.reshape(O, K)


def nm_mask_from_scores(scores: np.ndarray, N: int, M: int) -> np.ndarray:
    """Eq. (1) with a saliency supplied from outside (Section 3.1: rho may be the weight magnitude, a Taylor
    score, ...): boolean mask [O, K] keeping, in every aligned group of M, the N positions with the largest
    score; equal scores go to the lower index; -0 equals +0; a NaN score ranks above every number (kept first,
    like the NaN weights of the magnitude rule).  Scores are compared as float32.
    """
    check_level(N, M)
    s = np.ascontiguousarray(scores, dtype=np.float32)
    O, K = s.shape
    if K % M:
        raise ValueError("K must be a multiple of M")
    g = s.reshape(O, K // M, M)
    nan = np.isnan(g)
    val = np.where(nan, np.float32(0), g).astype(np.float64)
    # NaN first, then descending value, then ascending position: stable sorts compose, minor key first
    by_value = np.argsort(-val, axis=-1, kind="stable")
    nan_sorted = np.take_along_axis(nan, by_value, axis=-1)
    nan_first = np.argsort(~nan_sorted, axis=-1, kind="stable")
    order = np.take_along_axis(by_value, nan_first, axis=-1)
    mask = np.zeros((O, K // M, M), dtype=bool)
    np.put_along_axis(mask, order[..., :N], True, axis=-1)
    return mask.reshape(O, K)


def nm_rank(w_bits: np.ndarray, M: int) -> np.ndarray:
    """Section 3, subset-superset relationship: rank [O, K] (uint8, 0..M-1) of each weight inside
    its aligned group of M, counted in the order (saliency descending, position ascending).

    The weight of rank r is the (r+1)-th to be kept as N grows, so the mask of level N:M is
    rank < N for every N (and N = M keeps everything).
    """
    check_level(M, M)
    O, K = w_bits.shape
    if K % M:
        raise ValueError("K must be a multiple of M")
    key = saliency_key(w_bits).reshape(O, K // M, M)
    order = np.argsort(-key, axis=-1, kind="stable")
    rank = np.empty((O, K // M, M), dtype=np.uint8)
    np.put_along_axis(rank, order, np.broadcast_to(np.arange(M, dtype=np.uint8), order.shape), axis=-1)
    return rank.reshape(O, K)


def rank_nibbles(rank: np.ndarray) -> np.ndarray:
    """Stored form of the ranks: uint8 [O, K/2]; weight k sits in bits [4 (k mod 2), +4) of byte k // 2."""
    O, K = rank.shape
    if K % 2:
        raise ValueError("K must be even")
    r = rank.astype(np.uint8)
    return (r[:, 0::2] | (r[:, 1::2] << np.uint8(4))).astype(np.uint8)


def nibbles_to_rank(nib: np.ndarray) -> np.ndarray:
    O, H = nib.shape
    out = np.empty((O, 2 * H), dtype=np.uint8)
    out[:, 0::2] = nib & np.uint8(15)
    out[:, 1::2] = nib >> np.uint8(4)
    return out


def apply_mask(w_bits: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """W (.) m : pruned weights become +0 (Section 3.1)."""
    return np.where(mask, w_bits, np.uint16(0)).astype(np.uint16)


def mask_words_per_row(K: int) -> int:
    return (K + 31) // 32


def mask_to_words(mask: np.ndarray) -> np.ndarray:
    """Bit (k mod 32) of word floor(k/32) of row o is m[o, k]; uint32 [O, ceil(K/32)]."""
    O, K = mask.shape
    nw = mask_words_per_row(K)
    out = np.zeros((O, nw), dtype=np.uint32)
    for k in range(K):
        out[:, k // 32] |= mask[:, k].astype(np.uint32) << np.uint32(k % 32)
    return out


def words_to_mask(words: np.ndarray, K: int) -> np.ndarray:
    O = words.shape[0]
    mask = np.zeros((O, K), dtype=bool)
    for k in range(K):
        mask[:, k] = ((words[:, k // 32] >> np.uint32(k % 32)) & 1).astype(bool)
    return mask


def index_bits(M: int) -> int:
    return int(math.log2(M))


def values_per_row(K: int, N: int, M: int) -> int:
    return K // M * N


def index_words_per_row(K: int, N: int, M: int) -> int:
    return (values_per_row(K, N, M) * index_bits(M) + 31) // 32


def nm_pack(w_bits: np.ndarray, mask: np.ndarray, N: int, M: int) -> Tuple[np.ndarray, np.ndarray]:
    """Compressed form of W (.) m (Fig. 2, upper part).

    values  uint16 [O, K*N/M]: the kept weights of each group, ascending position.
    indices uint32 [O, ceil(K*N/M*log2(M)/32)]: field f = g*N + j holds the position
            (0..M-1) of the j-th kept weight of group g in bits [f*b, f*b+b) of the
            row's bit stream, least significant bit first, zero padded.
    The mask must have exactly N ones per group.
    """
    check_level(N, M)
    O, K = w_bits.shape
    G = K // M
    m3 = mask.reshape(O, G, M)
    if not np.all(m3.sum(axis=-1) == N):
        raise ValueError("mask does not keep exactly N per group")
    # positions of the ones, ascending: stable sort of "not kept" puts kept positions first in order
    pos = np.argsort(~m3, axis=-1, kind="stable")[..., :N]  # [O, G, N]
    vals = np.take_along_axis(w_bits.reshape(O, G, M), pos, axis=-1).reshape(O, G * N).astype(np.uint16)
    b = index_bits(M)
    nw = index_words_per_row(K, N, M)
    stream = np.zeros((O, nw), dtype=np.uint64)
    fields = pos.reshape(O, G * N).astype(np.uint64)
    for f in range(G * N):
        off = f * b
        w, s = off // 32, off % 32
        shifted = fields[:, f] << np.uint64(s)
        stream[:, w] |= shifted & np.uint64(0xFFFFFFFF)
        if s + b > 32:
            stream[:, w + 1] |= shifted >> np.uint64(32)
    return vals, stream.astype(np.uint32)


def nm_unpack(values: np.ndarray, indices: np.ndarray, K: int, N: int, M: int) -> np.ndarray:
    """Inverse of nm_pack: dense [O, K] bf16 bits with +0 in every pruned position."""
    check_level(N, M)
    O = values.shape[0]
    G = K // M
    b = index_bits(M)
    out = np.zeros((O, K), dtype=np.uint16)
    idx64 = indices.astype(np.uint64)
    rows = np.arange(O)
    for f in range(G * N):
        off = f * b
        w, s = off // 32, off % 32
        field = idx64[:, w] >> np.uint64(s)
        if s + b > 32:
            field = field | (idx64[:, w + 1] << np.uint64(32 - s))
        p = (field & np.uint64(M - 1)).astype(np.int64)
        out[rows, (f // N) * M + p] = values[:, f]
    return out


def nm_linear(x_bits: np.ndarray, w_bits: np.ndarray, mask: np.ndarray,
              bias: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
    """Y = X . (W (.) m)^T (+ bias) in fp64, and the bound B = |X| . |W (.) m|^T.

    Fig. 2 (lower part) states that the sparse product is the accurate matrix
    product; so this is the ordinary dense product with the masked weight.
    B[t, o] = sum_k |x_tk * w_ok| scales the acceptance tolerance.
    """
    X = bf16_bits_to_f64(x_bits)
    Ws = bf16_bits_to_f64(apply_mask(w_bits, mask))
    Y = X @ Ws.T
    B = np.abs(X) @ np.abs(Ws).T
    if bias is not None:
        Y = Y + np.asarray(bias, dtype=np.float64)[None, :]
    return Y, B


def nm_linear_from_bits(x_bits: np.ndarray, w_bits: np.ndarray, N: int, M: int,
                        bias: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
    """prune then multiply: the whole path for one layer."""
    return nm_linear(x_bits, w_bits, nm_mask(w_bits, N, M), bias)


def nm_linear_backward(dy_bits: np.ndarray, x_bits: np.ndarray, w_bits: np.ndarray, mask: np.ndarray,
                       masked_grad: bool = True) -> Tuple[np.ndarray, np.ndarray, np.ndarray, np.ndarray]:
    """Gradients through Y = X . (W (.) m)^T for a given dL/dY (Section 3.2: the gradient is taken
    with respect to the sparse weights of the chosen configuration; the mask is a constant of the step).

        dX[t, k] = sum_o dY[t, o] * (W (.) m)[o, k]
        dW[o, k] = m[o, k] * sum_t dY[t, o] * X[t, k]      (masked_grad: only kept weights are trained)
        dW[o, k] =           sum_t dY[t, o] * X[t, k]      (otherwise)

    Returns dX [T, K], dW [O, K] in fp64 and the bounds BX = |dY| . |W (.) m|, BW = |dY|^T . |X| (masked like
    dW) that scale the acceptance tolerance.
    """
    dY = bf16_bits_to_f64(dy_bits)
    X = bf16_bits_to_f64(x_bits)
    Ws = bf16_bits_to_f64(apply_mask(w_bits, mask))
    dX = dY @ Ws
    BX = np.abs(dY) @ np.abs(Ws)
    dW = dY.T @ X
    BW = np.abs(dY).T @ np.abs(X)
    if masked_grad:
        dW = np.where(mask, dW, 0.0)
        BW = np.where(mask, BW, 0.0)
    return dX, dW, BX, BW


def useful_macs(T: int, O: int, K: int, N: int, M: int) -> int:
    """Multiply-accumulates a sparse engine performs: N/M of the dense count (Section 2)."""
    return T * O * (K // M) * N


# --------------------------------------------------------------------------------------
# Loop-only forms for tiny inputs.  They follow the text literally, one group / one output
# at a time, and back the vectorised functions above in the tests.
# --------------------------------------------------------------------------------------

def nm_mask_loops(w_bits: np.ndarray, N: int, M: int) -> np.ndarray:
    """Eq. (1) one group at a time: prune the M-N least salient, lower index wins ties."""
    check_level(N, M)
    O, K = w_bits.shape
    mask = np.zeros((O, K), dtype=bool)
    for o in range(O):
        for g in range(K // M):
            grp = [int(w_bits[o, g * M + i]) & 0x7FFF for i in range(M)]
            kept = []
            for _ in range(N):
                best = -1
                for i in range(M):
                    if i in kept:
                        continue
                    if best < 0 or grp[i] > grp[best]:  # strict: an equal later score never displaces
                        best = i
                kept.append(best)
            for i in kept:
                mask[o, g * M + i] = True
    return mask


def nm_rank_loops(w_bits: np.ndarray, M: int) -> np.ndarray:
    """The rank by counting: how many members of the group come before this one, i.e. have a larger
    score, or the same score and a lower position."""
    O, K = w_bits.shape
    rank = np.zeros((O, K), dtype=np.uint8)
    for o in range(O):
        for g in range(K // M):
            grp = [int(w_bits[o, g * M + i]) & 0x7FFF for i in range(M)]
            for i in range(M):
                before = 0
                for j in range(M):
                    if grp[j] > grp[i] or (grp[j] == grp[i] and j < i):
                        before += 1
                rank[o, g * M + i] = before
    return rank


def spmm_gather_loops(values: np.ndarray, indices: np.ndarray, x_bits: np.ndarray,
                      K: int, N: int, M: int) -> np.ndarray:
    """Fig. 2 (lower part) literally: decode each index, select the activation, multiply, add.

    Y[t, o] = sum_g sum_{j<N} X[t, g*M + idx[o, g, j]] * val[o, g, j], fp64.
    """
    O = values.shape[0]
    T = x_bits.shape[0]
    b = index_bits(M)
    X = bf16_bits_to_f64(x_bits)
    V = bf16_bits_to_f64(values)
    Y = np.zeros((T, O), dtype=np.float64)
    for o in range(O):
        row = 0
        for wi, w in enumerate(indices[o]):
            row |= int(w) << (32 * wi)
        for g in range(K // M):
            for j in range(N):
                f = g * N + j
                p = (row >> (f * b)) & (M - 1)
                for t in range(T):
                    Y[t, o] += X[t, g * M + p] * V[o, f]
    return Y
