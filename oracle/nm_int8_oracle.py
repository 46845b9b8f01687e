"""CPU checker for the int8 form of the N:M-sparse linear layer.  TEST INFRASTRUCTURE ONLY.

Section 4 (the post-training-quantisation experiment, Table 6) applies 8-bit quantisation to the sparse
networks: the layer then multiplies int8 activations with an int8 weight that keeps the N:M pattern
(a pruned weight is zero before quantisation and a symmetric quantiser keeps zero at zero), accumulates
exactly in integers, and rescales.  The quantiser itself (how scales are calibrated) is not part of this
path; the checker takes the integers and the scales as given.

    acc[t, o] = sum_k m[o, k] * Wq[o, k] * Xq[t, k]                 exact integer
    Y[t, o]   = x_scale * w_scale[o] * acc[t, o] + bias[o]          fp64 here

The mask is an input (Section 3.1: any saliency may produce it; in the quantisation flow it is the mask of
the float weight).  Plain numpy, int64 accumulation; shares no code with the HIP path.

`nm_pack_i8` / `nm_unpack_i8` are the compressed form of the quantised sparse weight (Section 1; Section 2,
Fig. 2 upper part): the kept int8 values of every group in ascending position and a log2(M)-bit position for
each, in the index stream of the bfloat16 layer (per row, least significant bit first, field f = g*N + j in bits
[f*b, f*b + b), rows zero-padded to 32-bit words).  `nm_accumulate_i8_packed_loops` is Fig. 2 (lower part)
literally on that form: decode the position, select the activation, multiply, add.
"""
from __future__ import annotations

from typing import Optional

import numpy as np


def nm_accumulate_i8(xq: np.ndarray, wq: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """Exact integer product X . (W (.) m)^T of int8 operands, int64 [T, O]."""
    if xq.dtype != np.int8 or wq.dtype != np.int8:
        raise ValueError("operands must be int8")
    if mask.shape != wq.shape or xq.shape[1] != wq.shape[1]:
        raise ValueError("shape mismatch")
    ws = np.where(mask, wq, 0).astype(np.int64)
    return xq.astype(np.int64) @ ws.T


def nm_linear_i8(xq: np.ndarray, wq: np.ndarray, mask: np.ndarray, x_scale: float, w_scale: np.ndarray,
                 bias: Optional[np.ndarray] = None) -> np.ndarray:
    """Rescaled product in fp64: x_scale * w_scale[o] * acc[t, o] (+ bias[o])."""
    acc = nm_accumulate_i8(xq, wq, mask).astype(np.float64)
    y = acc * (np.float64(x_scale) * np.asarray(w_scale, dtype=np.float64))[None, :]
    if bias is not None:
        y = y + np.asarray(bias, dtype=np.float64)[None, :]
    return y


def nm_accumulate_i8_loops(xq: np.ndarray, wq: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """The same sum one product at a time, Python integers (tiny inputs only)."""
    T, K = xq.shape
    O = wq.shape[0]
    out = np.zeros((T, O), dtype=np.int64)
    for t in range(T):
        for o in range(O):
            s = 0
            for k in range(K):
                if mask[o, k]:
                    s += int(wq[o, k]) * int(xq[t, k])
            out[t, o] = s
    return out


def _index_bits(M: int) -> int:
    return {4: 2, 8: 3, 16: 4}[M]


def nm_pack_i8(wq: np.ndarray, mask: np.ndarray, N: int, M: int):
    """values int8 [O, K*N/M] (kept weights, ascending position inside each group) and indices uint32
    [O, ceil(K*N/M*log2(M)/32)] (their positions, LSB-first bit stream per row).  The mask must keep exactly N
    per aligned group of M along K."""
    if wq.dtype != np.int8 or mask.shape != wq.shape:
        raise ValueError("wq must be int8 and mask of its shape")
    O, K = wq.shape
    b = _index_bits(M)
    if K % M or not (1 <= N <= M):
        raise ValueError("illegal level or K")
    nf = K // M * N
    nw = (nf * b + 31) // 32
    values = np.zeros((O, nf), dtype=np.int8)
    indices = np.zeros((O, nw), dtype=np.uint32)
    for o in range(O):
        stream = 0  # the row's bit stream as one Python integer
        f = 0
        for g in range(K // M):
            kept = [p for p in range(M) if mask[o, g * M + p]]
            if len(kept) != N:
                raise ValueError("mask does not keep exactly N per group")
            for p in kept:
                values[o, f] = wq[o, g * M + p]
                stream |= p << (f * b)
                f += 1
        for w in range(nw):
            indices[o, w] = (stream >> (32 * w)) & 0xFFFFFFFF
    return values, indices


def nm_unpack_i8(values: np.ndarray, indices: np.ndarray, K: int, N: int, M: int) -> np.ndarray:
    """Inverse of nm_pack_i8: dense int8 [O, K], 0 in every pruned position."""
    O = values.shape[0]
    b = _index_bits(M)
    out = np.zeros((O, K), dtype=np.int8)
    for o in range(O):
        stream = 0
        for w, word in enumerate(indices[o]):
            stream |= int(word) << (32 * w)
        for f in range(K // M * N):
            p = (stream >> (f * b)) & (M - 1)
            out[o, (f // N) * M + p] = values[o, f]
    return out


def nm_accumulate_i8_packed_loops(values: np.ndarray, indices: np.ndarray, xq: np.ndarray, K: int, N: int,
                                  M: int) -> np.ndarray:
    """acc[t, o] = sum_g sum_{j<N} Xq[t, g*M + idx[o, g, j]] * val[o, g, j] in Python integers (tiny inputs)."""
    O = values.shape[0]
    T = xq.shape[0]
    b = _index_bits(M)
    out = np.zeros((T, O), dtype=np.int64)
    for o in range(O):
        stream = 0
        for w, word in enumerate(indices[o]):
            stream |= int(word) << (32 * w)
        for t in range(T):
            s = 0
            for f in range(K // M * N):
                p = (stream >> (f * b)) & (M - 1)
                s += int(xq[t, (f // N) * M + p]) * int(values[o, f])
            out[t, o] = s
    return out
