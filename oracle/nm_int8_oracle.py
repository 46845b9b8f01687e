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
