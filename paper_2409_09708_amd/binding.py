"""ctypes binding of libnm_sparse.so.  Argument marshalling only: every step of the path runs in the
HIP kernels behind the C ABI (include/nm_sparse.h).  torch provides device memory and the stream.

Tensor conventions: weights / activations / packed values are torch.bfloat16 CUDA tensors; index and
mask words are torch.int32 tensors holding the uint32 bit patterns.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import c_char_p, c_int32, c_int64, c_size_t, c_void_p
from typing import List, Optional, Sequence, Tuple

_LIB = None
_PKG_DIR = os.path.dirname(os.path.abspath(__file__))

NM_OK = 0
NM_OUT_F32, NM_OUT_BF16, NM_OUT_I32 = 0, 1, 2

EXPORTS = (
    "nm_status_string", "nm_last_hip_error", "nm_values_bytes", "nm_index_bytes", "nm_mask_bytes",
    "nm_spmm_workspace_bytes", "nm_prune", "nm_pack", "nm_pack_batched", "nm_unpack", "nm_mask_check",
    "nm_spmm", "nm_linear_forward", "nm_spmm_prepare", "nm_linear_forward_prepared",
    "nm_static_scratch_bytes", "nm_linear_forward_static",
    "nm_probe_sink_bytes", "nm_probe_matrix_rate", "nm_probe_copy",
    "nm_values_i8_bytes", "nm_pack_i8", "nm_unpack_i8", "nm_linear_forward_i8_packed", "nm_i8_prepare_packed",
    "nm_linear_forward_i8_packed_prepared",
    "nm_rank_bytes", "nm_rank", "nm_rank_batched", "nm_rank_mask", "nm_pack_ranked", "nm_pack_ranked_batched", "nm_pack_prepare_batched",
    "nm_config_cost", "nm_sample_config",
    "nm_backward_input_workspace_bytes", "nm_backward_weight_workspace_bytes", "nm_linear_backward_input", "nm_linear_backward_weight",
    "nm_linear_forward_prepared_batched", "nm_prune_scored", "nm_i8_workspace_bytes", "nm_linear_forward_i8", "nm_i8_prepare", "nm_linear_forward_i8_prepared",
)


class NmError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"nm_sparse status {status}: {text}")
        self.status = status


class PackDesc(ctypes.Structure):
    _fields_ = [("W", c_void_p), ("values", c_void_p), ("indices", c_void_p),
                ("O", c_int64), ("K", c_int64), ("N", c_int32), ("M", c_int32)]


class PackRankedDesc(ctypes.Structure):
    _fields_ = [("W", c_void_p), ("rank", c_void_p), ("values", c_void_p), ("indices", c_void_p),
                ("O", c_int64), ("K", c_int64), ("N", c_int32), ("M", c_int32)]


class LayerDesc(ctypes.Structure):
    _fields_ = [("W", c_void_p), ("values", c_void_p), ("indices", c_void_p),
                ("O", c_int64), ("K", c_int64), ("N", c_int32), ("M", c_int32),
                ("T", c_int64), ("workspace", c_void_p), ("workspace_bytes", c_size_t)]


class ForwardDesc(ctypes.Structure):
    _fields_ = [("values", c_void_p), ("indices", c_void_p), ("O", c_int64), ("K", c_int64), ("N", c_int32),
                ("M", c_int32), ("X", c_void_p), ("T", c_int64), ("ldx", c_int64), ("bias", c_void_p), ("Y", c_void_p),
                ("ldy", c_int64), ("out_dtype", c_int32), ("reserved", c_int32), ("workspace", c_void_p),
                ("workspace_bytes", c_size_t)]


class RankDesc(ctypes.Structure):
    _fields_ = [("W", c_void_p), ("rank", c_void_p), ("O", c_int64), ("K", c_int64), ("M", c_int32),
                ("reserved", c_int32)]


def library_path() -> str:
    return os.path.join(_PKG_DIR, "libnm_sparse.so")


def load_library() -> ctypes.CDLL:
    """Load the HIP library (once).  There is no fallback: a missing library is an error."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build it with `python -m paper_2409_09708_amd.build`")
    lib = ctypes.CDLL(path)
    lib.nm_status_string.restype = c_char_p
    lib.nm_status_string.argtypes = [c_int32]
    lib.nm_last_hip_error.restype = c_int32
    lib.nm_last_hip_error.argtypes = []
    for name in ("nm_values_bytes", "nm_index_bytes"):
        getattr(lib, name).restype = c_size_t
        getattr(lib, name).argtypes = [c_int64, c_int64, c_int32, c_int32]
    lib.nm_mask_bytes.restype = c_size_t
    lib.nm_mask_bytes.argtypes = [c_int64, c_int64]
    lib.nm_spmm_workspace_bytes.restype = c_size_t
    lib.nm_spmm_workspace_bytes.argtypes = [c_int64, c_int64, c_int32, c_int32, c_int64]
    lib.nm_prune.restype = c_int32
    lib.nm_prune.argtypes = [c_void_p, c_int64, c_int64, c_int64, c_int32, c_int32, c_void_p, c_void_p, c_void_p]
    lib.nm_pack.restype = c_int32
    lib.nm_pack.argtypes = [c_void_p, c_int64, c_int64, c_int64, c_int32, c_int32, c_void_p, c_void_p, c_void_p,
                            c_void_p]
    lib.nm_pack_batched.restype = c_int32
    lib.nm_pack_batched.argtypes = [ctypes.POINTER(PackDesc), c_int32, c_void_p]
    lib.nm_unpack.restype = c_int32
    lib.nm_unpack.argtypes = [c_void_p, c_void_p, c_int64, c_int64, c_int32, c_int32, c_void_p, c_int64, c_void_p]
    lib.nm_mask_check.restype = c_int32
    lib.nm_mask_check.argtypes = [c_void_p, c_int64, c_int64, c_int32, c_int32, c_void_p, c_void_p]
    lib.nm_spmm.restype = c_int32
    lib.nm_spmm.argtypes = [c_void_p, c_void_p, c_int64, c_int64, c_int32, c_int32, c_void_p, c_int64, c_int64,
                            c_void_p, c_int64, c_int32, c_void_p, c_size_t, c_void_p]
    lib.nm_linear_forward.restype = c_int32
    lib.nm_linear_forward.argtypes = [c_void_p, c_void_p, c_int64, c_int64, c_int32, c_int32, c_void_p, c_int64,
                                      c_int64, c_void_p, c_void_p, c_int64, c_int32, c_void_p, c_size_t, c_void_p]
    lib.nm_spmm_prepare.restype = c_int32
    lib.nm_spmm_prepare.argtypes = [c_void_p, c_void_p, c_int64, c_int64, c_int32, c_int32, c_int64, c_void_p, c_size_t,
                                    c_void_p]
    lib.nm_linear_forward_prepared.restype = c_int32
    lib.nm_linear_forward_prepared.argtypes = lib.nm_linear_forward.argtypes
    lib.nm_static_scratch_bytes.restype = c_size_t
    lib.nm_static_scratch_bytes.argtypes = []
    lib.nm_linear_forward_static.restype = c_int32
    lib.nm_linear_forward_static.argtypes = [c_void_p, c_void_p, c_int64, c_int64, c_int32, c_int32, c_void_p, c_int64,
                                             c_int64, c_void_p, c_void_p, c_int64, c_int32, c_void_p]
    lib.nm_probe_sink_bytes.restype = c_size_t
    lib.nm_probe_sink_bytes.argtypes = []
    lib.nm_probe_matrix_rate.restype = c_int32
    lib.nm_probe_matrix_rate.argtypes = [c_int32, c_int32, c_void_p, ctypes.POINTER(c_int64), c_void_p]
    lib.nm_probe_copy.restype = c_int32
    lib.nm_probe_copy.argtypes = [c_void_p, c_void_p, c_size_t, c_void_p]
    lib.nm_pack_prepare_batched.restype = c_int32
    lib.nm_pack_prepare_batched.argtypes = [ctypes.POINTER(LayerDesc), c_int32, c_void_p]
    lib.nm_rank_bytes.restype = c_size_t
    lib.nm_rank_bytes.argtypes = [c_int64, c_int64]
    lib.nm_rank.restype = c_int32
    lib.nm_rank.argtypes = [c_void_p, c_int64, c_int64, c_int64, c_int32, c_void_p, c_void_p]
    c_double_p, c_int32_p = ctypes.POINTER(ctypes.c_double), ctypes.POINTER(c_int32)
    lib.nm_config_cost.restype = ctypes.c_double
    lib.nm_config_cost.argtypes = [c_double_p, c_int32_p, c_int32_p, c_int32, ctypes.c_double]
    lib.nm_sample_config.restype = c_int32
    lib.nm_sample_config.argtypes = [c_double_p, c_int32, ctypes.c_double, c_int32_p, c_int32_p, c_int32, c_double_p,
                                     c_double_p, c_int32, c_double_p, c_int64, c_int32_p, c_int32_p,
                                     ctypes.POINTER(c_int64)]
    lib.nm_rank_batched.restype = c_int32
    lib.nm_rank_batched.argtypes = [ctypes.POINTER(RankDesc), c_int32, c_void_p]
    lib.nm_rank_mask.restype = c_int32
    lib.nm_rank_mask.argtypes = [c_void_p, c_int64, c_int64, c_int32, c_int32, c_void_p, c_void_p]
    lib.nm_pack_ranked.restype = c_int32
    lib.nm_pack_ranked.argtypes = [c_void_p, c_void_p, c_int64, c_int64, c_int64, c_int32, c_int32, c_void_p, c_void_p,
                                   c_void_p]
    lib.nm_pack_ranked_batched.restype = c_int32
    lib.nm_pack_ranked_batched.argtypes = [ctypes.POINTER(PackRankedDesc), c_int32, c_void_p]
    lib.nm_backward_weight_workspace_bytes.restype = c_size_t
    lib.nm_backward_weight_workspace_bytes.argtypes = [c_int64, c_int64, c_int64]
    lib.nm_linear_backward_input.restype = c_int32
    lib.nm_backward_input_workspace_bytes.restype = c_size_t
    lib.nm_backward_input_workspace_bytes.argtypes = [c_int64, c_int64, c_int64]
    lib.nm_linear_backward_input.argtypes = [c_void_p, c_int64, c_int64, c_int64, c_void_p, c_int64, c_int64, c_void_p,
                                             c_int64, c_int32, c_void_p, c_size_t, c_void_p]
    lib.nm_linear_backward_weight.restype = c_int32
    lib.nm_linear_backward_weight.argtypes = [c_void_p, c_int64, c_int64, c_int64, c_void_p, c_int64, c_int64, c_void_p,
                                              c_void_p, c_int64, c_int32, c_void_p, c_size_t, c_void_p]
    lib.nm_linear_forward_prepared_batched.restype = c_int32
    lib.nm_linear_forward_prepared_batched.argtypes = [ctypes.POINTER(ForwardDesc), c_int32, c_void_p]
    lib.nm_prune_scored.restype = c_int32
    lib.nm_prune_scored.argtypes = [c_void_p, c_int64, c_int64, c_int64, c_int32, c_int32, c_void_p, c_void_p]
    lib.nm_i8_workspace_bytes.restype = c_size_t
    lib.nm_i8_workspace_bytes.argtypes = [c_int64, c_int64, c_int32, c_int32, c_int64]
    i8_args = [c_void_p, c_int64, c_int64, c_int64, c_void_p, c_int32, c_int32, c_void_p, c_int64, c_int64,
               ctypes.c_float, c_void_p, c_void_p, c_void_p, c_int64, c_int32, c_void_p, c_size_t, c_void_p]
    lib.nm_linear_forward_i8.restype = c_int32
    lib.nm_linear_forward_i8.argtypes = i8_args
    lib.nm_linear_forward_i8_prepared.restype = c_int32
    lib.nm_linear_forward_i8_prepared.argtypes = i8_args
    lib.nm_i8_prepare.restype = c_int32
    lib.nm_i8_prepare.argtypes = [c_void_p, c_int64, c_int64, c_int64, c_void_p, c_int32, c_int32, c_int64, c_void_p, c_size_t,
                                  c_void_p]
    lib.nm_values_i8_bytes.restype = c_size_t
    lib.nm_values_i8_bytes.argtypes = [c_int64, c_int64, c_int32, c_int32]
    lib.nm_pack_i8.restype = c_int32
    lib.nm_pack_i8.argtypes = [c_void_p, c_int64, c_int64, c_int64, c_int32, c_int32, c_void_p, c_void_p, c_void_p, c_void_p]
    lib.nm_unpack_i8.restype = c_int32
    lib.nm_unpack_i8.argtypes = [c_void_p, c_void_p, c_int64, c_int64, c_int32, c_int32, c_void_p, c_int64, c_void_p]
    i8p_args = [c_void_p, c_void_p, c_int64, c_int64, c_int32, c_int32, c_void_p, c_int64, c_int64, ctypes.c_float,
                c_void_p, c_void_p, c_void_p, c_int64, c_int32, c_void_p, c_size_t, c_void_p]
    lib.nm_linear_forward_i8_packed.restype = c_int32
    lib.nm_linear_forward_i8_packed.argtypes = i8p_args
    lib.nm_linear_forward_i8_packed_prepared.restype = c_int32
    lib.nm_linear_forward_i8_packed_prepared.argtypes = i8p_args
    lib.nm_i8_prepare_packed.restype = c_int32
    lib.nm_i8_prepare_packed.argtypes = [c_void_p, c_void_p, c_int64, c_int64, c_int32, c_int32, c_int64, c_void_p, c_size_t,
                                         c_void_p]
    _LIB = lib
    return lib


def nm_status_string(status: int) -> str:
    return load_library().nm_status_string(status).decode()


def _check(status: int) -> None:
    if status != NM_OK:
        raise NmError(status, nm_status_string(status))


def nm_values_bytes(O: int, K: int, N: int, M: int) -> int:
    return int(load_library().nm_values_bytes(O, K, N, M))


def nm_index_bytes(O: int, K: int, N: int, M: int) -> int:
    return int(load_library().nm_index_bytes(O, K, N, M))


def nm_mask_bytes(O: int, K: int) -> int:
    return int(load_library().nm_mask_bytes(O, K))


def nm_spmm_workspace_bytes(O: int, K: int, N: int, M: int, T: int) -> int:
    return int(load_library().nm_spmm_workspace_bytes(O, K, N, M, T))


# ------------------------------------------------------------------------------------------------
# tensor marshalling
# ------------------------------------------------------------------------------------------------
def _torch():
    import torch
    return torch


def _stream_handle(stream) -> int:
    torch = _torch()
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


def _need(t, dtype, what: str) -> None:
    if not t.is_cuda:
        raise ValueError(f"{what} must be a device tensor")
    if t.dtype != dtype:
        raise ValueError(f"{what} must be {dtype}, got {t.dtype}")


def _rows(t, what: str) -> Tuple[int, int, int]:
    """(rows, cols, leading dimension) of a 2-D tensor whose rows are contiguous."""
    if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
        raise ValueError(f"{what} must be 2-D with unit stride along its rows")
    return int(t.shape[0]), int(t.shape[1]), int(t.stride(0)) if t.shape[0] > 1 else int(t.shape[1])


def _empty_packed(O: int, K: int, N: int, M: int, device):
    torch = _torch()
    vb, ib = nm_values_bytes(O, K, N, M), nm_index_bytes(O, K, N, M)
    if vb == 0:  # illegal level or shape: let the library name the error (it returns before touching a pointer)
        _check(load_library().nm_pack(16, O, K, K, N, M, None, 16, 16, None))
    values = torch.empty((O, vb // (2 * O)), dtype=torch.bfloat16, device=device)
    indices = torch.empty((O, ib // (4 * O)), dtype=torch.int32, device=device)
    return values, indices


def nm_prune(W, N: int, M: int, W_masked=None, stream=None):
    """Mask words [O, ceil(K/32)] (int32) of Eq. (1); optionally writes the pruned weight to W_masked."""
    torch = _torch()
    _need(W, torch.bfloat16, "W")
    O, K, ldw = _rows(W, "W")
    mask = torch.empty((O, (K + 31) // 32), dtype=torch.int32, device=W.device)
    wm_ptr = None
    if W_masked is not None:
        _need(W_masked, torch.bfloat16, "W_masked")
        if _rows(W_masked, "W_masked") != (O, K, ldw):
            raise ValueError("W_masked must have the shape and leading dimension of W")
        wm_ptr = W_masked.data_ptr()
    _check(load_library().nm_prune(W.data_ptr(), O, K, ldw, N, M, mask.data_ptr(), wm_ptr, _stream_handle(stream)))
    return mask


def nm_prune_scored(score, N: int, M: int, stream=None):
    """Mask words [O, ceil(K/32)] (int32) keeping the N largest of every M scores (float32 [O, K])."""
    torch = _torch()
    _need(score, torch.float32, "score")
    O, K, lds = _rows(score, "score")
    mask = torch.empty((O, (K + 31) // 32), dtype=torch.int32, device=score.device)
    _check(load_library().nm_prune_scored(score.data_ptr(), O, K, lds, N, M, mask.data_ptr(), _stream_handle(stream)))
    return mask


def _doubles(xs):
    return (ctypes.c_double * len(xs))(*[float(x) for x in xs])


def _ints(xs):
    return (c_int32 * len(xs))(*[int(x) for x in xs])


def nm_config_cost(layer_macs, levels, fixed_cost: float = 0.0) -> float:
    """F(alpha) = fixed_cost + sum_l layer_macs[l] * N_l / M_l (host only)."""
    L = len(layer_macs)
    c = load_library().nm_config_cost(_doubles(layer_macs), _ints([n for n, _ in levels]), _ints([m for _, m in levels]),
                                      L, float(fixed_cost))
    if c < 0:
        raise ValueError("illegal level or layer cost")
    return float(c)


def nm_sample_config(layer_macs, fixed_cost, choices, probs, edges, uniforms):
    """Two-step sampling (host only): (interval, [choice index per layer], uniforms used); raises NmError with
    status NM_ERR_EXHAUSTED when the uniforms run out."""
    L, S = len(layer_macs), len(choices)
    flat = [float(p) for row in probs for p in row]
    choice = (c_int32 * L)()
    interval, used = c_int32(0), c_int64(0)
    _check(load_library().nm_sample_config(_doubles(layer_macs), L, float(fixed_cost), _ints([n for n, _ in choices]),
                                           _ints([m for _, m in choices]), S, _doubles(flat), _doubles(edges),
                                           len(edges), _doubles(uniforms), len(uniforms), choice,
                                           ctypes.byref(interval), ctypes.byref(used)))
    return int(interval.value), [int(c) for c in choice], int(used.value)


def nm_rank_bytes(O: int, K: int) -> int:
    return int(load_library().nm_rank_bytes(O, K))


def nm_rank(W, M: int, stream=None):
    """Ranks (uint8 [O, K/2], two 4-bit ranks per byte) of the weights inside their groups of M."""
    torch = _torch()
    _need(W, torch.bfloat16, "W")
    O, K, ldw = _rows(W, "W")
    rank = torch.empty((O, K // 2), dtype=torch.uint8, device=W.device)
    _check(load_library().nm_rank(W.data_ptr(), O, K, ldw, M, rank.data_ptr(), _stream_handle(stream)))
    return rank


def nm_rank_batched(layers: Sequence[Tuple[object, int]], stream=None, out=None):
    """One launch for many (W, M); returns the rank tensors."""
    torch = _torch()
    descs = (RankDesc * len(layers))()
    outs = []
    for i, (W, M) in enumerate(layers):
        _need(W, torch.bfloat16, "W")
        if not W.is_contiguous():
            raise ValueError("nm_rank_batched needs contiguous weights")
        O, K = int(W.shape[0]), int(W.shape[1])
        rank = out[i] if out is not None else torch.empty((O, K // 2), dtype=torch.uint8, device=W.device)
        outs.append(rank)
        descs[i] = RankDesc(W.data_ptr(), rank.data_ptr(), O, K, M, 0)
    _check(load_library().nm_rank_batched(descs, len(layers), _stream_handle(stream)))
    return outs


def _need_rank(rank, O: int, K: int) -> None:
    torch = _torch()
    _need(rank, torch.uint8, "rank")
    if tuple(rank.shape) != (O, K // 2) or not rank.is_contiguous():
        raise ValueError("rank must be contiguous [O, K/2]")


def nm_rank_mask(rank, K: int, N: int, M: int, stream=None):
    """Mask words [O, ceil(K/32)] (int32) of level N:M from stored ranks: bit = rank < N."""
    torch = _torch()
    O = int(rank.shape[0])
    _need_rank(rank, O, K)
    mask = torch.empty((O, (K + 31) // 32), dtype=torch.int32, device=rank.device)
    _check(load_library().nm_rank_mask(rank.data_ptr(), O, K, N, M, mask.data_ptr(), _stream_handle(stream)))
    return mask


def nm_pack_ranked(W, rank, N: int, M: int, stream=None):
    """nm_pack with the selection read from stored ranks."""
    torch = _torch()
    _need(W, torch.bfloat16, "W")
    O, K, ldw = _rows(W, "W")
    _need_rank(rank, O, K)
    values, indices = _empty_packed(O, K, N, M, W.device)
    _check(load_library().nm_pack_ranked(W.data_ptr(), rank.data_ptr(), O, K, ldw, N, M, values.data_ptr(),
                                         indices.data_ptr(), _stream_handle(stream)))
    return values, indices


def nm_pack_ranked_batched(layers: Sequence[Tuple[object, object, int, int]], stream=None, out=None):
    """One launch for many (W, rank, N, M); returns [(values, indices), ...]."""
    torch = _torch()
    descs = (PackRankedDesc * len(layers))()
    outs: List[Tuple[object, object]] = []
    for i, (W, rank, N, M) in enumerate(layers):
        _need(W, torch.bfloat16, "W")
        if not W.is_contiguous():
            raise ValueError("nm_pack_ranked_batched needs contiguous weights")
        O, K = int(W.shape[0]), int(W.shape[1])
        _need_rank(rank, O, K)
        values, indices = out[i] if out is not None else _empty_packed(O, K, N, M, W.device)
        outs.append((values, indices))
        descs[i] = PackRankedDesc(W.data_ptr(), rank.data_ptr(), values.data_ptr(), indices.data_ptr(), O, K, N, M)
    _check(load_library().nm_pack_ranked_batched(descs, len(layers), _stream_handle(stream)))
    return outs


def nm_pack(W, N: int, M: int, mask=None, stream=None):
    """(values bf16 [O, K*N/M], indices int32 [O, words]) of W at level N:M."""
    torch = _torch()
    _need(W, torch.bfloat16, "W")
    O, K, ldw = _rows(W, "W")
    values, indices = _empty_packed(O, K, N, M, W.device)
    mask_ptr = None
    if mask is not None:
        _need(mask, torch.int32, "mask")
        if tuple(mask.shape) != (O, (K + 31) // 32) or not mask.is_contiguous():
            raise ValueError("mask must be contiguous [O, ceil(K/32)]")
        mask_ptr = mask.data_ptr()
    _check(load_library().nm_pack(W.data_ptr(), O, K, ldw, N, M, mask_ptr, values.data_ptr(), indices.data_ptr(),
                                  _stream_handle(stream)))
    return values, indices


def nm_pack_batched(layers: Sequence[Tuple[object, int, int]], stream=None, out=None):
    """One launch for many (W, N, M); returns [(values, indices), ...]."""
    torch = _torch()
    descs = (PackDesc * len(layers))()
    outs: List[Tuple[object, object]] = []
    for i, (W, N, M) in enumerate(layers):
        _need(W, torch.bfloat16, "W")
        if not W.is_contiguous():
            raise ValueError("nm_pack_batched needs contiguous weights")
        O, K = int(W.shape[0]), int(W.shape[1])
        values, indices = out[i] if out is not None else _empty_packed(O, K, N, M, W.device)
        outs.append((values, indices))
        descs[i] = PackDesc(W.data_ptr(), values.data_ptr(), indices.data_ptr(), O, K, N, M)
    _check(load_library().nm_pack_batched(descs, len(layers), _stream_handle(stream)))
    return outs


def nm_pack_prepare_batched(layers: Sequence[Tuple[object, int, int, int]], stream=None, out=None, workspaces=None):
    """nm_pack + nm_spmm_prepare for many (W, N, M, T); returns ([(values, indices), ...], [workspace or None, ...])."""
    torch = _torch()
    descs = (LayerDesc * len(layers))()
    outs: List[Tuple[object, object]] = []
    wss: List[object] = []
    for i, (W, N, M, T) in enumerate(layers):
        _need(W, torch.bfloat16, "W")
        if not W.is_contiguous():
            raise ValueError("nm_pack_prepare_batched needs contiguous weights")
        O, K = int(W.shape[0]), int(W.shape[1])
        values, indices = out[i] if out is not None else _empty_packed(O, K, N, M, W.device)
        need = nm_spmm_workspace_bytes(O, K, N, M, T)
        ws = workspaces[i] if workspaces is not None else (
            torch.empty((need,), dtype=torch.uint8, device=W.device) if need else None)
        outs.append((values, indices))
        wss.append(ws)
        descs[i] = LayerDesc(W.data_ptr(), values.data_ptr(), indices.data_ptr(), O, K, N, M, T,
                             ws.data_ptr() if ws is not None else None,
                             ws.numel() * ws.element_size() if ws is not None else 0)
    _check(load_library().nm_pack_prepare_batched(descs, len(layers), _stream_handle(stream)))
    return outs, wss


def nm_unpack(values, indices, K: int, N: int, M: int, stream=None):
    torch = _torch()
    _need(values, torch.bfloat16, "values")
    _need(indices, torch.int32, "indices")
    O = int(values.shape[0])
    Wd = torch.empty((O, K), dtype=torch.bfloat16, device=values.device)
    _check(load_library().nm_unpack(values.data_ptr(), indices.data_ptr(), O, K, N, M, Wd.data_ptr(), K,
                                    _stream_handle(stream)))
    return Wd


def nm_mask_check(mask, K: int, N: int, M: int, stream=None) -> int:
    """Number of groups of `mask` that do not hold exactly N ones (synchronises to read it)."""
    torch = _torch()
    _need(mask, torch.int32, "mask")
    O = int(mask.shape[0])
    bad = torch.empty((1,), dtype=torch.int32, device=mask.device)
    _check(load_library().nm_mask_check(mask.data_ptr(), O, K, N, M, bad.data_ptr(), _stream_handle(stream)))
    return int(bad.item()) & 0xFFFFFFFF


def bf16_tensor(bits, device="cuda"):
    """numpy uint16 bf16 bit patterns -> torch.bfloat16 tensor on `device` (a copy of the bits)."""
    import numpy as np
    torch = _torch()
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device).view(torch.bfloat16)


def bf16_bits(t):
    """torch.bfloat16 tensor -> numpy uint16 bit patterns on the host."""
    import numpy as np
    torch = _torch()
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


_WORKSPACES = {}


def _workspace(nbytes: int, device, stream=None):
    """A cached scratch tensor per (device, stream), grown on demand (allocated by torch, not by the library).
    Calls on different streams may overlap, and concurrent calls need distinct workspaces, hence one per
    stream.  A tensor that is replaced may still be read by kernels on its stream: it is marked as in use on
    that stream so that the allocator does not hand its memory out before they finish."""
    torch = _torch()
    index = device.index if device.index is not None else torch.cuda.current_device()
    handle = _stream_handle(stream)
    key = (device.type, index, handle)
    ws = _WORKSPACES.get(key)
    if ws is None or ws.numel() < nbytes:
        if ws is not None and handle:
            ws.record_stream(torch.cuda.ExternalStream(handle, device=index))
        ws = torch.empty((max(nbytes, 1 << 20),), dtype=torch.uint8, device=device)
        _WORKSPACES[key] = ws
    return ws


def nm_spmm_prepare(values, indices, K: int, N: int, M: int, T: int, workspace=None, stream=None):
    """Fill (and return) the workspace nm_linear_forward_prepared reads; None if the level needs none."""
    torch = _torch()
    _need(values, torch.bfloat16, "values")
    _need(indices, torch.int32, "indices")
    O = int(values.shape[0])
    need = nm_spmm_workspace_bytes(O, K, N, M, T)
    if workspace is None and need:
        workspace = torch.empty((need,), dtype=torch.uint8, device=values.device)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(load_library().nm_spmm_prepare(values.data_ptr(), indices.data_ptr(), O, K, N, M, T, ws_ptr, ws_bytes,
                                          _stream_handle(stream)))
    return workspace


def nm_linear_forward_prepared(values, indices, K: int, N: int, M: int, X, workspace, bias=None, out_dtype=None,
                               out=None, stream=None):
    """The product alone, from a workspace filled by nm_spmm_prepare."""
    return nm_linear_forward(values, indices, K, N, M, X, bias, out_dtype, out, workspace, stream, _prepared=True)


def nm_linear_forward(values, indices, K: int, N: int, M: int, X, bias=None, out_dtype=None, out=None,
                      workspace=None, stream=None, _prepared=False, from_packed=False):
    """Y = X * W_s^T (+ bias) from the packed weight; Y is float32 (default) or bfloat16 [T, O].
    from_packed: hand the library no workspace, so that a product of up to 208 tokens runs straight from the packed
    format (the library reports a missing workspace for shapes that path does not take)."""
    torch = _torch()
    _need(values, torch.bfloat16, "values")
    _need(indices, torch.int32, "indices")
    _need(X, torch.bfloat16, "X")
    O = int(values.shape[0])
    T, KX, ldx = _rows(X, "X")
    if KX != K:
        raise ValueError("X must be [T, K]")
    if not values.is_contiguous() or not indices.is_contiguous():
        raise ValueError("packed tensors must be contiguous")
    if out is not None:
        out_dtype = out.dtype
    out_dtype = out_dtype or torch.float32
    if out_dtype not in (torch.float32, torch.bfloat16):
        raise ValueError("out dtype must be float32 or bfloat16")
    if out is None:
        out = torch.empty((T, O), dtype=out_dtype, device=X.device)
    TY, OY, ldy = _rows(out, "out")
    if (TY, OY) != (T, O):
        raise ValueError("out must be [T, O]")
    need = 0 if from_packed else nm_spmm_workspace_bytes(O, K, N, M, T)
    if workspace is None and need:
        if _prepared:
            raise ValueError("a prepared call needs the workspace nm_spmm_prepare filled")
        workspace = _workspace(need, X.device, stream)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    bias_ptr = None
    if bias is not None:
        _need(bias, torch.float32, "bias")
        if bias.numel() != O or not bias.is_contiguous():
            raise ValueError("bias must be contiguous [O]")
        bias_ptr = bias.data_ptr()
    code = NM_OUT_F32 if out_dtype == torch.float32 else NM_OUT_BF16
    lib = load_library()
    if _prepared:
        st = lib.nm_linear_forward_prepared(values.data_ptr(), indices.data_ptr(), O, K, N, M, X.data_ptr(), T, ldx,
                                            bias_ptr, out.data_ptr(), ldy, code, ws_ptr, ws_bytes,
                                            _stream_handle(stream))
    elif bias_ptr is None:
        st = lib.nm_spmm(values.data_ptr(), indices.data_ptr(), O, K, N, M, X.data_ptr(), T, ldx, out.data_ptr(), ldy,
                         code, ws_ptr, ws_bytes, _stream_handle(stream))
    else:
        st = lib.nm_linear_forward(values.data_ptr(), indices.data_ptr(), O, K, N, M, X.data_ptr(), T, ldx, bias_ptr,
                                   out.data_ptr(), ldy, code, ws_ptr, ws_bytes, _stream_handle(stream))
    _check(st)
    return out


def nm_static_scratch_bytes() -> int:
    return int(load_library().nm_static_scratch_bytes())


def nm_linear_forward_static(values, indices, K: int, N: int, M: int, X, bias=None, out_dtype=None, out=None,
                             stream=None):
    """nm_linear_forward on the library's own fixed scratch: the call itself allocates nothing (pass `out`)."""
    torch = _torch()
    _need(values, torch.bfloat16, "values")
    _need(indices, torch.int32, "indices")
    _need(X, torch.bfloat16, "X")
    if not values.is_contiguous() or not indices.is_contiguous():
        raise ValueError("packed tensors must be contiguous")
    O = int(values.shape[0])
    T, KX, ldx = _rows(X, "X")
    if KX != K:
        raise ValueError("X must be [T, K]")
    out, ldy, code = _out_matrix(out, out_dtype, T, O, X.device, "out")
    bias_ptr = None
    if bias is not None:
        _need(bias, torch.float32, "bias")
        if bias.numel() != O or not bias.is_contiguous():
            raise ValueError("bias must be contiguous [O]")
        bias_ptr = bias.data_ptr()
    _check(load_library().nm_linear_forward_static(values.data_ptr(), indices.data_ptr(), O, K, N, M, X.data_ptr(), T,
                                                   ldx, bias_ptr, out.data_ptr(), ldy, code, _stream_handle(stream)))
    return out


def nm_probe_matrix_rate(kind: int, iters: int, sink=None, stream=None):
    """Launch the matrix-instruction loop (kind 0: 2:4 sparse bf16, 1: dense bf16); returns (sink, operations)."""
    torch = _torch()
    lib = load_library()
    if sink is None:
        sink = torch.empty((lib.nm_probe_sink_bytes(),), dtype=torch.uint8, device="cuda")
    ops = c_int64(0)
    _check(lib.nm_probe_matrix_rate(kind, iters, sink.data_ptr(), ctypes.byref(ops), _stream_handle(stream)))
    return sink, int(ops.value)


def nm_probe_copy(src, dst, stream=None):
    """dst = src with the library's plain streaming copy kernel (equal-sized contiguous device tensors)."""
    nbytes = src.numel() * src.element_size()
    if not (src.is_contiguous() and dst.is_contiguous()) or dst.numel() * dst.element_size() != nbytes:
        raise ValueError("src and dst must be contiguous and of equal size")
    _check(load_library().nm_probe_copy(src.data_ptr(), dst.data_ptr(), nbytes, _stream_handle(stream)))
    return dst


def _out_matrix(out, out_dtype, rows: int, cols: int, device, name: str):
    torch = _torch()
    if out is not None:
        out_dtype = out.dtype
    out_dtype = out_dtype or torch.float32
    if out_dtype not in (torch.float32, torch.bfloat16):
        raise ValueError("out dtype must be float32 or bfloat16")
    if out is None:
        out = torch.empty((rows, cols), dtype=out_dtype, device=device)
    r, c, ld = _rows(out, name)
    if (r, c) != (rows, cols):
        raise ValueError(f"{name} must be [{rows}, {cols}]")
    return out, ld, (NM_OUT_F32 if out_dtype == torch.float32 else NM_OUT_BF16)


def nm_backward_input_workspace_bytes(O: int, K: int, T: int) -> int:
    return int(load_library().nm_backward_input_workspace_bytes(O, K, T))


def nm_linear_backward_input(Ws, dY, out_dtype=None, out=None, workspace=None, stream=None):
    """dX = dY * Ws for the masked dense weight Ws [O, K] and dY [T, O]; float32 (default) or bfloat16 [T, K]."""
    torch = _torch()
    _need(Ws, torch.bfloat16, "Ws")
    _need(dY, torch.bfloat16, "dY")
    O, K, ldw = _rows(Ws, "Ws")
    T, OY, ldy = _rows(dY, "dY")
    if OY != O:
        raise ValueError("dY must be [T, O]")
    out, ldx, code = _out_matrix(out, out_dtype, T, K, dY.device, "dX")
    need = nm_backward_input_workspace_bytes(O, K, T)
    if workspace is None and need:
        workspace = _workspace(need, dY.device, stream)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(load_library().nm_linear_backward_input(Ws.data_ptr(), O, K, ldw, dY.data_ptr(), T, ldy, out.data_ptr(), ldx,
                                                   code, ws_ptr, ws_bytes, _stream_handle(stream)))
    return out


def nm_backward_weight_workspace_bytes(O: int, K: int, T: int) -> int:
    return int(load_library().nm_backward_weight_workspace_bytes(O, K, T))


def nm_linear_backward_weight(dY, X, mask=None, out_dtype=None, out=None, workspace=None, stream=None):
    """dW = dY^T * X, with pruned positions zeroed when the step's mask words are given; [O, K]."""
    torch = _torch()
    _need(dY, torch.bfloat16, "dY")
    _need(X, torch.bfloat16, "X")
    T, O, ldy = _rows(dY, "dY")
    TX, K, ldx = _rows(X, "X")
    if TX != T:
        raise ValueError("dY and X must have the same number of rows")
    mask_ptr = None
    if mask is not None:
        _need(mask, torch.int32, "mask")
        if tuple(mask.shape) != (O, (K + 31) // 32) or not mask.is_contiguous():
            raise ValueError("mask must be contiguous [O, ceil(K/32)] words")
        mask_ptr = mask.data_ptr()
    out, lddw, code = _out_matrix(out, out_dtype, O, K, dY.device, "dW")
    need = nm_backward_weight_workspace_bytes(O, K, T)
    if workspace is None and need:
        workspace = _workspace(need, dY.device, stream)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(load_library().nm_linear_backward_weight(dY.data_ptr(), T, O, ldy, X.data_ptr(), K, ldx, mask_ptr,
                                                    out.data_ptr(), lddw, code, ws_ptr, ws_bytes, _stream_handle(stream)))
    return out


def forward_descs(layers):
    """The descriptor array of nm_linear_forward_prepared_batched for a list of
    (values, indices, K, N, M, X, workspace, bias or None, out); build it once when the buffers stay put."""
    torch = _torch()
    descs = (ForwardDesc * len(layers))()
    for n, (values, indices, K, N, M, X, workspace, bias, out) in enumerate(layers):
        _need(values, torch.bfloat16, "values")
        _need(indices, torch.int32, "indices")
        _need(X, torch.bfloat16, "X")
        if not values.is_contiguous() or not indices.is_contiguous():
            raise ValueError("packed tensors must be contiguous")
        O = int(values.shape[0])
        T, KX, ldx = _rows(X, "X")
        if KX != K:
            raise ValueError("X must be [T, K]")
        if out.dtype not in (torch.float32, torch.bfloat16):
            raise ValueError("out dtype must be float32 or bfloat16")
        TY, OY, ldy = _rows(out, "out")
        if (TY, OY) != (T, O):
            raise ValueError("out must be [T, O]")
        bias_ptr = None
        if bias is not None:
            _need(bias, torch.float32, "bias")
            if bias.numel() != O or not bias.is_contiguous():
                raise ValueError("bias must be contiguous [O]")
            bias_ptr = bias.data_ptr()
        descs[n] = ForwardDesc(values.data_ptr(), indices.data_ptr(), O, K, N, M, X.data_ptr(), T, ldx, bias_ptr,
                               out.data_ptr(), ldy, NM_OUT_F32 if out.dtype == torch.float32 else NM_OUT_BF16, 0,
                               workspace.data_ptr() if workspace is not None else None,
                               workspace.numel() * workspace.element_size() if workspace is not None else 0)
    return descs


def nm_linear_forward_prepared_batched(layers, stream=None):
    """The products of many prepared layers in as few launches as their shapes allow; `layers` is a list of
    (values, indices, K, N, M, X, workspace, bias or None, out) or an array made by forward_descs."""
    descs = layers if isinstance(layers, ctypes.Array) else forward_descs(layers)
    _check(load_library().nm_linear_forward_prepared_batched(descs, len(descs), _stream_handle(stream)))


def nm_i8_workspace_bytes(O: int, K: int, N: int, M: int, T: int) -> int:
    return int(load_library().nm_i8_workspace_bytes(O, K, N, M, T))


def _i8_weight(Wq, mask):
    torch = _torch()
    _need(Wq, torch.int8, "Wq")
    _need(mask, torch.int32, "mask")
    O, K, ldw = _rows(Wq, "Wq")
    if tuple(mask.shape) != (O, (K + 31) // 32) or not mask.is_contiguous():
        raise ValueError("mask must be contiguous [O, ceil(K/32)] words")
    return O, K, ldw


def nm_i8_prepare(Wq, mask, N: int, M: int, T: int, workspace=None, stream=None):
    """Compress the int8 weight into the operand order of the product at T tokens; returns the workspace (None if
    none is needed)."""
    torch = _torch()
    O, K, ldw = _i8_weight(Wq, mask)
    need = nm_i8_workspace_bytes(O, K, N, M, T)
    if workspace is None and need:
        workspace = torch.empty((need,), dtype=torch.uint8, device=Wq.device)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(load_library().nm_i8_prepare(Wq.data_ptr(), O, K, ldw, mask.data_ptr(), N, M, T, ws_ptr, ws_bytes,
                                        _stream_handle(stream)))
    return workspace


def nm_linear_forward_i8(Wq, mask, N: int, M: int, Xq, x_scale: float = 1.0, w_scale=None, bias=None, out_dtype=None,
                         out=None, workspace=None, stream=None, _prepared=False):
    """Y = x_scale * w_scale[o] * (Xq . (Wq (.) m)^T) + bias from int8 operands: float32 (default), bfloat16, or
    the exact int32 sums (out dtype int32)."""
    torch = _torch()
    O, K, ldw = _i8_weight(Wq, mask)
    _need(Xq, torch.int8, "Xq")
    T, KX, ldx = _rows(Xq, "Xq")
    if KX != K:
        raise ValueError("Xq must be [T, K]")
    if out is not None:
        out_dtype = out.dtype
    out_dtype = out_dtype or torch.float32
    codes = {torch.float32: NM_OUT_F32, torch.bfloat16: NM_OUT_BF16, torch.int32: NM_OUT_I32}
    if out_dtype not in codes:
        raise ValueError("out dtype must be float32, bfloat16 or int32")
    if out is None:
        out = torch.empty((T, O), dtype=out_dtype, device=Xq.device)
    TY, OY, ldy = _rows(out, "out")
    if (TY, OY) != (T, O):
        raise ValueError("out must be [T, O]")
    ptrs = []
    for t, name in ((w_scale, "w_scale"), (bias, "bias")):
        if t is None:
            ptrs.append(None)
            continue
        _need(t, torch.float32, name)
        if t.numel() != O or not t.is_contiguous():
            raise ValueError(f"{name} must be contiguous [O]")
        ptrs.append(t.data_ptr())
    need = nm_i8_workspace_bytes(O, K, N, M, T)
    if workspace is None and need:
        if _prepared:
            raise ValueError("a prepared call needs the workspace nm_i8_prepare filled")
        workspace = _workspace(need, Xq.device, stream)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    lib = load_library()
    fn = lib.nm_linear_forward_i8_prepared if _prepared else lib.nm_linear_forward_i8
    _check(fn(Wq.data_ptr(), O, K, ldw, mask.data_ptr(), N, M, Xq.data_ptr(), T, ldx, float(x_scale), ptrs[0], ptrs[1],
              out.data_ptr(), ldy, codes[out_dtype], ws_ptr, ws_bytes, _stream_handle(stream)))
    return out


def nm_linear_forward_i8_prepared(Wq, mask, N: int, M: int, Xq, workspace, x_scale: float = 1.0, w_scale=None, bias=None,
                                  out_dtype=None, out=None, stream=None):
    """The product alone, from a workspace filled by nm_i8_prepare."""
    return nm_linear_forward_i8(Wq, mask, N, M, Xq, x_scale, w_scale, bias, out_dtype, out, workspace, stream,
                                _prepared=True)


def nm_pack_i8(Wq, mask, N: int, M: int, stream=None):
    """Compressed form of the int8 weight under `mask`: (values int8 [O, K*N/M], indices int32 words)."""
    torch = _torch()
    O, K, ldw = _i8_weight(Wq, mask)
    lib = load_library()
    values = torch.empty((O, K // M * N), dtype=torch.int8, device=Wq.device)
    indices = torch.empty((O, lib.nm_index_bytes(O, K, N, M) // (4 * O)), dtype=torch.int32, device=Wq.device)
    _check(lib.nm_pack_i8(Wq.data_ptr(), O, K, ldw, N, M, mask.data_ptr(), values.data_ptr(), indices.data_ptr(),
                          _stream_handle(stream)))
    return values, indices


def _i8_packed(values, indices):
    torch = _torch()
    _need(values, torch.int8, "values")
    _need(indices, torch.int32, "indices")
    if not values.is_contiguous() or not indices.is_contiguous():
        raise ValueError("packed tensors must be contiguous")
    return int(values.shape[0])


def nm_unpack_i8(values, indices, K: int, N: int, M: int, stream=None):
    torch = _torch()
    O = _i8_packed(values, indices)
    out = torch.empty((O, K), dtype=torch.int8, device=values.device)
    _check(load_library().nm_unpack_i8(values.data_ptr(), indices.data_ptr(), O, K, N, M, out.data_ptr(), K,
                                       _stream_handle(stream)))
    return out


def nm_i8_prepare_packed(values, indices, K: int, N: int, M: int, T: int, workspace=None, stream=None):
    """nm_i8_prepare from the compressed form: fills (and returns) the same workspace."""
    torch = _torch()
    O = _i8_packed(values, indices)
    need = nm_i8_workspace_bytes(O, K, N, M, T)
    if workspace is None and need:
        workspace = torch.empty((need,), dtype=torch.uint8, device=values.device)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(load_library().nm_i8_prepare_packed(values.data_ptr(), indices.data_ptr(), O, K, N, M, T, ws_ptr, ws_bytes,
                                               _stream_handle(stream)))
    return workspace


def nm_linear_forward_i8_packed(values, indices, K: int, N: int, M: int, Xq, x_scale: float = 1.0, w_scale=None, bias=None,
                                out_dtype=None, out=None, workspace=None, stream=None, _prepared=False):
    """nm_linear_forward_i8 with the weight in its compressed form."""
    torch = _torch()
    O = _i8_packed(values, indices)
    _need(Xq, torch.int8, "Xq")
    T, KX, ldx = _rows(Xq, "Xq")
    if KX != K:
        raise ValueError("Xq must be [T, K]")
    if out is not None:
        out_dtype = out.dtype
    out_dtype = out_dtype or torch.float32
    codes = {torch.float32: NM_OUT_F32, torch.bfloat16: NM_OUT_BF16, torch.int32: NM_OUT_I32}
    if out_dtype not in codes:
        raise ValueError("out dtype must be float32, bfloat16 or int32")
    if out is None:
        out = torch.empty((T, O), dtype=out_dtype, device=Xq.device)
    TY, OY, ldy = _rows(out, "out")
    if (TY, OY) != (T, O):
        raise ValueError("out must be [T, O]")
    ptrs = []
    for t, name in ((w_scale, "w_scale"), (bias, "bias")):
        if t is None:
            ptrs.append(None)
            continue
        _need(t, torch.float32, name)
        if t.numel() != O or not t.is_contiguous():
            raise ValueError(f"{name} must be contiguous [O]")
        ptrs.append(t.data_ptr())
    need = nm_i8_workspace_bytes(O, K, N, M, T)
    if workspace is None and need:
        if _prepared:
            raise ValueError("a prepared call needs the workspace nm_i8_prepare_packed filled")
        workspace = _workspace(need, Xq.device, stream)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    lib = load_library()
    fn = lib.nm_linear_forward_i8_packed_prepared if _prepared else lib.nm_linear_forward_i8_packed
    _check(fn(values.data_ptr(), indices.data_ptr(), O, K, N, M, Xq.data_ptr(), T, ldx, float(x_scale), ptrs[0], ptrs[1],
              out.data_ptr(), ldy, codes[out_dtype], ws_ptr, ws_bytes, _stream_handle(stream)))
    return out


def nm_linear_forward_i8_packed_prepared(values, indices, K: int, N: int, M: int, Xq, workspace, x_scale: float = 1.0,
                                         w_scale=None, bias=None, out_dtype=None, out=None, stream=None):
    return nm_linear_forward_i8_packed(values, indices, K, N, M, Xq, x_scale, w_scale, bias, out_dtype, out, workspace,
                                       stream, _prepared=True)


def nm_spmm(values, indices, K: int, N: int, M: int, X, out_dtype=None, out=None, workspace=None, stream=None,
            from_packed=False):
    return nm_linear_forward(values, indices, K, N, M, X, None, out_dtype, out, workspace, stream,
                             from_packed=from_packed)
