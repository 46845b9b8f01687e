"""Helpers shared by the GPU tests: host bit patterns <-> device tensors, acceptance checks."""
import numpy as np
import torch

from oracle import nm_oracle as orc


from paper_2409_09708_amd.binding import bf16_bits as host_bits
from paper_2409_09708_amd.binding import bf16_tensor as dev_bf16


def host_words(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().cpu().numpy().view(np.uint32)


def dev_words(w: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(w).view(np.int32)).cuda()


def host_output(y: torch.Tensor) -> np.ndarray:
    """Y as float64, whatever its storage type."""
    if y.dtype == torch.bfloat16:
        return orc.bf16_bits_to_f64(host_bits(y))
    return y.cpu().numpy().astype(np.float64)


def check_output(Y: np.ndarray, Yref: np.ndarray, B: np.ndarray, terms: int, fp32_out: bool, what=""):
    """Acceptance: every element within 1e-2 * sum_k |x_k w_k|, relative Frobenius error <= 5e-3.
    For fp32 outputs also the rounding bound of an fp32 sum of `terms` exact products in any order,
    (terms + 2) * 2^-24 * B, which is far tighter and catches a single dropped or doubled product."""
    err = np.abs(Y - Yref)
    assert np.all(np.isfinite(Y)), what
    assert np.all(err <= 1e-2 * B + 1e-30), (what, float((err / (B + 1e-30)).max()))
    fro = np.linalg.norm(Y - Yref) / max(np.linalg.norm(Yref), 1e-30)
    assert fro <= 5e-3, (what, fro)
    if fp32_out:
        tight = (terms + 2) * 2.0 ** -24 * B + 1e-30
        assert np.all(err <= tight), (what, float((err / tight).max()))
    return float((err / (B + 1e-30)).max()), float(fro)
