"""Seeded synthetic inputs for the N:M-sparse linear layer.

This module only draws numbers and names shapes.  It holds none of the method's
arithmetic (no saliency, no selection, no packing, no product): both the HIP
path and the CPU checker are fed from here so that they see identical bits.

The layers are the four linear modules of a transformer block (qkv, proj, fc1,
fc2; Section 3, "Problem Formulation", and Section 3.1), with the layer sizes
of DeiT-S/B and of a Swin-B-shaped hierarchy.  Trained weights and ImageNet
images are replaced by Gaussians: activations ~ N(0, 1), weights ~ N(0, 0.02),
both rounded to bfloat16 (round to nearest, ties to even) and carried as raw
uint16 bit patterns.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Iterator, List, Sequence, Tuple

import numpy as np

Level = Tuple[int, int]

# Levels named by the workloads (N, M).
LEVELS_N4: Tuple[Level, ...] = ((1, 4), (2, 4))
LEVELS_5: Tuple[Level, ...] = ((1, 4), (2, 4), (1, 8), (2, 8), (4, 8))
LEVELS_7: Tuple[Level, ...] = ((1, 4), (2, 4), (1, 8), (2, 8), (4, 8), (1, 16), (4, 16))
LEVELS_SWIN: Tuple[Level, ...] = ((2, 4), (1, 8), (2, 8), (2, 16))
LEVELS_ALL: Tuple[Level, ...] = (
    (1, 4), (2, 4), (3, 4), (4, 4),
    (1, 8), (2, 8), (3, 8), (4, 8), (8, 8),
    (1, 16), (2, 16), (4, 16), (16, 16),
)


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit pattern (uint16), round to nearest even.

    Inputs here are finite Gaussians; NaN payloads are not preserved.
    """
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return ((u >> 16) & 0xFFFF).astype(np.uint16)


@dataclass(frozen=True)
class Layer:
    name: str
    T: int  # tokens (batch x tokens per image)
    K: int  # in features (reduction dimension, the N:M groups run along it)
    O: int  # out features
    N: int
    M: int

    @property
    def dense_flops(self) -> float:
        return 2.0 * self.T * self.O * self.K

    @property
    def useful_flops(self) -> float:
        return self.dense_flops * self.N / self.M


def block_shapes(C: int) -> List[Tuple[str, int, int]]:
    """(name, K, O) of the four linear modules of a block of width C."""
    return [("qkv", C, 3 * C), ("proj", C, C), ("fc1", C, 4 * C), ("fc2", 4 * C, C)]


def draw_levels(seed: int, levels: Sequence[Level], count: int) -> List[Level]:
    """Layer-wise level assignment: one uniform draw per layer from `levels`."""
    rng = np.random.default_rng(seed)
    picks = rng.integers(0, len(levels), size=count)
    return [levels[int(i)] for i in picks]


def single_2to4(seed: int = 0) -> List[Layer]:
    """One 2:4 linear, X 197x384, W 384x384."""
    return [Layer("proj", 197, 384, 384, 2, 4)]


def deit_b_block(batch: int = 64, seed: int = 0, levels: Sequence[Level] = LEVELS_5) -> List[Layer]:
    """The four linears of one DeiT-B block at `batch` images of 197 tokens."""
    T = batch * 197
    lv = draw_levels(seed, levels, 4)
    return [Layer(n, T, K, O, N, M) for (n, K, O), (N, M) in zip(block_shapes(768), lv)]


def deit_b_stack(batch: int = 256, seed: int = 0, levels: Sequence[Level] = LEVELS_7,
                 blocks: int = 12) -> List[Layer]:
    """All 4 x `blocks` linears of DeiT-B, block-major (qkv, proj, fc1, fc2)."""
    T = batch * 197
    lv = draw_levels(seed, levels, 4 * blocks)
    out = []
    for b in range(blocks):
        for i, (n, K, O) in enumerate(block_shapes(768)):
            N, M = lv[4 * b + i]
            out.append(Layer(f"blk{b}.{n}", T, K, O, N, M))
    return out


def swin_b_stages(batch: int = 64, seed: int = 0, levels: Sequence[Level] = LEVELS_SWIN) -> List[Layer]:
    """One block per stage of a Swin-B-shaped hierarchy; level drawn per stage."""
    dims = (128, 256, 512, 1024)
    toks = (3136, 784, 196, 49)
    lv = draw_levels(seed, levels, 4)
    out = []
    for s, (C, t) in enumerate(zip(dims, toks)):
        N, M = lv[s]
        for n, K, O in block_shapes(C):
            out.append(Layer(f"stage{s}.{n}", batch * t, K, O, N, M))
    return out


def small_batch() -> List[Layer]:
    """Batch 1 (197 tokens) DeiT-B fc1/fc2 at 1:8 and 2:4."""
    out = []
    for (N, M) in ((1, 8), (2, 4)):
        out.append(Layer(f"fc1.{N}:{M}", 197, 768, 3072, N, M))
        out.append(Layer(f"fc2.{N}:{M}", 197, 3072, 768, N, M))
    return out


def draw_activations(rng: np.random.Generator, T: int, K: int) -> np.ndarray:
    """X ~ N(0,1) as bf16 bits, shape [T, K]."""
    return f32_to_bf16_bits(rng.standard_normal((T, K), dtype=np.float32))


def draw_weights(rng: np.random.Generator, O: int, K: int) -> np.ndarray:
    """W ~ N(0, 0.02) as bf16 bits, shape [O, K]."""
    w = rng.standard_normal((O, K), dtype=np.float32)
    w *= np.float32(0.02)
    return f32_to_bf16_bits(w)


def draw_int8(rng: np.random.Generator, rows: int, cols: int, spread: float = 40.0) -> np.ndarray:
    """Quantised operand: round(N(0, spread)) clipped to [-127, 127], int8 [rows, cols]."""
    v = np.rint(rng.standard_normal((rows, cols), dtype=np.float32) * np.float32(spread))
    return np.clip(v, -127, 127).astype(np.int8)


def draw_layers(layers: Sequence[Layer], seed: int = 0) -> Iterator[Tuple[Layer, np.ndarray, np.ndarray]]:
    """Yield (layer, X bits, W bits) in layer order from one generator: X then W per layer."""
    rng = np.random.default_rng(seed)
    for L in layers:
        X = draw_activations(rng, L.T, L.K)
        W = draw_weights(rng, L.O, L.K)
        yield L, X, W


def tie_heavy_weights(rng: np.random.Generator, O: int, K: int, distinct: int = 5) -> np.ndarray:
    """Weights drawn from a handful of magnitudes with random signs (many equal saliencies),
    with some +0/-0 entries mixed in.  bf16 bits, shape [O, K]."""
    mags = np.array([0.0, 0.25, 0.5, 1.0, 1.5, 2.0, 3.0, 0.125], dtype=np.float32)[:max(2, distinct)]
    w = mags[rng.integers(0, len(mags), size=(O, K))]
    sign = rng.integers(0, 2, size=(O, K)).astype(np.float32) * 2 - 1
    return f32_to_bf16_bits(w * sign)
