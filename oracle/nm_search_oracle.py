"""CPU checker for the configuration cost and the two-step sampler.  TEST INFRASTRUCTURE ONLY.

Plain Python / numpy, shares no code with the library; only the tests call it.

* `config_cost`     -- Section 3.2 ("Prioritizing Sparser Subnets") and the appendix on settings: the
                       cost F(alpha) of a configuration alpha = (s^1 ... s^L) is the network's FLOPs; a
                       linear layer at level N:M performs N/M of its dense multiply-accumulates
                       (Section 2), everything else is unchanged.
* `cost_edges`      -- Section 3.2 ("Sampling Strategy"): the costs between C_lower and C_upper are cut
                       into K levels C_1 .. C_K, i.e. K-1 intervals [C_i, C_i+1).
* `two_step_sample` -- the two-step sampling algorithm: first an interval, uniformly; then a configuration
                       drawn layer by layer from the current choice probabilities, conditioned on its cost
                       falling in the interval.  Conditioning is done by drawing again until it holds,
                       which is the conditional distribution itself.

Readings (the text leaves them open): the random numbers are uniforms in [0, 1) handed in by the caller,
consumed in order (one for the interval, then one per layer and attempt); a choice is the first one whose
cumulative probability exceeds the uniform; the last interval includes C_K (configurations with
F = C_upper are admitted by the text); intervals are equally wide.
"""
from __future__ import annotations

from typing import List, Optional, Sequence, Tuple

import numpy as np


def config_cost(layer_macs: Sequence[float], levels: Sequence[Tuple[int, int]], fixed: float = 0.0) -> float:
    total = float(fixed)
    for macs, (N, M) in zip(layer_macs, levels):
        total += float(macs) * N / M
    return total


def cost_edges(c_lower: float, c_upper: float, K: int) -> np.ndarray:
    return np.array([c_lower + (c_upper - c_lower) * i / (K - 1) for i in range(K)], dtype=np.float64)


def pick(prob_row: Sequence[float], u: float) -> int:
    acc = 0.0
    for s, p in enumerate(prob_row):
        acc += float(p)
        if u < acc:
            return s
    return len(prob_row) - 1


def two_step_sample(layer_macs, fixed, choices, probs, edges, uniforms) -> Optional[Tuple[int, List[int], int]]:
    """Returns (interval, choice index per layer, uniforms used), or None when the uniforms run out."""
    L, n_int = len(layer_macs), len(edges) - 1
    if len(uniforms) < 1:
        return None
    interval = min(int(uniforms[0] * n_int), n_int - 1)
    lo, hi = edges[interval], edges[interval + 1]
    used = 1
    while used + L <= len(uniforms):
        alpha = [pick(probs[l], uniforms[used + l]) for l in range(L)]
        used += L
        cost = config_cost(layer_macs, [choices[s] for s in alpha], fixed)
        inside = lo <= cost < hi or (interval == n_int - 1 and cost == hi)
        if inside:
            return interval, alpha, used
    return None
