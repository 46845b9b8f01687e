"""Pins of the configuration-cost model and the two-step sampler (CPU checker side)."""
import itertools
import os

import numpy as np
import pytest

from oracle import nm_search_oracle as so

HERE = os.path.dirname(os.path.abspath(__file__))


def deit_b_macs():
    tokens, blocks, d = 197, 12, 768
    linear = [tokens * o * k for o, k in ((2304, 768), (768, 768), (3072, 768), (768, 3072))] * blocks
    fixed = blocks * 2 * tokens * tokens * d + 196 * (3 * 16 * 16) * d + d * 1000
    return linear, fixed


def golden():
    out = {}
    for line in open(os.path.join(HERE, "golden", "table1_deit_b_cost.txt")):
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            out[k] = float(v)
    return out


def test_cost_model_reproduces_the_printed_costs_of_deit_b():
    linear, fixed = deit_b_macs()
    g = golden()
    dense = so.config_cost(linear, [(4, 4)] * 48, fixed)
    half = so.config_cost(linear, [(2, 4)] * 48, fixed)
    assert round(dense / 1e9, 1) == g["dense"]
    assert round(half / 1e9, 1) == g["uniform_2_4"]
    assert abs(sum(linear) - 16.73e9) < 0.01e9


def test_cost_is_linear_in_each_layer_density():
    macs = [10.0, 20.0, 40.0]
    assert so.config_cost(macs, [(1, 4), (2, 8), (16, 16)], fixed=3.0) == 3.0 + 2.5 + 5.0 + 40.0
    assert so.config_cost(macs, [(4, 4)] * 3) == 70.0


def test_edges_are_equally_spaced_and_include_both_ends():
    e = so.cost_edges(2.0, 10.0, 5)
    assert e.tolist() == [2.0, 4.0, 6.0, 8.0, 10.0]


def test_with_one_interval_the_sampler_is_the_inverse_cdf_per_layer():
    macs, choices = [1.0, 1.0], [(1, 4), (2, 4), (4, 4)]
    probs = [[0.2, 0.3, 0.5], [0.5, 0.5, 0.0]]
    edges = so.cost_edges(0.0, 2.0, 2)
    assert so.two_step_sample(macs, 0.0, choices, probs, edges, [0.9, 0.19, 0.49]) == (0, [0, 0], 3)
    assert so.two_step_sample(macs, 0.0, choices, probs, edges, [0.0, 0.2, 0.5]) == (0, [1, 1], 3)
    assert so.two_step_sample(macs, 0.0, choices, probs, edges, [0.5, 0.999, 0.0]) == (0, [2, 0], 3)
    assert so.two_step_sample(macs, 0.0, choices, probs, edges, [0.5, 0.999]) is None  # uniforms run out


def test_sample_lies_in_its_interval_and_intervals_are_hit_uniformly():
    rng = np.random.default_rng(7)
    macs = [3.0, 5.0, 2.0, 7.0, 4.0, 6.0]
    choices = [(1, 4), (2, 4), (4, 4)]
    probs = [[1 / 3] * 3] * 6
    lo = so.config_cost(macs, [(1, 4)] * 6)
    hi = so.config_cost(macs, [(4, 4)] * 6)
    edges = so.cost_edges(lo, hi, 5)
    hits = np.zeros(4, dtype=int)
    for _ in range(4000):
        r = so.two_step_sample(macs, 0.0, choices, probs, edges, rng.random(1 + 6 * 400))
        assert r is not None
        i, alpha, used = r
        c = so.config_cost(macs, [choices[s] for s in alpha])
        assert edges[i] <= c < edges[i + 1] or (i == 3 and c == edges[4])
        assert (used - 1) % 6 == 0
        hits[i] += 1
    assert np.all(np.abs(hits - 1000) < 5 * np.sqrt(1000 * 0.75))  # uniform over intervals (5 sigma)


def test_conditional_distribution_matches_exhaustive_enumeration():
    # 3 layers x 2 choices: every configuration's probability given its interval, by enumeration
    macs, choices = [4.0, 2.0, 1.0], [(1, 4), (4, 4)]
    probs = [[0.7, 0.3], [0.4, 0.6], [0.5, 0.5]]
    edges = so.cost_edges(so.config_cost(macs, [(1, 4)] * 3), so.config_cost(macs, [(4, 4)] * 3), 3)
    exact = {}
    for alpha in itertools.product(range(2), repeat=3):
        c = so.config_cost(macs, [choices[s] for s in alpha])
        i = 0 if c < edges[1] else 1
        exact[alpha] = (i, np.prod([probs[l][s] for l, s in enumerate(alpha)]))
    mass = [sum(p for i, p in exact.values() if i == k) for k in range(2)]
    rng = np.random.default_rng(11)
    counts, n = {}, 20000
    for _ in range(n):
        i, alpha, _ = so.two_step_sample(macs, 0.0, choices, probs, edges, rng.random(1 + 3 * 200))
        counts[tuple(alpha)] = counts.get(tuple(alpha), 0) + 1
    for alpha, (i, p) in exact.items():
        expect = 0.5 * p / mass[i]  # interval uniformly, then the conditional probability
        got = counts.get(alpha, 0) / n
        assert abs(got - expect) < 5 * np.sqrt(expect * (1 - expect) / n) + 1e-9, (alpha, got, expect)


# --------------------------------------------------------------------------------------
# The library's host functions against the checker (no GPU involved: they run anywhere).
# --------------------------------------------------------------------------------------
def test_library_cost_matches_the_checker_and_table_1():
    import paper_2409_09708_amd as nm
    linear, fixed = deit_b_macs()
    g = golden()
    assert round(nm.nm_config_cost(linear, [(4, 4)] * 48, fixed) / 1e9, 1) == g["dense"]
    assert round(nm.nm_config_cost(linear, [(2, 4)] * 48, fixed) / 1e9, 1) == g["uniform_2_4"]
    rng = np.random.default_rng(3)
    levels = [(1, 4), (2, 4), (1, 8), (2, 8), (4, 8), (1, 16), (4, 16)]
    for _ in range(20):
        cfg = [levels[i] for i in rng.integers(0, 7, 48)]
        assert nm.nm_config_cost(linear, cfg, fixed) == so.config_cost(linear, cfg, fixed)
    with pytest.raises(ValueError):
        nm.nm_config_cost([1.0], [(3, 2)])


def test_library_sampler_matches_the_checker_draw_for_draw():
    import paper_2409_09708_amd as nm
    from paper_2409_09708_amd.binding import NmError
    rng = np.random.default_rng(5)
    linear, fixed = deit_b_macs()
    choices = [(1, 4), (2, 4), (4, 4)]
    probs = rng.dirichlet(np.full(3, 8.0), size=48).tolist()
    lo = so.config_cost(linear, [(1, 4)] * 48, fixed)
    hi = 0.5 * so.config_cost(linear, [(4, 4)] * 48, fixed)  # C_upper = 50 % of the dense cost (appendix)
    edges = so.cost_edges(lo, hi, 6).tolist()
    seen = 0
    for _ in range(40):
        u = rng.random(1 + 48 * 300).tolist()
        ref = so.two_step_sample(linear, fixed, choices, probs, edges, u)
        if ref is None:
            with pytest.raises(NmError) as e:
                nm.nm_sample_config(linear, fixed, choices, probs, edges, u)
            assert e.value.status == 8
        else:
            assert nm.nm_sample_config(linear, fixed, choices, probs, edges, u) == (ref[0], ref[1], ref[2])
            seen += 1
    assert seen >= 5
    assert nm.nm_sample_config([1.0, 1.0], 0.0, choices, [[0.2, 0.3, 0.5], [0.5, 0.5, 0.0]], [0.0, 2.0],
                               [0.9, 0.19, 0.49]) == (0, [0, 0], 3)
