"""Pins for the int8 checker (Section 4, Table 6: 8-bit quantisation on top of the sparse networks).  The
integer sum is tied to plain Python integers, to the pinned float checker on inputs both can hold exactly, and
to closed forms; the rescaling to cases where it is exact."""
import numpy as np
import pytest

from oracle import nm_int8_oracle as q
from oracle import nm_oracle as orc
from paper_2409_09708_amd import workloads as wl


def legal_mask(rng, O, K, N, M):
    m = np.zeros((O, K // M, M), dtype=bool)
    for o in range(O):
        for g in range(K // M):
            m[o, g, rng.choice(M, size=N, replace=False)] = True
    return m.reshape(O, K)


@pytest.mark.parametrize("N,M", [(1, 4), (2, 4), (2, 8), (4, 8), (4, 16), (16, 16)])
def test_integer_sum_against_python_integers(N, M):
    rng = np.random.default_rng(100 + N + M)
    T, O, K = 5, 6, 2 * M
    xq, wq = wl.draw_int8(rng, T, K), wl.draw_int8(rng, O, K)
    mask = legal_mask(rng, O, K, N, M)
    assert np.array_equal(q.nm_accumulate_i8(xq, wq, mask), q.nm_accumulate_i8_loops(xq, wq, mask))


def test_extreme_values_do_not_wrap():
    # -128 * -128 summed over K = 4096 kept positions exceeds 2^25: the sum must be carried wider than int8/int16
    K = 4096
    xq = np.full((1, K), -128, dtype=np.int8)
    wq = np.full((1, K), -128, dtype=np.int8)
    mask = np.ones((1, K), dtype=bool)
    assert q.nm_accumulate_i8(xq, wq, mask)[0, 0] == 128 * 128 * K


@pytest.mark.parametrize("N,M", [(1, 4), (2, 4), (1, 8), (4, 8)])
def test_closed_forms(N, M):
    T, O, K = 3, 4, 8 * M
    rng = np.random.default_rng(7)
    mask = legal_mask(rng, O, K, N, M)
    ones = np.ones((T, K), dtype=np.int8)
    wq = np.full((O, K), 3, dtype=np.int8)
    # all-ones activations count the kept weights: N per group
    assert np.all(q.nm_accumulate_i8(ones, wq, mask) == 3 * N * (K // M))
    # a one-hot activation reads one column of W (.) m
    for k in (0, 5, K - 1):
        e = np.zeros((1, K), dtype=np.int8)
        e[0, k] = 1
        assert np.array_equal(q.nm_accumulate_i8(e, wq, mask)[0], np.where(mask[:, k], 3, 0))


@pytest.mark.parametrize("N,M", [(2, 4), (1, 8), (4, 16)])
def test_agrees_with_the_float_checker_on_integers_both_hold_exactly(N, M):
    # integers up to 127 are exact in bfloat16 and their products and sums are exact in fp64, so the float
    # checker's product of the same numbers must give the same integers; the mask comes from the float side
    rng = np.random.default_rng(200 + N + M)
    T, O, K = 9, 8, 4 * M
    xq, wq = wl.draw_int8(rng, T, K), wl.draw_int8(rng, O, K)
    xb = wl.f32_to_bf16_bits(xq.astype(np.float32))
    wb = wl.f32_to_bf16_bits(wq.astype(np.float32))
    assert np.array_equal(orc.bf16_bits_to_f64(wb), wq.astype(np.float64))
    mask = orc.nm_mask(wb, N, M)  # magnitude saliency on the same integers
    Y, _ = orc.nm_linear(xb, wb, mask)
    assert np.array_equal(q.nm_accumulate_i8(xq, wq, mask).astype(np.float64), Y)


def test_rescaling():
    rng = np.random.default_rng(5)
    T, O, K = 4, 6, 16
    xq, wq = wl.draw_int8(rng, T, K), wl.draw_int8(rng, O, K)
    mask = legal_mask(rng, O, K, 2, 4)
    acc = q.nm_accumulate_i8(xq, wq, mask)
    # power-of-two scales are exact: Y = acc * 2^-3 * 2^(o-2)
    w_scale = np.array([2.0 ** (o - 2) for o in range(O)])
    y = q.nm_linear_i8(xq, wq, mask, 0.125, w_scale)
    assert np.array_equal(y, acc * 0.125 * w_scale[None, :])
    bias = np.arange(O, dtype=np.float64) - 2.5
    assert np.array_equal(q.nm_linear_i8(xq, wq, mask, 0.125, w_scale, bias), y + bias[None, :])
    # scaling the activations' scale scales the output: linear in x_scale
    assert np.array_equal(q.nm_linear_i8(xq, wq, mask, 0.25, w_scale), 2 * y)


def test_pruned_weights_are_ignored_whatever_they_hold():
    rng = np.random.default_rng(6)
    xq, wq = wl.draw_int8(rng, 3, 16), wl.draw_int8(rng, 4, 16)
    mask = legal_mask(rng, 4, 16, 1, 4)
    other = wq.copy()
    other[~mask] = 99
    assert np.array_equal(q.nm_accumulate_i8(xq, wq, mask), q.nm_accumulate_i8(xq, other, mask))


# ---- the compressed int8 form ---------------------------------------------------------------------------------

def test_packed_int8_hand_example():
    # the worked 2:4 group of tests/golden/hand_example_2to4.txt scaled to integers: weights (5, -20, 10, -10)
    # keep positions 1 and 2, so values (-20, 10) and the two 2-bit fields 1, 2 -> nibble 0b1001; a second group
    # (7, 0, 0, -3) keeps positions 0 and 3 -> fields 0, 3 -> nibble 0b1100; LSB first: byte 0xC9
    wq = np.array([[5, -20, 10, -10, 7, 0, 0, -3]], dtype=np.int8)
    mask = np.array([[0, 1, 1, 0, 1, 0, 0, 1]], dtype=bool)
    values, indices = q.nm_pack_i8(wq, mask, 2, 4)
    assert values.tolist() == [[-20, 10, 7, -3]]
    assert indices.tolist() == [[0xC9]]
    assert np.array_equal(q.nm_unpack_i8(values, indices, 8, 2, 4), np.where(mask, wq, 0))


@pytest.mark.parametrize("N,M", [(1, 4), (2, 4), (3, 4), (1, 8), (2, 8), (3, 8), (4, 8), (1, 16), (2, 16), (4, 16), (8, 8)])
def test_packed_int8_index_stream_is_the_float_layers(N, M):
    # the positions depend on the mask alone: the index words must be those the (pinned) bfloat16 checker writes
    # for any weight with the same mask; 3-bit fields straddle words at K = 96 (36 bits at 1:8, 108 at 3:8)
    rng = np.random.default_rng(300 + N + M)
    O, K = 5, 96 if M == 8 else 64
    wq = wl.draw_int8(rng, O, K)
    mask = legal_mask(rng, O, K, N, M)
    values, indices = q.nm_pack_i8(wq, mask, N, M)
    wb = wl.f32_to_bf16_bits(wq.astype(np.float32))
    fvals, findex = orc.nm_pack(wb, mask, N, M)
    assert np.array_equal(indices, findex)
    # and the values are the float layer's values (integers up to 127 are exact in bfloat16)
    assert np.array_equal(values.astype(np.float64), orc.bf16_bits_to_f64(fvals))
    # sizes: N/M of the weights, log2(M) bits each, rows padded to words
    assert values.shape == (O, K // M * N) and indices.shape == (O, orc.index_words_per_row(K, N, M))


@pytest.mark.parametrize("N,M", [(1, 4), (2, 4), (2, 8), (4, 8), (1, 16), (4, 16)])
def test_packed_int8_round_trip_and_kept_values_by_definition(N, M):
    rng = np.random.default_rng(400 + N + M)
    O, K = 4, 4 * M
    wq = wl.draw_int8(rng, O, K)
    wq[0, :M] = -128  # the extreme value survives packing
    mask = legal_mask(rng, O, K, N, M)
    values, indices = q.nm_pack_i8(wq, mask, N, M)
    assert np.array_equal(q.nm_unpack_i8(values, indices, K, N, M), np.where(mask, wq, 0))
    # by definition: the j-th kept weight of group g, counted in ascending position
    for o in range(O):
        for g in range(K // M):
            kept = [int(wq[o, g * M + p]) for p in range(M) if mask[o, g * M + p]]
            assert values[o, g * N:(g + 1) * N].tolist() == kept
    # padding bits of the last index word are zero
    used = (K // M * N * {4: 2, 8: 3, 16: 4}[M]) % 32
    if used:
        assert np.all(indices[:, -1] >> np.uint32(used) == 0)


@pytest.mark.parametrize("N,M", [(1, 4), (2, 4), (2, 8), (4, 16)])
def test_gather_form_on_the_packed_int8_equals_the_masked_product(N, M):
    rng = np.random.default_rng(500 + N + M)
    T, O, K = 3, 4, 2 * M
    xq, wq = wl.draw_int8(rng, T, K), wl.draw_int8(rng, O, K)
    mask = legal_mask(rng, O, K, N, M)
    values, indices = q.nm_pack_i8(wq, mask, N, M)
    assert np.array_equal(q.nm_accumulate_i8_packed_loops(values, indices, xq, K, N, M),
                          q.nm_accumulate_i8_loops(xq, wq, mask))


def test_packed_int8_rejects_an_illegal_mask():
    wq = np.zeros((1, 8), dtype=np.int8)
    mask = np.array([[1, 1, 1, 0, 0, 0, 0, 1]], dtype=bool)
    with pytest.raises(ValueError):
        q.nm_pack_i8(wq, mask, 2, 4)
