"""Pins for the CPU checker: each test ties it to something other than itself
(brute force, closed forms, invariants the paper states, library routines)."""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import nm_oracle as orc
from paper_2409_09708_amd import workloads as wl

HERE = os.path.dirname(os.path.abspath(__file__))
LEVELS = [(1, 4), (2, 4), (3, 4), (4, 4), (1, 8), (2, 8), (3, 8), (4, 8), (8, 8), (1, 16), (2, 16), (4, 16)]


def bits(a):
    return wl.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))


def exact_abs(b):
    """|value| of a bf16 bit pattern as an exact Fraction (independent of the integer-key trick)."""
    b = int(b)
    e = (b >> 7) & 0xFF
    f = b & 0x7F
    if e == 0:
        return Fraction(f, 1 << 7) * Fraction(1, 1 << 126)
    return (1 + Fraction(f, 1 << 7)) * (Fraction(2) ** (e - 127))


def brute_force_group(group_bits, N):
    """All C(M,N) subsets: maximise the exact sum of magnitudes; among maximisers take the
    lexicographically smallest ascending index tuple (= equal magnitudes go to the lower index)."""
    M = len(group_bits)
    mags = [exact_abs(b) for b in group_bits]
    best, best_sum = None, None
    for S in itertools.combinations(range(M), N):  # generated in lexicographic order
        s = sum(mags[i] for i in S)
        if best_sum is None or s > best_sum:
            best, best_sum = S, s
    return best


def load_golden():
    out = {}
    with open(os.path.join(HERE, "golden", "hand_example_2to4.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, *v = line.split()
            out[k] = v
    return out


# ---------------------------------------------------------------- bf16 helpers

def test_bf16_rounding_and_exact_widening():
    # round to nearest even on the 16 dropped bits
    a = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.0e-39, 65504.0], dtype=np.float32)
    b = wl.f32_to_bf16_bits(a)
    # 1.00390625 = 1 + 2^-8 is a tie between 1.0 (even) and 1 + 2^-7 -> 1.0
    assert b[0] == 0x3F80 and b[1] == 0x3F80
    # 1.01171875 = 1 + 3*2^-8 ties between 1+2^-7 (odd) and 1+2^-6 (even) -> 1+2^-6
    assert b[2] == 0x3F82
    assert b[3] == 0xC020
    back = orc.bf16_bits_to_f64(b)
    assert back[0] == 1.0 and back[2] == 1.015625 and back[3] == -2.5
    # every bf16 pattern widens exactly: compare with Fractions on a sample of finite patterns
    for pat in [0x0001, 0x007F, 0x0080, 0x3F80, 0x3FFF, 0x7F7F, 0x8001, 0xBF80]:
        v = orc.bf16_bits_to_f64(np.array([pat], dtype=np.uint16))[0]
        assert Fraction(abs(v)) == exact_abs(pat)


# ---------------------------------------------------------------- mask (Eq. 1)

@pytest.mark.parametrize("N,M", LEVELS)
def test_mask_matches_brute_force_over_all_subsets(N, M):
    rng = np.random.default_rng(100 + 16 * N + M)
    for kind in ("gauss", "ties"):
        if kind == "gauss":
            W = wl.draw_weights(rng, 6, 2 * M)
        else:
            W = wl.tie_heavy_weights(rng, 12, 2 * M, distinct=4)
        if M == 16 and N == 4:
            W = W[:3]  # C(16,4)=1820 subsets per group: keep it quick
        mask = orc.nm_mask(W, N, M)
        for o in range(W.shape[0]):
            for g in range(W.shape[1] // M):
                grp = W[o, g * M:(g + 1) * M]
                S = brute_force_group(grp, N)
                got = tuple(np.nonzero(mask[o, g * M:(g + 1) * M])[0])
                assert got == S, (kind, o, g, [hex(int(x)) for x in grp])
                # threshold form of Eq. (1): every kept score >= every pruned score
                mags = [exact_abs(b) for b in grp]
                pruned = [mags[i] for i in range(M) if i not in S]
                if pruned:
                    assert min(mags[i] for i in S) >= max(pruned)


@pytest.mark.parametrize("N,M", LEVELS)
def test_mask_vectorised_equals_loop_form(N, M):
    rng = np.random.default_rng(7)
    for W in (wl.draw_weights(rng, 9, 4 * M), wl.tie_heavy_weights(rng, 9, 4 * M)):
        assert np.array_equal(orc.nm_mask(W, N, M), orc.nm_mask_loops(W, N, M))


@pytest.mark.parametrize("N,M", LEVELS)
def test_exactly_n_per_group(N, M):
    rng = np.random.default_rng(3)
    W = wl.tie_heavy_weights(rng, 32, 8 * M, distinct=3)
    m = orc.nm_mask(W, N, M).reshape(32, 8, M)
    assert np.all(m.sum(-1) == N)


@pytest.mark.parametrize("M", [4, 8, 16])
def test_subset_superset_nesting_and_dense_level(M):
    # Section 3.1, "Subset-Superset Relationship": mask(N1:M) is inside mask(N2:M) for N1 < N2; M:M keeps all
    rng = np.random.default_rng(11)
    for W in (wl.draw_weights(rng, 16, 4 * M), wl.tie_heavy_weights(rng, 16, 4 * M)):
        prev = np.zeros(W.shape, dtype=bool)
        for N in range(1, M + 1):
            m = orc.nm_mask(W, N, M)
            assert np.all(m[prev]), (N, M)
            assert (m & ~prev).sum() == W.shape[0] * W.shape[1] // M  # exactly one more per group
            prev = m
        assert prev.all()


@pytest.mark.parametrize("N,M", LEVELS)
def test_mask_closed_forms(N, M):
    dec = bits(np.arange(M, 0, -1, dtype=np.float32)[None, :])       # strictly decreasing |w|
    inc = bits(np.arange(1, M + 1, dtype=np.float32)[None, :])       # strictly increasing |w|
    eq = bits(np.full((1, M), -0.75, dtype=np.float32))              # all equal
    first = np.zeros(M, bool); first[:N] = True
    last = np.zeros(M, bool); last[M - N:] = True
    assert np.array_equal(orc.nm_mask(dec, N, M)[0], first)
    assert np.array_equal(orc.nm_mask(inc, N, M)[0], last)
    assert np.array_equal(orc.nm_mask(eq, N, M)[0], first)
    # +0 and -0 are equal scores
    z = np.array([[0x8000, 0x0000] * (M // 2)], dtype=np.uint16)
    assert np.array_equal(orc.nm_mask(z, N, M)[0], first)


def test_sign_flips_never_change_the_mask():
    rng = np.random.default_rng(5)
    W = wl.draw_weights(rng, 16, 64)
    flip = (rng.integers(0, 2, size=W.shape).astype(np.uint16) << 15)
    for N, M in LEVELS:
        assert np.array_equal(orc.nm_mask(W, N, M), orc.nm_mask(W ^ flip, N, M))


def test_integer_key_orders_like_float_magnitude():
    # a float |w| + stable argsort must agree with the integer key on all finite inputs
    rng = np.random.default_rng(9)
    W = np.concatenate([wl.draw_weights(rng, 8, 64), wl.tie_heavy_weights(rng, 8, 64)])
    # sprinkle subnormals and large values
    W[0, :8] = np.array([0x0001, 0x8001, 0x007F, 0x0080, 0x7F7F, 0xFF7F, 0x0000, 0x8000], dtype=np.uint16)
    for N, M in [(1, 4), (2, 4), (2, 8), (4, 8), (4, 16)]:
        a = np.abs(orc.bf16_bits_to_f64(W)).reshape(W.shape[0], -1, M)
        order = np.argsort(-a, axis=-1, kind="stable")[..., :N]
        ref = np.zeros(a.shape, bool)
        np.put_along_axis(ref, order, True, axis=-1)
        assert np.array_equal(orc.nm_mask(W, N, M), ref.reshape(W.shape))


def test_inf_and_nan_ordering_is_deterministic():
    # Inf beats finite; NaN patterns carry the largest keys and are kept
    W = np.array([[0x3F80, 0x7F80, 0x7FC0, 0x4000]], dtype=np.uint16)  # 1, +inf, nan, 2
    assert list(orc.nm_mask(W, 1, 4)[0]) == [False, False, True, False]
    assert list(orc.nm_mask(W, 2, 4)[0]) == [False, True, True, False]


def test_illegal_levels_and_shapes_raise():
    W = np.zeros((2, 12), dtype=np.uint16)
    with pytest.raises(ValueError):
        orc.nm_mask(W, 2, 8)   # 12 % 8 != 0
    for N, M in [(0, 4), (5, 4), (1, 3), (1, 32)]:
        with pytest.raises(ValueError):
            orc.nm_mask(np.zeros((2, 96), dtype=np.uint16), N, M)


# ---------------------------------------------------------------- hand example

def test_hand_example_fixture():
    g = load_golden()
    W = bits([[float(v) for v in g["weights"]]])
    m = orc.nm_mask(W, 2, 4)
    assert [int(v) for v in m[0]] == [int(v) for v in g["mask"]]
    vals, idx = orc.nm_pack(W, m, 2, 4)
    assert list(orc.bf16_bits_to_f64(vals)[0]) == [float(v) for v in g["values"]]
    assert int(idx[0, 0]) == int(g["index_word"][0], 16)
    assert int(orc.mask_to_words(m)[0, 0]) == int(g["mask_word"][0], 16)
    x = bits([[float(v) for v in g["x"]]])
    Y, B = orc.nm_linear(x, W, m)
    assert Y[0, 0] == float(g["y_2to4"][0])
    assert B[0, 0] == 4 + 3 + 15 + 32
    m1 = orc.nm_mask(W, 1, 4)
    v1, i1 = orc.nm_pack(W, m1, 1, 4)
    assert list(orc.bf16_bits_to_f64(v1)[0]) == [float(v) for v in g["values_1to4"]]
    assert int(i1[0, 0]) == int(g["index_word_1to4"][0], 16)
    assert orc.nm_linear(x, W, m1)[0][0, 0] == float(g["y_1to4"][0])
    # literal decode-select-multiply-add on the packed form gives the same numbers
    assert orc.spmm_gather_loops(vals, idx, x, 8, 2, 4)[0, 0] == float(g["y_2to4"][0])


# ---------------------------------------------------------------- pack / unpack

@pytest.mark.parametrize("N,M", LEVELS)
def test_pack_roundtrip_sizes_order_padding(N, M):
    rng = np.random.default_rng(21)
    for K in (M, 3 * M, 64, 80):
        if K % M:
            continue
        W = wl.tie_heavy_weights(rng, 5, K) if K == 80 else wl.draw_weights(rng, 5, K)
        m = orc.nm_mask(W, N, M)
        vals, idx = orc.nm_pack(W, m, N, M)
        b = {4: 2, 8: 3, 16: 4}[M]
        nf = K // M * N
        assert vals.shape == (5, nf) and vals.dtype == np.uint16
        assert idx.shape == (5, (nf * b + 31) // 32) and idx.dtype == np.uint32
        # exact round trip
        assert np.array_equal(orc.nm_unpack(vals, idx, K, N, M), orc.apply_mask(W, m))
        # decode the stream independently with Python integers: ascending positions, zero padding
        for o in range(5):
            row = 0
            for wi, w in enumerate(idx[o]):
                row |= int(w) << (32 * wi)
            assert row >> (nf * b) == 0
            pos = [(row >> (f * b)) & (M - 1) for f in range(nf)]
            assert row == sum(p << (f * b) for f, p in enumerate(pos))
            for g in range(K // M):
                pg = pos[g * N:(g + 1) * N]
                assert pg == sorted(set(pg))
                assert pg == list(np.nonzero(m[o, g * M:(g + 1) * M])[0])
                assert [int(v) for v in vals[o, g * N:(g + 1) * N]] == [int(W[o, g * M + p]) for p in pg]


@pytest.mark.parametrize("M", [4, 8, 16])
def test_pack_dense_level_reproduces_w(M):
    rng = np.random.default_rng(2)
    W = wl.draw_weights(rng, 4, 4 * M)
    m = orc.nm_mask(W, M, M)
    vals, idx = orc.nm_pack(W, m, M, M)
    assert np.array_equal(vals, W)
    assert np.array_equal(orc.nm_unpack(vals, idx, 4 * M, M, M), W)


def test_three_bit_fields_straddle_words():
    # M = 8: field 10 occupies bits 30..32, across the first word boundary
    K = 8 * 11
    W = np.zeros((1, K), dtype=np.uint16)
    W[0, 10 * 8 + 5] = 0x3F80  # group 10 keeps position 5 = 0b101
    m = orc.nm_mask(W, 1, 8)
    vals, idx = orc.nm_pack(W, m, 1, 8)
    assert idx.shape == (1, 2)
    assert int(idx[0, 0]) == (0b01 << 30) and int(idx[0, 1]) == 0b1
    assert np.array_equal(orc.nm_unpack(vals, idx, K, 1, 8), W)


def test_pack_rejects_wrong_mask():
    W = np.zeros((1, 8), dtype=np.uint16)
    bad = np.array([[1, 1, 1, 0, 1, 0, 0, 1]], dtype=bool)
    with pytest.raises(ValueError):
        orc.nm_pack(W, bad, 2, 4)


def test_mask_words_roundtrip():
    rng = np.random.default_rng(4)
    m = rng.integers(0, 2, size=(3, 80)).astype(bool)
    w = orc.mask_to_words(m)
    assert w.shape == (3, 3)
    assert np.array_equal(orc.words_to_mask(w, 80), m)
    assert int(w[0, 2]) >> 16 == 0


# ---------------------------------------------------------------- sparse product

def test_dense_level_is_a_plain_gemm():
    rng = np.random.default_rng(31)
    X = wl.draw_activations(rng, 7, 32)
    W = wl.draw_weights(rng, 5, 32)
    for M in (4, 8, 16):
        Y, B = orc.nm_linear_from_bits(X, W, M, M)
        Xf = (X.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        Wf = (W.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        assert np.allclose(Y, np.matmul(Xf, Wf.T), rtol=1e-13, atol=0)
        assert np.allclose(B, np.matmul(np.abs(Xf), np.abs(Wf).T), rtol=1e-13, atol=0)


@pytest.mark.parametrize("N,M", [(1, 4), (2, 4), (2, 8), (3, 8), (4, 16)])
def test_identity_and_ones_activations(N, M):
    rng = np.random.default_rng(41)
    K = 32
    W = wl.draw_weights(rng, 6, K)
    m = orc.nm_mask(W, N, M)
    I = bits(np.eye(K, dtype=np.float32))
    Y, _ = orc.nm_linear(I, W, m)
    assert np.array_equal(Y, orc.bf16_bits_to_f64(orc.apply_mask(W, m)).T)  # X = I -> Y = W_s^T exactly
    ones = bits(np.ones((2, K), dtype=np.float32))
    Y1, _ = orc.nm_linear(ones, W, m)
    vals, _ = orc.nm_pack(W, m, N, M)
    rowsum = np.array([sum(Fraction(float(v)) for v in orc.bf16_bits_to_f64(vals[o])) for o in range(6)], dtype=object)
    for o in range(6):
        assert Fraction(float(Y1[0, o])) == rowsum[o] or abs(Y1[0, o] - float(rowsum[o])) < 1e-15


@pytest.mark.parametrize("N,M", [(1, 4), (2, 4), (1, 8), (2, 8), (3, 8), (4, 8), (1, 16), (2, 16), (4, 16)])
def test_gather_form_equals_dense_form(N, M):
    # two formulations that share nothing: dense GEMM against the masked weight vs.
    # decode-select-multiply-add on the packed form
    rng = np.random.default_rng(51 + N + M)
    K, O, T = 3 * 16, 4, 3
    X = wl.draw_activations(rng, T, K)
    W = wl.draw_weights(rng, O, K)
    m = orc.nm_mask(W, N, M)
    vals, idx = orc.nm_pack(W, m, N, M)
    Yd, B = orc.nm_linear(X, W, m)
    Yg = orc.spmm_gather_loops(vals, idx, X, K, N, M)
    assert np.all(np.abs(Yd - Yg) <= 1e-14 * B + 1e-300)
    assert orc.useful_macs(T, O, K, N, M) == int(m.sum()) * T


def test_exact_small_integer_product_and_bias():
    # integers are exact in bf16 and fp64: compare with exact integer arithmetic
    rng = np.random.default_rng(61)
    Xi = rng.integers(-8, 9, size=(5, 16))
    Wi = rng.integers(-8, 9, size=(3, 16))
    X, W = bits(Xi), bits(Wi)
    m = orc.nm_mask(W, 2, 4)
    Y, B = orc.nm_linear(X, W, m, bias=np.array([1.0, -2.0, 0.5]))
    ref = Xi @ (Wi * m).T
    assert np.array_equal(Y, ref + np.array([1.0, -2.0, 0.5]))
    assert np.array_equal(B, np.abs(Xi) @ np.abs(Wi * m).T)
    # a transposed operand or a dropped mask would not survive this
    assert not np.array_equal(Y, Xi @ Wi.T + np.array([1.0, -2.0, 0.5]))


# ---------------------------------------------------------------- workload recipe

def test_level_draws_are_the_documented_ones():
    lv = wl.draw_levels(0, wl.LEVELS_7, 48)
    assert len(lv) == 48 and set(lv) <= set(wl.LEVELS_7)
    stack = wl.deit_b_stack()
    assert len(stack) == 48 and stack[0].T == 50432
    dense = sum(L.dense_flops for L in stack)
    assert abs(dense - 2 * 50432 * 84934656) < 1
    # DeiT-B: the 48 linears are 84,934,656 MACs per token (12 x (768*2304 + 768*768 + 2*768*3072))
    assert sum(L.K * L.O for L in stack) == 84934656
    blk = wl.deit_b_block()
    assert [L.O for L in blk] == [2304, 768, 3072, 768] and blk[0].T == 12608
    sw = wl.swin_b_stages()
    assert [L.T for L in sw[::4]] == [200704, 50176, 12544, 3136]


# --------------------------------------------------------------------------------------
# Ranks inside a group (Section 3, subset-superset relationship): one rank per weight holds
# every level of that M.  Pinned by the counting definition, by the nesting it expresses
# (against the mask, which is pinned above) and by closed forms.
# --------------------------------------------------------------------------------------
@pytest.mark.parametrize("M", [4, 8, 16])
def test_rank_is_the_number_of_members_that_come_first(M):
    rng = np.random.default_rng(300 + M)
    W = wl.tie_heavy_weights(rng, 6, 4 * M)
    assert np.array_equal(orc.nm_rank(W, M), orc.nm_rank_loops(W, M))
    W = wl.draw_weights(rng, 5, 3 * M)
    assert np.array_equal(orc.nm_rank(W, M), orc.nm_rank_loops(W, M))


@pytest.mark.parametrize("M", [4, 8, 16])
def test_rank_is_a_permutation_per_group_and_every_level_is_rank_below_n(M):
    rng = np.random.default_rng(310 + M)
    for W in (wl.draw_weights(rng, 16, 8 * M), wl.tie_heavy_weights(rng, 16, 8 * M)):
        rank = orc.nm_rank(W, M)
        groups = rank.reshape(W.shape[0], -1, M)
        assert np.array_equal(np.sort(groups, axis=-1), np.broadcast_to(np.arange(M), groups.shape))
        for N in range(1, M + 1):
            assert np.array_equal(rank < N, orc.nm_mask(W, N, M)), (N, M)


def test_rank_closed_forms():
    M = 8
    dec = wl.f32_to_bf16_bits(np.array([[8, -7, 6, -5, 4, -3, 2, -1]], dtype=np.float32))
    assert orc.nm_rank(dec, M).tolist() == [[0, 1, 2, 3, 4, 5, 6, 7]]
    inc = dec[:, ::-1].copy()
    assert orc.nm_rank(inc, M).tolist() == [[7, 6, 5, 4, 3, 2, 1, 0]]
    same = wl.f32_to_bf16_bits(np.full((1, M), -0.5, dtype=np.float32))
    assert orc.nm_rank(same, M).tolist() == [[0, 1, 2, 3, 4, 5, 6, 7]]
    mixed = wl.f32_to_bf16_bits(np.array([[1, -2, 2, 0]], dtype=np.float32))  # the tie goes to the lower index
    assert orc.nm_rank(mixed, 4).tolist() == [[2, 0, 1, 3]]


def test_rank_nibbles_round_trip_and_layout():
    rank = np.array([[0, 3, 1, 2, 15, 14, 0, 9]], dtype=np.uint8)
    nib = orc.rank_nibbles(rank)
    assert nib.tolist() == [[0x30, 0x21, 0xEF, 0x90]]
    assert np.array_equal(orc.nibbles_to_rank(nib), rank)


# ------------------------------------------------------------------ masks from a supplied saliency (Section 3.1)

def test_score_mask_equals_the_magnitude_mask_when_the_score_is_the_magnitude():
    rng = np.random.default_rng(81)
    for (N, M) in [(1, 4), (2, 4), (3, 8), (4, 16), (8, 8)]:
        W = wl.tie_heavy_weights(rng, 12, 4 * M)
        score = np.abs(orc.bf16_bits_to_f64(W)).astype(np.float32)  # exact: bfloat16 magnitudes are float32 numbers
        assert np.array_equal(orc.nm_mask_from_scores(score, N, M), orc.nm_mask(W, N, M))


def test_score_mask_brute_force_and_monotone_invariance():
    import itertools
    rng = np.random.default_rng(82)
    for (N, M) in [(1, 4), (2, 4), (2, 8), (3, 8)]:
        s = rng.integers(-3, 4, size=(20, M)).astype(np.float32)  # many ties, negative scores too
        mask = orc.nm_mask_from_scores(s, N, M)
        for row, m in zip(s, mask):
            assert m.sum() == N
            kept = tuple(np.flatnonzero(m))
            # threshold property, and among all sets with it the lexicographically smallest
            best = None
            for c in itertools.combinations(range(M), N):
                out = [i for i in range(M) if i not in c]
                if all(row[i] >= row[j] for i in c for j in out):
                    best = c if best is None else min(best, c)
            assert kept == best
        # a strictly increasing map of the scores changes nothing
        assert np.array_equal(orc.nm_mask_from_scores(2.0 * s + 1.0, N, M), mask)
        assert np.array_equal(orc.nm_mask_from_scores(np.exp(s), N, M), mask)


def test_score_mask_special_values_and_a_taylor_example():
    # -0 ties +0 (lower index wins); NaN ranks first; -inf last
    s = np.array([[-0.0, 0.0, -1.0, -np.inf], [1.0, np.nan, 2.0, np.inf]], dtype=np.float32)
    assert orc.nm_mask_from_scores(s, 1, 4).tolist() == [[True, False, False, False], [False, True, False, False]]
    assert orc.nm_mask_from_scores(s, 2, 4).tolist() == [[True, True, False, False], [False, True, False, True]]
    # a NaN ranks above +inf wherever it stands
    t = np.array([[np.inf, 5.0, np.nan, np.inf]], dtype=np.float32)
    assert orc.nm_mask_from_scores(t, 1, 4).tolist() == [[False, False, True, False]]
    assert orc.nm_mask_from_scores(t, 2, 4).tolist() == [[True, False, True, False]]
    # first-order Taylor saliency |w * g| of one group: w = (4, -1, 2, 0.5), g = (0.1, -3, 1, 8) -> (0.4, 3, 2, 4):
    # the largest weight is pruned, which the magnitude rule would keep
    w = np.array([[4.0, -1.0, 2.0, 0.5]])
    g = np.array([[0.1, -3.0, 1.0, 8.0]])
    assert orc.nm_mask_from_scores(np.abs(w * g), 2, 4).tolist() == [[False, True, False, True]]
