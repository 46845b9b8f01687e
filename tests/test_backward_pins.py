"""Pins for the checker's training gradients (Section 3.2, Section 3.1 weight-update figure).  The gradients
are tied to the forward definition, not to their own formula: Y is linear in X and in the kept weights, so a
finite change of one input changes L = <G, Y> by exactly gradient * change; pruned weights do not reach Y at
all.  Plus the adjoint identities and a hand-computed case."""
import numpy as np
import pytest

from oracle import nm_oracle as orc
from paper_2409_09708_amd import workloads as wl


def f64_to_bf16_bits(a):
    """bf16 bit patterns of values that are exactly representable (test inputs only)."""
    a32 = np.asarray(a, dtype=np.float32)
    bits = (a32.view(np.uint32) >> 16).astype(np.uint16)
    assert np.array_equal(orc.bf16_bits_to_f64(bits), a32.astype(np.float64))
    return bits


def loss(G, x_bits, w_bits, mask):
    Y, _ = orc.nm_linear(x_bits, w_bits, mask)
    return float(np.sum(G * Y))


def case(seed, T=7, O=6, K=16, N=2, M=4):
    rng = np.random.default_rng(seed)
    X = wl.draw_activations(rng, T, K)
    W = wl.draw_weights(rng, O, K)
    dY = wl.draw_activations(rng, T, O)
    mask = orc.nm_mask(W, N, M)
    return X, W, dY, mask


def test_hand_computed_case():
    # one group of four, 2:4 keeps positions 1 and 3 (|-3| and |4|); T = 2, O = 1
    W = f64_to_bf16_bits([[1.0, -3.0, 2.0, 4.0]])
    X = f64_to_bf16_bits([[1.0, 2.0, 3.0, 4.0], [-1.0, 0.5, 2.0, -2.0]])
    dY = f64_to_bf16_bits([[2.0], [-1.0]])
    mask = orc.nm_mask(W, 2, 4)
    assert mask.tolist() == [[False, True, False, True]]
    dX, dW, BX, BW = orc.nm_linear_backward(dY, X, W, mask)
    assert dX.tolist() == [[0.0, -6.0, 0.0, 8.0], [0.0, 3.0, 0.0, -4.0]]
    # dY^T X = 2*[1,2,3,4] - [-1,.5,2,-2] = [3, 3.5, 4, 10]
    assert dW.tolist() == [[0.0, 3.5, 0.0, 10.0]]
    assert BX.tolist() == [[0.0, 6.0, 0.0, 8.0], [0.0, 3.0, 0.0, 4.0]]
    assert BW.tolist() == [[0.0, 4.5, 0.0, 10.0]]
    _, dWd, _, BWd = orc.nm_linear_backward(dY, X, W, mask, masked_grad=False)
    assert dWd.tolist() == [[3.0, 3.5, 4.0, 10.0]]
    assert BWd.tolist() == [[3.0, 4.5, 8.0, 10.0]]


@pytest.mark.parametrize("N,M", [(1, 4), (2, 4), (2, 8), (4, 16), (8, 8)])
def test_input_gradient_is_the_change_of_the_forward_product(N, M):
    X, W, dY, mask = case(10 + N + M, K=2 * M, N=N, M=M)
    G = orc.bf16_bits_to_f64(dY)
    dX, _, _, _ = orc.nm_linear_backward(dY, X, W, mask)
    base = loss(G, X, W, mask)
    rng = np.random.default_rng(3)
    for _ in range(12):
        t, k = int(rng.integers(X.shape[0])), int(rng.integers(X.shape[1]))
        X2 = X.copy()
        X2[t, k] = X[t, k] ^ 0x0040  # another bf16 value
        dx = float(orc.bf16_bits_to_f64(X2[t, k:k + 1])[0] - orc.bf16_bits_to_f64(X[t, k:k + 1])[0])
        assert dx != 0.0
        assert loss(G, X2, W, mask) - base == pytest.approx(dX[t, k] * dx, rel=1e-9, abs=1e-12)


@pytest.mark.parametrize("N,M", [(1, 4), (2, 4), (2, 8), (4, 16), (8, 8)])
def test_weight_gradient_is_the_change_of_the_forward_product(N, M):
    X, W, dY, mask = case(20 + N + M, K=2 * M, N=N, M=M)
    G = orc.bf16_bits_to_f64(dY)
    _, dW, _, _ = orc.nm_linear_backward(dY, X, W, mask)
    _, dW_dense, _, _ = orc.nm_linear_backward(dY, X, W, mask, masked_grad=False)
    base = loss(G, X, W, mask)
    for o in range(W.shape[0]):
        for k in range(W.shape[1]):
            W2 = W.copy()
            W2[o, k] = W[o, k] ^ 0x0040  # another bf16 value; the mask of the step stays as it is
            dw = float(orc.bf16_bits_to_f64(W2[o, k:k + 1])[0] - orc.bf16_bits_to_f64(W[o, k:k + 1])[0])
            change = loss(G, X, W2, mask) - base
            if mask[o, k]:
                assert change == pytest.approx(dW[o, k] * dw, rel=1e-9, abs=1e-12)
                assert dW_dense[o, k] == dW[o, k]
            else:
                assert change == 0.0 and dW[o, k] == 0.0  # a pruned weight does not reach the output
                # the unmasked variant still carries the product of its position
                want = sum(float(G[t, o]) * float(orc.bf16_bits_to_f64(X[t, k:k + 1])[0]) for t in range(X.shape[0]))
                assert dW_dense[o, k] == pytest.approx(want, rel=1e-12, abs=1e-15)


def test_adjoint_identities():
    # <G, Y> = <X, dX> = <W (.) m, dW>: the product is linear in each operand
    X, W, dY, mask = case(31, T=9, O=8, K=32, N=2, M=8)
    G = orc.bf16_bits_to_f64(dY)
    Y, _ = orc.nm_linear(X, W, mask)
    dX, dW, _, _ = orc.nm_linear_backward(dY, X, W, mask)
    lhs = float(np.sum(G * Y))
    assert float(np.sum(orc.bf16_bits_to_f64(X) * dX)) == pytest.approx(lhs, rel=1e-12)
    assert float(np.sum(orc.bf16_bits_to_f64(orc.apply_mask(W, mask)) * dW)) == pytest.approx(lhs, rel=1e-12)


def test_bounds_dominate_and_follow_the_mask():
    X, W, dY, mask = case(41, T=5, O=8, K=16, N=1, M=4)
    dX, dW, BX, BW = orc.nm_linear_backward(dY, X, W, mask)
    assert np.all(np.abs(dX) <= BX + 1e-15) and np.all(np.abs(dW) <= BW + 1e-15)
    assert np.all(BW[~mask] == 0.0) and np.all(BW[mask] > 0.0)
    # columns of W (.) m that are pruned in every row receive no input gradient
    dead = ~mask.any(axis=0)
    assert np.all(dX[:, dead] == 0.0)
