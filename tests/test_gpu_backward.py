"""GPU parity of the training products (Section 3.2; Section 3.1 weight-update figure): dX = dY (W (.) m) and
dW = (dY^T X) (.) m from the HIP library, called through its C ABI, against the CPU checker on the same seeded
inputs.  Acceptance as for the forward product: every element within 1e-2 of the sum of the magnitudes of its
terms, relative Frobenius error <= 5e-3, and for fp32 outputs the rounding bound of an fp32 sum in any order."""
import numpy as np
import pytest
import torch

import paper_2409_09708_amd as nm
from oracle import nm_oracle as orc
from paper_2409_09708_amd import workloads as wl
from gpu_util import check_output, dev_bf16, dev_words, host_bits, host_output, host_words

pytestmark = pytest.mark.gpu


def draw(seed, T, K, O, N, M):
    rng = np.random.default_rng(seed)
    X = wl.draw_activations(rng, T, K)
    W = wl.draw_weights(rng, O, K)
    dY = wl.draw_activations(rng, T, O)
    mask = orc.nm_mask(W, N, M)
    return X, W, dY, mask


@pytest.mark.parametrize("N,M", [(2, 4), (1, 8), (4, 16), (8, 8)])
@pytest.mark.parametrize("out_dtype", [torch.float32, torch.bfloat16])
def test_input_gradient_tiles(N, M, out_dtype):
    # several tiles with ragged edges in both output directions: T = 591, K = 336 (not a multiple of the tile),
    # O = 352 (11 reduction steps)
    T, K, O = 591, 336, 352
    X, W, dY, mask = draw(6100 + N * 17 + M, T, K, O, N, M)
    dXref, _, BX, _ = orc.nm_linear_backward(dY, X, W, mask)
    Wd = dev_bf16(W)
    Ws = torch.empty_like(Wd)
    nm.nm_prune(Wd, N, M, W_masked=Ws)
    assert np.array_equal(host_bits(Ws), orc.apply_mask(W, mask))
    dX = nm.nm_linear_backward_input(Ws, dev_bf16(dY), out_dtype=out_dtype)
    check_output(host_output(dX), dXref, BX, O, out_dtype == torch.float32, (N, M))
    # the packed form unpacks to the same operand
    v, i = nm.nm_pack(Wd, N, M)
    back = nm.nm_unpack(v, i, K, N, M)
    assert torch.equal(nm.nm_linear_backward_input(back, dev_bf16(dY), out_dtype=out_dtype), dX)


@pytest.mark.parametrize("out_dtype", [torch.float32, torch.bfloat16])
def test_input_gradient_large_layers(out_dtype):
    # a shape the library gives to the persistent kernel of the forward path (252 output tiles of 256 x 256, one
    # round of the chip; the weight is written transposed into its operand order first): ragged in both output
    # directions, K not a multiple of the tile
    T, K, O, N, M = 27 * 256 + 37, 8 * 256 + 8, 128, 2, 8
    assert nm.nm_backward_input_workspace_bytes(O, K, T) == 9 * 256 * O * 2
    X, W, dY, mask = draw(6150, T, K, O, N, M)
    dXref, _, BX, _ = orc.nm_linear_backward(dY, X, W, mask)
    Ws = dev_bf16(orc.apply_mask(W, mask))
    dX = nm.nm_linear_backward_input(Ws, dev_bf16(dY), out_dtype=out_dtype)
    check_output(host_output(dX), dXref, BX, O, out_dtype == torch.float32, "large")
    # a leading dimension larger than the row, on both operands and the output
    Ws_big = torch.zeros((O, K + 8), dtype=torch.bfloat16, device="cuda")
    Ws_big[:, :K] = Ws
    dY_big = torch.zeros((T, O + 8), dtype=torch.bfloat16, device="cuda")
    dY_big[:, :O] = dev_bf16(dY)
    out = torch.full((T, K + 16), 7.0, dtype=out_dtype, device="cuda")
    nm.nm_linear_backward_input(Ws_big[:, :K], dY_big[:, :O], out=out[:, 8:8 + K])
    assert torch.equal(out[:, 8:8 + K], dX)
    assert torch.all(out[:, :8] == 7.0) and torch.all(out[:, 8 + K:] == 7.0)


def test_input_gradient_views_and_general_shapes():
    # operands and output as views of wider buffers; an output view without 16-byte rows; and shapes the
    # matrix-core kernel does not take (O % 32 != 0, K % 8 != 0) on the general kernel
    for (T, K, O, pad) in [(200, 136, 96, 8), (200, 136, 96, 3), (77, 52, 40, 0), (65, 64, 70, 0), (1, 8, 32, 0)]:
        X, W, dY, mask = draw(6200 + T + K + O + pad, T, K, O, 2, 4)
        dXref, _, BX, _ = orc.nm_linear_backward(dY, X, W, mask)
        Ws_big = torch.zeros((O, K + 16), dtype=torch.bfloat16, device="cuda")
        Ws_big[:, :K] = dev_bf16(orc.apply_mask(W, mask))
        dY_big = torch.zeros((T, O + 8), dtype=torch.bfloat16, device="cuda")
        dY_big[:, :O] = dev_bf16(dY)
        out = torch.full((T, K + 2 * pad), 7.0, dtype=torch.float32, device="cuda")
        view = out[:, pad:pad + K]
        nm.nm_linear_backward_input(Ws_big[:, :K], dY_big[:, :O], out=view)
        check_output(host_output(view), dXref, BX, O, True, (T, K, O, pad))
        if pad:
            assert torch.all(out[:, :pad] == 7.0) and torch.all(out[:, pad + K:] == 7.0)


@pytest.mark.parametrize("N,M", [(2, 4), (1, 8), (4, 16), (8, 8)])
@pytest.mark.parametrize("T", [591, 197, 31, 2048])
def test_weight_gradient_tiles(N, M, T):
    # O = 328, K = 320: ragged tiles in both output directions; token counts with a ragged last step (591, 197),
    # shorter than one step (31: most ranges of the split reduction are empty) and a whole number of steps (2048)
    K, O = 320, 328
    X, W, dY, mask = draw(6300 + N * 17 + M + T, T, K, O, N, M)
    _, dWref, _, BW = orc.nm_linear_backward(dY, X, W, mask)
    _, dWall, _, BWall = orc.nm_linear_backward(dY, X, W, mask, masked_grad=False)
    Xd, dYd = dev_bf16(X), dev_bf16(dY)
    words = nm.nm_prune(dev_bf16(W), N, M)
    assert np.array_equal(host_words(words), orc.mask_to_words(mask))
    dW = nm.nm_linear_backward_weight(dYd, Xd, mask=words)
    got = host_output(dW)
    check_output(got, dWref, BW, T, True, (N, M, T, "masked"))
    assert np.all(got[~mask] == 0.0)
    dense = nm.nm_linear_backward_weight(dYd, Xd)
    check_output(host_output(dense), dWall, BWall, T, True, (N, M, T, "dense"))
    # kept positions carry the same number in both variants; the sum order is fixed, so calls repeat bit for bit
    assert torch.equal(torch.where(torch.from_numpy(mask).cuda(), dense, torch.zeros_like(dense)), dW)
    assert torch.equal(nm.nm_linear_backward_weight(dYd, Xd, mask=words), dW)
    d16 = nm.nm_linear_backward_weight(dYd, Xd, mask=words, out_dtype=torch.bfloat16)
    check_output(host_output(d16), dWref, BW, T, False, (N, M, T, "bf16"))


def test_weight_gradient_views_and_general_shapes():
    for (T, K, O, pad) in [(300, 136, 96, 8), (300, 136, 96, 1), (77, 52, 40, 0), (65, 64, 70, 0), (3, 8, 8, 0)]:
        N, M = (1, 4)
        X, W, dY, mask = draw(6400 + T + K + O + pad, T, K, O, N, M)
        _, dWref, _, BW = orc.nm_linear_backward(dY, X, W, mask)
        X_big = torch.zeros((T, K + 8), dtype=torch.bfloat16, device="cuda")
        X_big[:, :K] = dev_bf16(X)
        dY_big = torch.zeros((T, O + 16), dtype=torch.bfloat16, device="cuda")
        dY_big[:, :O] = dev_bf16(dY)
        out = torch.full((O, K + 2 * pad), 7.0, dtype=torch.float32, device="cuda")
        view = out[:, pad:pad + K]
        nm.nm_linear_backward_weight(dY_big[:, :O], X_big[:, :K], mask=dev_words(orc.mask_to_words(mask)), out=view)
        check_output(host_output(view), dWref, BW, T, True, (T, K, O, pad))
        if pad:
            assert torch.all(out[:, :pad] == 7.0) and torch.all(out[:, pad + K:] == 7.0)


def test_gradients_at_batch256_sampled():
    # DeiT-B fc2 at batch 256 (T = 50432, K = 3072, O = 768) in bf16, the shapes a training step of the
    # benchmark's workload meets; the checker computes sampled token rows of dX and sampled weight rows of dW
    T, K, O, N, M = 256 * 197, 3072, 768, 2, 8
    rng = np.random.default_rng(6500)
    X = wl.draw_activations(rng, T, K)
    W = wl.draw_weights(rng, O, K)
    dY = wl.draw_activations(rng, T, O)
    mask = orc.nm_mask(W, N, M)
    Wd, Xd, dYd = dev_bf16(W), dev_bf16(X), dev_bf16(dY)
    Ws = torch.empty_like(Wd)
    words = nm.nm_prune(Wd, N, M, W_masked=Ws)
    dX = nm.nm_linear_backward_input(Ws, dYd, out_dtype=torch.bfloat16)
    rows = np.unique(np.concatenate([np.arange(16), np.arange(T - 16, T), rng.integers(16, T - 16, size=16)]))
    dXref, _, BX, _ = orc.nm_linear_backward(dY[rows], X[rows], W, mask)
    check_output(host_output(dX[torch.from_numpy(rows).cuda()]), dXref, BX, O, False, "dX")
    dW = nm.nm_linear_backward_weight(dYd, Xd, mask=words)
    orows = np.unique(np.concatenate([np.arange(4), np.arange(O - 4, O), rng.integers(4, O - 4, size=8)]))
    _, dWref, _, BW = orc.nm_linear_backward(dY[:, orows], X, W[orows], mask[orows])
    check_output(host_output(dW[torch.from_numpy(orows).cuda()]), dWref, BW, T, True, "dW")
