"""GPU parity of the product at few tokens (up to 208) that reads the packed format itself, the path of a call that
comes without a workspace: every level of its set, windows over the reduction from one to many, ragged row groups,
bias, both output types, strided views, the batched call, and the identity activations that tie it to the packed
bytes exactly."""
import numpy as np
import pytest
import torch

import paper_2409_09708_amd as nm
from oracle import nm_oracle as orc
from paper_2409_09708_amd import workloads as wl
from gpu_util import check_output, dev_bf16, host_bits, host_output

pytestmark = pytest.mark.gpu

LEVELS = [(1, 4), (1, 8), (2, 8), (4, 8), (1, 16), (2, 16), (4, 16)]  # 2:4 never needs a workspace
# (T, K, O): one window / several / an odd count / many; O below, at and above one 128-row item, ragged 16-row blocks
SHAPES = [(197, 768, 768), (1, 64, 16), (208, 128, 144), (16, 192, 132), (100, 3072, 256), (37, 320, 4)]


@pytest.mark.parametrize("N,M", LEVELS)
@pytest.mark.parametrize("shape", SHAPES)
def test_parity_with_bias_in_both_output_types(N, M, shape):
    T, K, O = shape
    assert nm.nm_spmm_workspace_bytes(O, K, N, M, T) > 0  # with a workspace the call would take another kernel
    rng = np.random.default_rng(9100 + N * 17 + M + T + K + O)
    X = wl.draw_activations(rng, T, K)
    W = wl.tie_heavy_weights(rng, O, K) if (T + O) % 2 else wl.draw_weights(rng, O, K)
    bias = rng.standard_normal(O).astype(np.float32)
    Yref, B = orc.nm_linear_from_bits(X, W, N, M, bias=bias)
    B = B + np.abs(bias)[None, :]
    Xd, bd = dev_bf16(X), torch.from_numpy(bias).cuda()
    v, i = nm.nm_pack(dev_bf16(W), N, M)
    y32 = nm.nm_linear_forward(v, i, K, N, M, Xd, bias=bd, from_packed=True)
    check_output(host_output(y32), Yref, B, K // M * N + 1, True, (N, M, shape))
    y16 = nm.nm_linear_forward(v, i, K, N, M, Xd, bias=bd, out_dtype=torch.bfloat16, from_packed=True)
    check_output(host_output(y16), Yref, B, K // M * N + 1, False, (N, M, shape))
    # without bias the two calls differ by the bias alone
    y0 = nm.nm_spmm(v, i, K, N, M, Xd, from_packed=True)
    Yref0, B0 = orc.nm_linear_from_bits(X, W, N, M)
    check_output(host_output(y0), Yref0, B0, K // M * N, True, (N, M, shape, "no bias"))


@pytest.mark.parametrize("N,M", LEVELS)
def test_identity_activations_reproduce_the_packed_weight_exactly(N, M):
    # X = I (T = K <= 208): Y = W_s^T bit for bit in bfloat16, whatever the summation order
    for K in (64, 128, 192):
        O = 160
        rng = np.random.default_rng(9300 + N * 17 + M + K)
        W = wl.draw_weights(rng, O, K)
        mask = orc.nm_mask(W, N, M)
        Ws = orc.apply_mask(W, mask)
        eye = np.zeros((K, K), dtype=np.uint16)
        eye[np.arange(K), np.arange(K)] = 0x3F80  # 1.0
        v, i = nm.nm_pack(dev_bf16(W), N, M)
        y = nm.nm_spmm(v, i, K, N, M, dev_bf16(eye), out_dtype=torch.bfloat16, from_packed=True)
        canon = lambda b: np.where((b & 0x7FFF) == 0, 0, b)  # -0 and +0 are the same value
        assert np.array_equal(canon(host_bits(y)), canon(Ws.T))


def test_views_of_wider_buffers_and_guard_columns():
    T, K, O, N, M = 197, 256, 264, 2, 8
    rng = np.random.default_rng(9400)
    X = wl.draw_activations(rng, T, K)
    W = wl.draw_weights(rng, O, K)
    Yref, B = orc.nm_linear_from_bits(X, W, N, M)
    v, i = nm.nm_pack(dev_bf16(W), N, M)
    Xbig = torch.zeros((T + 3, K + 16), dtype=torch.bfloat16, device="cuda")
    Xbig[1:T + 1, 8:8 + K] = dev_bf16(X)
    for dt, pad in ((torch.float32, 4), (torch.bfloat16, 8)):
        out = torch.full((T + 2, O + 2 * pad), 7.0, dtype=dt, device="cuda")
        nm.nm_spmm(v, i, K, N, M, Xbig[1:T + 1, 8:8 + K], out=out[1:T + 1, pad:pad + O], from_packed=True)
        check_output(host_output(out[1:T + 1, pad:pad + O].contiguous()), Yref, B, K // M * N, dt == torch.float32, dt)
        assert torch.all(out[0] == 7.0) and torch.all(out[T + 1] == 7.0)
        assert torch.all(out[:, :pad] == 7.0) and torch.all(out[:, pad + O:] == 7.0)


def test_batched_call_equals_the_single_calls():
    # layers of every level, different shapes and output types, in one call: the same bytes as one call each
    rng = np.random.default_rng(9500)
    layers, singles, outs = [], [], []
    for n, (N, M) in enumerate(LEVELS * 2):
        T = (197, 64, 208, 5)[n % 4]
        K = (768, 3072, 128, 192)[n % 4]
        O = (768, 128, 400, 2304)[(n // 2) % 4]
        dt = torch.bfloat16 if n % 3 else torch.float32
        X = dev_bf16(wl.draw_activations(rng, T, K))
        v, i = nm.nm_pack(dev_bf16(wl.draw_weights(rng, O, K)), N, M)
        bias = torch.from_numpy(rng.standard_normal(O).astype(np.float32)).cuda() if n % 2 else None
        singles.append(nm.nm_linear_forward(v, i, K, N, M, X, bias=bias, out_dtype=dt, from_packed=True))
        outs.append(torch.zeros((T, O), dtype=dt, device="cuda"))
        layers.append((v, i, K, N, M, X, None, bias, outs[-1]))
    nm.nm_linear_forward_prepared_batched(layers)
    for n, (a, b) in enumerate(zip(outs, singles)):
        assert torch.equal(a, b), n


def test_batch_one_stack_against_the_checker():
    # the 48 linears of the model at one image (197 tokens), one batched call without workspaces, every output
    # element (the 2:4 layers of the draw need none and take the tiled kernel)
    stack = list(wl.draw_layers(wl.deit_b_stack(batch=1), seed=0))
    layers, outs = [], []
    for (L, X, W) in stack:
        v, i = nm.nm_pack(dev_bf16(W), L.N, L.M)
        outs.append(torch.zeros((L.T, L.O), dtype=torch.bfloat16, device="cuda"))
        layers.append((v, i, L.K, L.N, L.M, dev_bf16(X), None, None, outs[-1]))
    nm.nm_linear_forward_prepared_batched(layers)
    for (L, X, W), y in zip(stack, outs):
        Yref, B = orc.nm_linear_from_bits(X, W, L.N, L.M)
        check_output(host_output(y), Yref, B, L.K // L.M * L.N, False, L.name)
