"""GPU parity of products whose reduction is cut into ranges (few output tiles, long K: one image through a wide
layer): partial sums + reduce launch against the CPU checker, the same bytes alone and inside a batched call, the
uncut product when the caller brings only the operand part of the workspace."""
import numpy as np
import pytest
import torch

import paper_2409_09708_amd as nm
from oracle import nm_oracle as orc
from paper_2409_09708_amd import workloads as wl
from gpu_util import check_output, dev_bf16, host_output

pytestmark = pytest.mark.gpu

# (T, K, O): a ViT-L fc2 at one image; a ViT-H-like fc2 at four images (128 x 128 tiles); a ragged one (O not a
# multiple of 4: element-wise partial rows; odd step count per range)
SHAPES = [(197, 4096, 1024), (788, 5120, 1280), (130, 4160, 90)]
LEVELS = [(2, 4), (1, 8), (4, 8), (2, 16), (8, 8)]


@pytest.mark.parametrize("N,M", LEVELS)
@pytest.mark.parametrize("shape", SHAPES)
def test_cut_reduction_against_the_checker(N, M, shape):
    T, K, O = shape
    rng = np.random.default_rng(9700 + N * 17 + M + T + K)
    X = wl.draw_activations(rng, T, K)
    W = wl.draw_weights(rng, O, K)
    bias = rng.standard_normal(O).astype(np.float32)
    Yref, B = orc.nm_linear_from_bits(X, W, N, M, bias=bias)
    B = B + np.abs(bias)[None, :]
    Xd, bd = dev_bf16(X), torch.from_numpy(bias).cuda()
    v, i = nm.nm_pack(dev_bf16(W), N, M)
    need = nm.nm_spmm_workspace_bytes(O, K, N, M, T)
    # the partial sums are part of the workspace: at least two ranges of T * O floats
    assert need >= 2 * T * O * 4, (need, shape)
    y32 = nm.nm_linear_forward(v, i, K, N, M, Xd, bias=bd)
    check_output(host_output(y32), Yref, B, K // M * N + 1, True, (N, M, shape))
    y16 = nm.nm_linear_forward(v, i, K, N, M, Xd, bias=bd, out_dtype=torch.bfloat16)
    check_output(host_output(y16), Yref, B, K // M * N + 1, False, (N, M, shape))
    # prepared: the same bytes; twice in a row (the partial sums are overwritten, never accumulated into)
    ws = nm.nm_spmm_prepare(v, i, K, N, M, T)
    for _ in range(2):
        assert torch.equal(y32, nm.nm_linear_forward_prepared(v, i, K, N, M, Xd, ws, bias=bd))
    # an output view of a wider buffer with guard columns
    wide = torch.full((T, O + 8), 7.0, dtype=torch.float32, device="cuda")
    nm.nm_linear_forward_prepared(v, i, K, N, M, Xd, ws, bias=bd, out=wide[:, 4:4 + O])
    assert torch.equal(wide[:, 4:4 + O], y32)
    assert torch.all(wide[:, :4] == 7.0) and torch.all(wide[:, 4 + O:] == 7.0)


def test_batched_call_cuts_the_same_way_as_single_calls():
    rng = np.random.default_rng(9800)
    layers, singles, outs = [], [], []
    # few tiles in all (the call keeps its tile sizes): the long layers are cut, the short one is not
    specs = [(197, 4096, 256, 2, 4), (197, 4096, 384, 1, 8), (64, 4160, 128, 4, 8), (197, 5120, 256, 1, 16),
             (197, 768, 256, 2, 4), (100, 4096, 132, 1, 4)]
    for n, (T, K, O, N, M) in enumerate(specs):
        dt = torch.bfloat16 if n % 2 else torch.float32
        X = dev_bf16(wl.draw_activations(rng, T, K))
        v, i = nm.nm_pack(dev_bf16(wl.draw_weights(rng, O, K)), N, M)
        bias = torch.from_numpy(rng.standard_normal(O).astype(np.float32)).cuda() if n % 3 else None
        ws = nm.nm_spmm_prepare(v, i, K, N, M, T)
        singles.append(nm.nm_linear_forward_prepared(v, i, K, N, M, X, ws, bias=bias, out_dtype=dt))
        ws2 = nm.nm_spmm_prepare(v, i, K, N, M, T)
        outs.append(torch.zeros((T, O), dtype=dt, device="cuda"))
        layers.append((v, i, K, N, M, X, ws2, bias, outs[-1]))
    nm.nm_linear_forward_prepared_batched(layers)
    for n, (a, b) in enumerate(zip(outs, singles)):
        assert torch.equal(a, b), (n, specs[n])


def test_operand_part_of_the_workspace_alone_gives_the_uncut_product():
    T, K, O, N, M = 197, 4096, 1024, 1, 8
    rng = np.random.default_rng(9900)
    X, W = wl.draw_activations(rng, T, K), wl.draw_weights(rng, O, K)
    Yref, B = orc.nm_linear_from_bits(X, W, N, M)
    v, i = nm.nm_pack(dev_bf16(W), N, M)
    full = nm.nm_spmm_workspace_bytes(O, K, N, M, T)
    operand = O * K + O * K // 8  # the 2:4-form copy of this layer
    assert full > operand
    small = torch.empty((operand,), dtype=torch.uint8, device="cuda")
    y = nm.nm_linear_forward(v, i, K, N, M, dev_bf16(X), workspace=small)
    check_output(host_output(y), Yref, B, K // M * N, True, "operand part only")
    y_cut = nm.nm_linear_forward(v, i, K, N, M, dev_bf16(X))
    check_output(host_output(y_cut), Yref, B, K // M * N, True, "full workspace")
