"""GPU parity of the int8 layer (Section 4, Table 6: 8-bit quantisation on top of the sparse networks): the
integer sums from the HIP library must equal the CPU checker's bit for bit; the rescaled outputs within the
rounding of one fp32 multiply-add (and of the bfloat16 store)."""
import numpy as np
import pytest
import torch

import paper_2409_09708_amd as nm
from oracle import nm_int8_oracle as q
from oracle import nm_oracle as orc
from paper_2409_09708_amd import workloads as wl
from gpu_util import dev_bf16, dev_words, host_output

pytestmark = pytest.mark.gpu

LEVELS = [(1, 4), (2, 4), (3, 4), (1, 8), (2, 8), (4, 8), (8, 8), (1, 16), (2, 16), (4, 16)]


def random_mask(rng, O, K, N, M):
    keys = rng.random((O, K // M, M))
    order = np.argsort(keys, axis=2)
    m = np.zeros((O, K // M, M), dtype=bool)
    np.put_along_axis(m, order[:, :, :N], True, axis=2)
    return m.reshape(O, K)


def magnitude_mask(wq, N, M):
    """Mask of the float weight the integers stand for (integers up to 127 are exact in bfloat16)."""
    return orc.nm_mask(wl.f32_to_bf16_bits(wq.astype(np.float32)), N, M)


def dev_i8(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def check_scaled(Y, Yref, acc, scale_row, bias, bf16_out, what):
    # fp32: one product x_scale * w_scale, one conversion of the integer and one fused multiply-add
    mag = np.abs(acc) * np.abs(scale_row)[None, :] + (0 if bias is None else np.abs(bias)[None, :])
    tol = mag * (2.0 ** -22 + (2.0 ** -8 if bf16_out else 0.0)) + 1e-30
    err = np.abs(Y - Yref)
    assert np.all(err <= tol), (what, float((err / tol).max()))


@pytest.mark.parametrize("N,M", LEVELS)
@pytest.mark.parametrize("mask_kind", ["magnitude", "random"])
def test_integer_sums_bit_exact_tiled(N, M, mask_kind):
    # several tiles with ragged edges: T = 591, O = 328, K = 384 (three K steps)
    rng = np.random.default_rng(7000 + N * 17 + M)
    T, K, O = 591, 384, 328
    xq, wq = wl.draw_int8(rng, T, K), wl.draw_int8(rng, O, K)
    mask = magnitude_mask(wq, N, M) if mask_kind == "magnitude" else random_mask(rng, O, K, N, M)
    ref = q.nm_accumulate_i8(xq, wq, mask)
    words = dev_words(orc.mask_to_words(mask))
    acc = nm.nm_linear_forward_i8(dev_i8(wq), words, N, M, dev_i8(xq), out_dtype=torch.int32)
    assert np.array_equal(acc.cpu().numpy().astype(np.int64), ref)


def test_mask_from_the_float_weights_pruning_call():
    # the quantisation flow: prune the float weight on the device, quantise (here: the integers themselves),
    # multiply with the mask words nm_prune wrote
    rng = np.random.default_rng(7100)
    T, K, O, N, M = 200, 256, 136, 2, 8
    xq, wq = wl.draw_int8(rng, T, K), wl.draw_int8(rng, O, K)
    wf = dev_bf16(wl.f32_to_bf16_bits(wq.astype(np.float32)))
    words = nm.nm_prune(wf, N, M)
    acc = nm.nm_linear_forward_i8(dev_i8(wq), words, N, M, dev_i8(xq), out_dtype=torch.int32)
    assert np.array_equal(acc.cpu().numpy().astype(np.int64), q.nm_accumulate_i8(xq, wq, magnitude_mask(wq, N, M)))


@pytest.mark.parametrize("N,M", [(2, 4), (1, 8), (4, 8)])
@pytest.mark.parametrize("out_dtype", [torch.float32, torch.bfloat16])
def test_rescaled_outputs(N, M, out_dtype):
    rng = np.random.default_rng(7200 + N + M)
    T, K, O = 300, 256, 200
    xq, wq = wl.draw_int8(rng, T, K), wl.draw_int8(rng, O, K)
    mask = magnitude_mask(wq, N, M)
    x_scale = 0.0173
    w_scale = (0.001 + 0.002 * rng.random(O)).astype(np.float32)
    bias = rng.standard_normal(O).astype(np.float32)
    acc = q.nm_accumulate_i8(xq, wq, mask)
    x_scale32 = float(np.float32(x_scale))
    Yref = q.nm_linear_i8(xq, wq, mask, x_scale32, w_scale, bias)
    words = dev_words(orc.mask_to_words(mask))
    Y = nm.nm_linear_forward_i8(dev_i8(wq), words, N, M, dev_i8(xq), x_scale=x_scale, w_scale=torch.from_numpy(w_scale).cuda(),
                                bias=torch.from_numpy(bias).cuda(), out_dtype=out_dtype)
    check_scaled(host_output(Y), Yref, acc, x_scale32 * w_scale.astype(np.float64), bias, out_dtype == torch.bfloat16,
                 (N, M))
    # no scales, no bias: the integers as floats
    Y1 = nm.nm_linear_forward_i8(dev_i8(wq), words, N, M, dev_i8(xq), out_dtype=torch.float32)
    assert np.array_equal(Y1.cpu().numpy().astype(np.float64), acc.astype(np.float32).astype(np.float64))


@pytest.mark.parametrize("N,M", [(2, 4), (1, 16), (4, 8)])
@pytest.mark.parametrize("edge", [128, 256])
def test_large_tile_paths_and_prepared_calls(N, M, edge):
    # at least 256 tiles of 128 x 128, and of 256 x 256, with ragged edges (the two larger tile shapes); a prepared
    # workspace serves repeated products unchanged
    rng = np.random.default_rng(7300 + N + M + edge)
    T, K, O = 16 * edge + 37, 256, 16 * edge + 36
    xq, wq = wl.draw_int8(rng, T, K), wl.draw_int8(rng, O, K)
    mask = random_mask(rng, O, K, N, M)
    words = dev_words(orc.mask_to_words(mask))
    Wd, Xd = dev_i8(wq), dev_i8(xq)
    whole = nm.nm_linear_forward_i8(Wd, words, N, M, Xd, out_dtype=torch.int32)
    assert np.array_equal(whole.cpu().numpy().astype(np.int64), q.nm_accumulate_i8(xq, wq, mask))
    ws = nm.nm_i8_prepare(Wd, words, N, M, T)
    assert ws.numel() == nm.nm_i8_workspace_bytes(O, K, N, M, T)
    snapshot = ws.clone()
    for _ in range(2):
        assert torch.equal(nm.nm_linear_forward_i8_prepared(Wd, words, N, M, Xd, ws, out_dtype=torch.int32), whole)
    assert torch.equal(ws, snapshot)


@pytest.mark.parametrize("N,M,K", [(2, 4, 640), (2, 16, 640), (4, 8, 640), (8, 8, 640), (1, 8, 384), (4, 8, 384)])
def test_persistent_kernel_all_outputs(N, M, K):
    # enough 256 x 256 tiles and at least three K steps: the persistent kernel, operands in stream order.  Ragged
    # tiles in both directions, an odd and an even number of K steps, scales and bias through LDS, every output
    # type, a prepared workspace serving repeated calls
    rng = np.random.default_rng(7700 + N * 17 + M + K)
    T, O = 16 * 256 + 37, 16 * 256 + 36
    xq, wq = wl.draw_int8(rng, T, K), wl.draw_int8(rng, O, K)
    mask = random_mask(rng, O, K, N, M)
    words = dev_words(orc.mask_to_words(mask))
    Wd, Xd = dev_i8(wq), dev_i8(xq)
    acc = q.nm_accumulate_i8(xq, wq, mask)
    ws = nm.nm_i8_prepare(Wd, words, N, M, T)
    o_pad = 17 * 256
    assert ws.numel() == (o_pad * K // 2 + o_pad * K // 8 if N <= 2 else o_pad * K)
    snapshot = ws.clone()
    got = nm.nm_linear_forward_i8_prepared(Wd, words, N, M, Xd, ws, out_dtype=torch.int32)
    assert np.array_equal(got.cpu().numpy().astype(np.int64), acc)
    x_scale = 0.0173
    x_scale32 = float(np.float32(x_scale))
    w_scale = (0.001 + 0.002 * rng.random(O)).astype(np.float32)
    bias = rng.standard_normal(O).astype(np.float32)
    Yref = q.nm_linear_i8(xq, wq, mask, x_scale32, w_scale, bias)
    ws_d, b_d = torch.from_numpy(w_scale).cuda(), torch.from_numpy(bias).cuda()
    for dt in (torch.float32, torch.bfloat16):
        Y = nm.nm_linear_forward_i8_prepared(Wd, words, N, M, Xd, ws, x_scale=x_scale, w_scale=ws_d, bias=b_d, out_dtype=dt)
        check_scaled(host_output(Y), Yref, acc, x_scale32 * w_scale.astype(np.float64), bias, dt == torch.bfloat16, (N, M, K, dt))
    # scales without bias, bias without scales
    Y = nm.nm_linear_forward_i8_prepared(Wd, words, N, M, Xd, ws, x_scale=x_scale, w_scale=ws_d)
    check_scaled(host_output(Y), q.nm_linear_i8(xq, wq, mask, x_scale32, w_scale), acc, x_scale32 * w_scale.astype(np.float64),
                 None, False, "scale only")
    Y = nm.nm_linear_forward_i8_prepared(Wd, words, N, M, Xd, ws, bias=b_d)
    check_scaled(host_output(Y), q.nm_linear_i8(xq, wq, mask, 1.0, np.ones(O), bias), acc, np.ones(O), bias, False, "bias only")
    assert torch.equal(ws, snapshot)
    whole = nm.nm_linear_forward_i8(Wd, words, N, M, Xd, out_dtype=torch.int32)
    assert torch.equal(whole, got)


def test_pruned_positions_are_ignored_whatever_they_hold():
    rng = np.random.default_rng(7400)
    T, K, O = 70, 128, 72
    xq, wq = wl.draw_int8(rng, T, K), wl.draw_int8(rng, O, K)
    for (N, M) in [(1, 4), (4, 8)]:
        mask = random_mask(rng, O, K, N, M)
        dirty = wq.copy()
        dirty[~mask] = -128
        words = dev_words(orc.mask_to_words(mask))
        a = nm.nm_linear_forward_i8(dev_i8(wq), words, N, M, dev_i8(xq), out_dtype=torch.int32)
        b = nm.nm_linear_forward_i8(dev_i8(dirty), words, N, M, dev_i8(xq), out_dtype=torch.int32)
        assert torch.equal(a, b)
        assert np.array_equal(a.cpu().numpy().astype(np.int64), q.nm_accumulate_i8(xq, wq, mask))


def test_extreme_values_and_edges():
    # -128 everywhere over K = 1024 kept weights: 2^24 per output, far beyond int16; one token; one row
    K = 1024
    xq = np.full((1, K), -128, dtype=np.int8)
    wq = np.full((1, K), -128, dtype=np.int8)
    mask = np.ones((1, K), dtype=bool)
    acc = nm.nm_linear_forward_i8(dev_i8(wq), dev_words(orc.mask_to_words(mask)), 4, 4, dev_i8(xq), out_dtype=torch.int32)
    assert int(acc[0, 0]) == 128 * 128 * K


def test_general_shapes_and_views():
    # K not a multiple of 128, operands as views of wider buffers, an output view without 16-byte rows
    rng = np.random.default_rng(7500)
    for (T, K, O, N, M, pad) in [(33, 48, 20, 1, 8, 0), (65, 128, 40, 2, 4, 3), (65, 256, 40, 2, 4, 16), (9, 16, 3, 4, 16, 0)]:
        xq, wq = wl.draw_int8(rng, T, K), wl.draw_int8(rng, O, K)
        mask = random_mask(rng, O, K, N, M)
        ref = q.nm_accumulate_i8(xq, wq, mask)
        Wbig = torch.zeros((O, K + 16), dtype=torch.int8, device="cuda")
        Wbig[:, :K] = dev_i8(wq)
        Xbig = torch.zeros((T, K + 32), dtype=torch.int8, device="cuda")
        Xbig[:, :K] = dev_i8(xq)
        out = torch.full((T, O + 2 * pad + 1), 7, dtype=torch.int32, device="cuda")
        view = out[:, pad:pad + O]
        nm.nm_linear_forward_i8(Wbig[:, :K], dev_words(orc.mask_to_words(mask)), N, M, Xbig[:, :K], out=view)
        assert np.array_equal(view.cpu().numpy().astype(np.int64), ref), (T, K, O, N, M, pad)
        assert torch.all(out[:, :pad] == 7) and torch.all(out[:, pad + O:] == 7)


def test_deit_b_fc1_at_batch256_sampled():
    # T = 50432, 768 -> 3072 at 2:4 and 4:8 in the configuration the benchmark times (bfloat16 output is checked
    # through the exact integers of sampled token rows)
    T, K, O = 256 * 197, 768, 3072
    rng = np.random.default_rng(7600)
    xq, wq = wl.draw_int8(rng, T, K), wl.draw_int8(rng, O, K)
    Xd, Wd = dev_i8(xq), dev_i8(wq)
    rows = np.unique(np.concatenate([np.arange(16), np.arange(T - 16, T), rng.integers(16, T - 16, size=32)]))
    for (N, M) in [(2, 4), (4, 8)]:
        mask = magnitude_mask(wq, N, M)
        words = dev_words(orc.mask_to_words(mask))
        acc = nm.nm_linear_forward_i8(Wd, words, N, M, Xd, out_dtype=torch.int32)
        got = acc[torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.int64)
        assert np.array_equal(got, q.nm_accumulate_i8(xq[rows], wq, mask)), (N, M)


# ---- the compressed int8 form -----------------------------------------------------------------------------------

@pytest.mark.parametrize("N,M", LEVELS)
def test_pack_i8_bit_exact_and_round_trip(N, M):
    # values and index words against the checker; a K whose 3-bit index rows straddle words; unpack restores W (.) m
    rng = np.random.default_rng(7600 + N * 17 + M)
    O, K = 37, 480 if M != 16 else 512
    wq = wl.draw_int8(rng, O, K)
    wq[0, :M] = -128
    mask = random_mask(rng, O, K, N, M)
    vals, idx = q.nm_pack_i8(wq, mask, N, M)
    v, i = nm.nm_pack_i8(dev_i8(wq), dev_words(orc.mask_to_words(mask)), N, M)
    assert np.array_equal(v.cpu().numpy(), vals)
    assert np.array_equal(i.cpu().numpy().view(np.uint32), idx)
    back = nm.nm_unpack_i8(v, i, K, N, M)
    assert np.array_equal(back.cpu().numpy(), np.where(mask, wq, 0))


def test_pack_i8_from_a_strided_weight_view():
    rng = np.random.default_rng(7601)
    O, K, N, M = 20, 64, 2, 8
    big = wl.draw_int8(rng, O, K + 32)
    wq = big[:, :K]
    mask = random_mask(rng, O, K, N, M)
    v, i = nm.nm_pack_i8(dev_i8(big)[:, :K], dev_words(orc.mask_to_words(mask)), N, M)
    vals, idx = q.nm_pack_i8(np.ascontiguousarray(wq), mask, N, M)
    assert np.array_equal(v.cpu().numpy(), vals) and np.array_equal(i.cpu().numpy().view(np.uint32), idx)


@pytest.mark.parametrize("N,M", [(1, 4), (2, 4), (1, 8), (2, 8), (4, 8), (1, 16), (4, 16), (8, 8)])
@pytest.mark.parametrize("shape", ["tiled", "persistent", "general"])
def test_products_from_the_compressed_form(N, M, shape):
    # the same integers whether the weight comes dense + mask or compressed, on every kernel family, and equal to
    # the checker's; the prepared workspace is the same bytes from both sources
    rng = np.random.default_rng(7700 + N * 17 + M + len(shape))
    T, K, O = {"tiled": (300, 384, 200), "persistent": (129 * 256 - 3, 384, 500), "general": (50, 96, 40)}[shape]
    xq, wq = wl.draw_int8(rng, T, K), wl.draw_int8(rng, O, K)
    mask = random_mask(rng, O, K, N, M)
    words = dev_words(orc.mask_to_words(mask))
    Wd, Xd = dev_i8(wq), dev_i8(xq)
    v, i = nm.nm_pack_i8(Wd, words, N, M)
    acc_dense = nm.nm_linear_forward_i8(Wd, words, N, M, Xd, out_dtype=torch.int32)
    acc_packed = nm.nm_linear_forward_i8_packed(v, i, K, N, M, Xd, out_dtype=torch.int32)
    assert torch.equal(acc_dense, acc_packed)
    rows = np.unique(np.concatenate([np.arange(0, min(T, 40)), np.arange(max(0, T - 40), T)]))
    ref = q.nm_accumulate_i8(xq[rows], wq, mask)
    assert np.array_equal(acc_packed[torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.int64), ref)
    if nm.nm_i8_workspace_bytes(O, K, N, M, T):
        ws_d = nm.nm_i8_prepare(Wd, words, N, M, T)
        ws_p = nm.nm_i8_prepare_packed(v, i, K, N, M, T)
        assert torch.equal(ws_d, ws_p)
        y = nm.nm_linear_forward_i8_packed_prepared(v, i, K, N, M, Xd, ws_p, out_dtype=torch.int32)
        assert torch.equal(y, acc_dense)


def test_rescaled_output_from_the_compressed_form():
    rng = np.random.default_rng(7800)
    T, K, O, N, M = 257, 256, 264, 2, 8
    xq, wq = wl.draw_int8(rng, T, K), wl.draw_int8(rng, O, K)
    mask = magnitude_mask(wq, N, M)
    w_scale = (0.001 + 0.002 * rng.random(O)).astype(np.float32)
    bias = rng.standard_normal(O).astype(np.float32)
    v, i = nm.nm_pack_i8(dev_i8(wq), dev_words(orc.mask_to_words(mask)), N, M)
    Y = nm.nm_linear_forward_i8_packed(v, i, K, N, M, dev_i8(xq), x_scale=0.02, w_scale=torch.from_numpy(w_scale).cuda(),
                                       bias=torch.from_numpy(bias).cuda(), out_dtype=torch.float32)
    acc = q.nm_accumulate_i8(xq, wq, mask)
    Yref = q.nm_linear_i8(xq, wq, mask, np.float32(0.02), w_scale, bias)
    check_scaled(host_output(Y), Yref, acc, np.float32(0.02) * w_scale, bias, False, "packed int8")
