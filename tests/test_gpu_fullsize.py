"""Parity at the benchmark's full sizes, in the launch configuration bench.py times (bf16 output, one fused
pack + operand-order launch, one batched product call): packed bytes and every output element of one layer per
(shape, operand form) are compared with the CPU checker; further full-size cases on sampled token rows that the
checker computes directly (first tile, last ragged tile, random rows)."""
import zlib

import numpy as np
import pytest
import torch

import paper_2409_09708_amd as nm
from oracle import nm_oracle as orc
from paper_2409_09708_amd import workloads as wl
from gpu_util import check_output, dev_bf16, host_bits, host_output, host_words

pytestmark = pytest.mark.gpu


def sample_rows(T, rng, n=16):
    rows = np.concatenate([np.arange(0, n), np.arange(T - n, T), rng.integers(n, T - n, size=n)])
    return np.unique(rows)


def check_layer_sampled(L, X, W, out_dtype, rng):
    mask = orc.nm_mask(W, L.N, L.M)
    vals, idx = orc.nm_pack(W, mask, L.N, L.M)
    v, i = nm.nm_pack(dev_bf16(W), L.N, L.M)
    assert np.array_equal(host_bits(v), vals), L
    assert np.array_equal(host_words(i), idx), L
    Y = nm.nm_spmm(v, i, L.K, L.N, L.M, dev_bf16(X), out_dtype=out_dtype)
    rows = sample_rows(L.T, rng)
    Yref, B = orc.nm_linear(X[rows], W, mask)
    Ys = host_output(Y[torch.from_numpy(rows).cuda()])
    return check_output(Ys, Yref, B, L.K // L.M * L.N, out_dtype == torch.float32, str(L))


DEIT_B256 = [  # (name, K, O, level): every level of the batch-256 configuration on every layer shape it can meet
    ("qkv", 768, 2304, (1, 16)), ("qkv", 768, 2304, (4, 8)), ("proj", 768, 768, (2, 8)), ("proj", 768, 768, (4, 16)),
    ("fc1", 768, 3072, (1, 4)), ("fc1", 768, 3072, (2, 4)), ("fc2", 3072, 768, (2, 4)), ("fc2", 3072, 768, (1, 8)),
]


def check_layer_whole(L, X, W, Y_host, chunk=4096):
    """Every element of a layer's output against the checker, in chunks of token rows (bounds the fp64 memory)."""
    mask = orc.nm_mask(W, L.N, L.M)
    worst = 0.0
    for r0 in range(0, L.T, chunk):
        r1 = min(L.T, r0 + chunk)
        Yref, B = orc.nm_linear(X[r0:r1], W, mask)
        ratio, _ = check_output(orc.bf16_bits_to_f64(Y_host[r0:r1]), Yref, B, L.K // L.M * L.N, False, f"{L} rows {r0}..{r1}")
        worst = max(worst, ratio)
    return worst


@pytest.fixture(scope="module")
def batch256_step_outputs():
    """The benchmark step's launch configuration on one layer per (shape, operand form) of the batch-256 stack:
    one fused pack + operand-order launch, then ONE batched product call for all eight (the 2:4-form layers share
    a launch of the persistent kernel, the dense-form layers another).  Outputs start as NaN, so a tile that is
    never written fails.  Returns the host copies."""
    T = 256 * 197
    layers, xs, ws_host = [], [], []
    for name, K, O, level in DEIT_B256:
        rng = np.random.default_rng(zlib.crc32(f"{name}-{level}".encode()))
        layers.append(wl.Layer(name, T, K, O, *level))
        xs.append(wl.draw_activations(rng, T, K))
        ws_host.append(wl.draw_weights(rng, O, K))
    Wd = [dev_bf16(W) for W in ws_host]
    Xd = [dev_bf16(X) for X in xs]
    packed, wss = nm.nm_pack_prepare_batched([(W, L.N, L.M, L.T) for W, L in zip(Wd, layers)])
    Ys = [torch.full((L.T, L.O), float("nan"), dtype=torch.bfloat16, device="cuda") for L in layers]
    nm.nm_linear_forward_prepared_batched([(v, i, L.K, L.N, L.M, X, ws, None, Y)
                                           for L, (v, i), X, ws, Y in zip(layers, packed, Xd, wss, Ys)])
    torch.cuda.synchronize()
    out = {}
    for (name, K, O, level), L, X, W, (v, i), Y in zip(DEIT_B256, layers, xs, ws_host, packed, Ys):
        out[(name, level)] = (L, X, W, host_bits(v), host_words(i), host_bits(Y))
    return out


@pytest.mark.parametrize("name,K,O,level", DEIT_B256)
def test_deit_b_batch256_step_launch_every_element(batch256_step_outputs, name, K, O, level):
    L, X, W, v, i, Y = batch256_step_outputs[(name, level)]
    vals, idx = orc.nm_pack(W, orc.nm_mask(W, L.N, L.M), L.N, L.M)
    assert np.array_equal(v, vals) and np.array_equal(i, idx), L
    check_layer_whole(L, X, W, Y)


def test_deit_b_batch256_fp32_output_sampled():
    rng = np.random.default_rng(77)
    L = wl.Layer("proj", 256 * 197, 768, 768, 2, 4)
    check_layer_sampled(L, wl.draw_activations(rng, L.T, L.K), wl.draw_weights(rng, L.O, L.K), torch.float32, rng)


@pytest.mark.parametrize("level,O,out_dtype", [((2, 4), 3072, torch.bfloat16), ((1, 8), 3000, torch.float32),
                                               ((4, 8), 2304, torch.bfloat16), ((3, 4), 1000, torch.float32)])
def test_linear_forward_with_bias_at_batch256(level, O, out_dtype):
    # bias on the large-tile kernels, sparse and dense operand forms, whole and ragged out-feature tiles
    T, K = 256 * 197, 768
    rng = np.random.default_rng(zlib.crc32(f"bias-{level}-{O}".encode()))
    X, W = wl.draw_activations(rng, T, K), wl.draw_weights(rng, O, K)
    bias = rng.standard_normal(O).astype(np.float32)
    v, i = nm.nm_pack(dev_bf16(W), *level)
    Y = nm.nm_linear_forward(v, i, K, *level, dev_bf16(X), bias=torch.from_numpy(bias).cuda(), out_dtype=out_dtype)
    rows = sample_rows(T, rng)
    Yref, B = orc.nm_linear_from_bits(X[rows], W, *level, bias=bias)
    Ys = host_output(Y[torch.from_numpy(rows).cuda()])
    check_output(Ys, Yref, B + np.abs(bias)[None, :], K // level[1] * level[0] + 1, out_dtype == torch.float32,
                 f"{level} O={O}")


def test_deit_b_block_batch64_seeded_levels():
    # the four linears of one block at 12608 tokens, levels drawn with seed 0 (4:8, 2:8, 1:8, 2:4)
    rng = np.random.default_rng(5)
    layers = wl.deit_b_block(batch=64, seed=0)
    assert [(L.N, L.M) for L in layers] == [(4, 8), (2, 8), (1, 8), (2, 4)]
    for L, X, W in wl.draw_layers(layers, seed=0):
        check_layer_sampled(L, X, W, torch.bfloat16, rng)


def test_swin_b_stage_shapes_sampled():
    # one block per stage at batch 64: 200704 / 50176 / 12544 / 3136 tokens, widths 128 / 256 / 512 / 1024
    rng = np.random.default_rng(6)
    layers = wl.swin_b_stages(batch=64, seed=0)
    picks = [layers[0], layers[3], layers[6], layers[9], layers[12], layers[15]]  # qkv/fc2 of stage 0, fc1 s1, proj s2, qkv/fc2 s3
    for L, X, W in wl.draw_layers(picks, seed=1):
        check_layer_sampled(L, X, W, torch.bfloat16, rng)


def test_batched_pack_of_the_whole_stack_matches_single_calls_and_the_checker():
    # all 48 DeiT-B weights in one launch, as the benchmark does; every matrix equals its single-call result,
    # and one matrix per level is compared with the CPU checker in full
    layers = wl.deit_b_stack(batch=256, seed=0)
    rng = np.random.default_rng(0)
    Ws = [dev_bf16(wl.draw_weights(rng, L.O, L.K)) for L in layers]
    outs = nm.nm_pack_batched([(W, L.N, L.M) for W, L in zip(Ws, layers)])
    seen = set()
    for W, L, (v, i) in zip(Ws, layers, outs):
        v1, i1 = nm.nm_pack(W, L.N, L.M)
        assert torch.equal(v.view(torch.int16), v1.view(torch.int16)) and torch.equal(i, i1), L
        if (L.N, L.M) not in seen:
            seen.add((L.N, L.M))
            Wh = host_bits(W)
            vals, idx = orc.nm_pack(Wh, orc.nm_mask(Wh, L.N, L.M), L.N, L.M)
            assert np.array_equal(host_bits(v), vals) and np.array_equal(host_words(i), idx), L
    assert len(seen) == 7


def test_pack_prepare_batched_writes_what_the_two_calls_write():
    # one block of DeiT-B at 50432 tokens (stream-order workspaces: 2:4 form and dense form), a layer with a
    # ragged number of rows and a small layer (row-major workspace): packed bytes and workspaces must be
    # identical to nm_pack + nm_spmm_prepare, and the prepared product must match the checker
    rng = np.random.default_rng(99)
    T = 256 * 197
    shapes = [(2304, 768, 1, 16), (768, 768, 4, 8), (3072, 768, 2, 8), (768, 3072, 2, 4), (3000, 768, 1, 4),
              (768, 768, 4, 16), (384, 384, 1, 8)]
    Ts = [T, T, T, T, T, T, 197]
    Ws = [wl.draw_weights(rng, O, K) for O, K, _, _ in shapes]
    Wd = [dev_bf16(W) for W in Ws]
    outs, wss = nm.nm_pack_prepare_batched([(w, N, M, t) for w, (_, _, N, M), t in zip(Wd, shapes, Ts)])
    for (O, K, N, M), t, w, (v, i), ws in zip(shapes, Ts, Wd, outs, wss):
        v2, i2 = nm.nm_pack(w, N, M)
        assert torch.equal(v.view(torch.int16), v2.view(torch.int16)) and torch.equal(i, i2), (O, K, N, M)
        ws2 = nm.nm_spmm_prepare(v2, i2, K, N, M, t)
        assert (ws is None) == (ws2 is None), (O, K, N, M)
        if ws is not None:
            assert torch.equal(ws, ws2), (O, K, N, M)
    # product through the fused preparation, checked on sampled rows
    for idx in (3, 1):
        O, K, N, M = shapes[idx]
        X = wl.draw_activations(rng, T, K)
        Y = nm.nm_linear_forward_prepared(outs[idx][0], outs[idx][1], K, N, M, dev_bf16(X), wss[idx],
                                          out_dtype=torch.bfloat16)
        rows = sample_rows(T, rng)
        Yref, B = orc.nm_linear_from_bits(X[rows], Ws[idx], N, M)
        check_output(host_output(Y[torch.from_numpy(rows).cuda()]), Yref, B, K // M * N, False, str(shapes[idx]))


@pytest.mark.parametrize("K,level,out_dtype", [(64, (2, 4), torch.float32), (192, (1, 8), torch.bfloat16),
                                               (192, (4, 8), torch.float32), (320, (2, 16), torch.bfloat16)])
def test_persistent_kernel_short_and_odd_reductions(K, level, out_dtype):
    # one, three and five K steps per tile (the step loop runs in pairs), a ragged last token tile and a
    # ragged out-feature tile, with bias: 2 x 129 tiles put the layer on the persistent kernel
    rng = np.random.default_rng(zlib.crc32(f"short-{K}-{level}".encode()))
    T, O = 128 * 256 + 37, 504
    X, W = wl.draw_activations(rng, T, K), wl.draw_weights(rng, O, K)
    bias = rng.standard_normal(O).astype(np.float32)
    v, i = nm.nm_pack(dev_bf16(W), *level)
    Y = nm.nm_linear_forward(v, i, K, *level, dev_bf16(X), bias=torch.from_numpy(bias).cuda(), out_dtype=out_dtype)
    rows = sample_rows(T, rng, n=40)
    Yref, B = orc.nm_linear_from_bits(X[rows], W, *level, bias=bias)
    check_output(host_output(Y[torch.from_numpy(rows).cuda()]), Yref, B + np.abs(bias)[None, :],
                 K // level[1] * level[0] + 1, out_dtype == torch.float32, f"K={K} {level}")


def test_batched_products_equal_the_single_calls():
    # the stack's launch configuration: all products of a block in one call.  Layers of both operand forms, with
    # different K (12 and 48 steps, and 24 / 96 for the dense form), a ragged out-feature tile, a bias, fp32 and
    # bf16 outputs; plus a layer too small for the persistent kernel and one the general kernel takes.  The
    # batched call must write the bytes the single calls write.
    rng = np.random.default_rng(4242)
    T = 256 * 197
    specs = [(768, 768, 2, 4, torch.bfloat16, False), (768, 3000, 1, 8, torch.bfloat16, True),
             (3072, 768, 2, 8, torch.float32, False), (768, 2304, 4, 8, torch.bfloat16, False),
             (3072, 768, 4, 16, torch.bfloat16, True), (768, 768, 1, 16, torch.bfloat16, False)]
    entries, singles = [], []
    for (K, O, N, M, dt, with_bias) in specs:
        X = dev_bf16(wl.draw_activations(rng, T, K))
        v, i = nm.nm_pack(dev_bf16(wl.draw_weights(rng, O, K)), N, M)
        ws = nm.nm_spmm_prepare(v, i, K, N, M, T)
        bias = torch.from_numpy(rng.standard_normal(O).astype(np.float32)).cuda() if with_bias else None
        singles.append(nm.nm_linear_forward_prepared(v, i, K, N, M, X, ws, bias=bias, out_dtype=dt))
        entries.append((v, i, K, N, M, X, ws, bias, torch.zeros((T, O), dtype=dt, device="cuda")))
    # a few tokens only (tiled kernel) and K not a multiple of 64 (general kernel)
    for (Ts, K, O, N, M) in [(197, 768, 768, 2, 4), (64, 48, 40, 1, 8)]:
        X = dev_bf16(wl.draw_activations(rng, Ts, K))
        v, i = nm.nm_pack(dev_bf16(wl.draw_weights(rng, O, K)), N, M)
        ws = nm.nm_spmm_prepare(v, i, K, N, M, Ts)
        singles.append(nm.nm_linear_forward_prepared(v, i, K, N, M, X, ws))
        entries.append((v, i, K, N, M, X, ws, None, torch.zeros((Ts, O), dtype=torch.float32, device="cuda")))
    nm.nm_linear_forward_prepared_batched(entries)
    torch.cuda.synchronize()
    for e, ref in zip(entries, singles):
        assert torch.equal(e[-1], ref)
    # and again through a prebuilt descriptor array (what a serving loop keeps)
    for e in entries:
        e[-1].zero_()
    descs = nm.forward_descs(entries)
    nm.nm_linear_forward_prepared_batched(descs)
    for e, ref in zip(entries, singles):
        assert torch.equal(e[-1], ref)


def test_batched_call_with_more_layers_than_one_launch_holds():
    # 50 layers of the 2:4 form that all take the persistent kernel (256 tiles each): the table of a launch holds
    # fewer, so the call flushes it and starts another; shallow K (three steps), one shared input
    rng = np.random.default_rng(777)
    T, K, O = 65536, 192, 256
    X = dev_bf16(wl.draw_activations(rng, T, K))
    entries, singles = [], []
    for n in range(50):
        N, M = ((2, 4), (1, 4), (2, 8), (1, 16))[n % 4]
        v, i = nm.nm_pack(dev_bf16(wl.draw_weights(rng, O, K)), N, M)
        ws = nm.nm_spmm_prepare(v, i, K, N, M, T)
        entries.append((v, i, K, N, M, X, ws, None, torch.zeros((T, O), dtype=torch.bfloat16, device="cuda")))
        if n % 7 == 0:
            singles.append((n, nm.nm_linear_forward_prepared(v, i, K, N, M, X, ws, out_dtype=torch.bfloat16)))
    nm.nm_linear_forward_prepared_batched(entries)
    torch.cuda.synchronize()
    for n, ref in singles:
        assert torch.equal(entries[n][-1], ref), n
    for e in entries:  # every output was written (no layer fell between two launches)
        assert int(e[-1][::4099].count_nonzero()) > 0
