"""GPU parity: the HIP library, called through its C ABI, against the CPU checker on the same seeded
inputs.  Masks, packed values and index words must be bit-exact; products within the stated tolerance."""
import numpy as np
import pytest
import torch

import paper_2409_09708_amd as nm
from oracle import nm_oracle as orc
from paper_2409_09708_amd import workloads as wl
from gpu_util import check_output, dev_bf16, dev_words, host_bits, host_output, host_words

pytestmark = pytest.mark.gpu

LEVELS = [(1, 4), (2, 4), (3, 4), (4, 4), (1, 8), (2, 8), (3, 8), (4, 8), (8, 8), (1, 16), (2, 16), (4, 16), (16, 16)]
BENCH_LEVELS = [(1, 4), (2, 4), (1, 8), (2, 8), (4, 8), (1, 16), (2, 16), (4, 16)]


def oracle_pack(W, N, M, mask=None):
    m = orc.nm_mask(W, N, M) if mask is None else mask
    vals, idx = orc.nm_pack(W, m, N, M)
    return m, vals, idx


def weights(rng, O, K, kind):
    return wl.tie_heavy_weights(rng, O, K) if kind == "ties" else wl.draw_weights(rng, O, K)


# ------------------------------------------------------------------ prune / pack / unpack

@pytest.mark.parametrize("N,M", LEVELS)
@pytest.mark.parametrize("kind", ["gauss", "ties"])
def test_prune_and_pack_bit_exact_streaming_shapes(N, M, kind):
    # contiguous, K % 32 == 0: the flat streaming kernels; 300 rows x 384 = 28 blocks with a ragged last one
    rng = np.random.default_rng(1000 + N * 17 + M)
    O, K = 301, 384
    W = weights(rng, O, K, kind)
    m, vals, idx = oracle_pack(W, N, M)
    Wd = dev_bf16(W)
    wm = torch.empty_like(Wd)
    mask = nm.nm_prune(Wd, N, M, W_masked=wm)
    assert np.array_equal(host_words(mask), orc.mask_to_words(m))
    assert np.array_equal(host_bits(wm), orc.apply_mask(W, m))
    v, i = nm.nm_pack(Wd, N, M)
    assert np.array_equal(host_bits(v), vals)
    assert np.array_equal(host_words(i), idx)
    # prune then pack with that mask writes the same bytes as the fused call
    v2, i2 = nm.nm_pack(Wd, N, M, mask=mask)
    assert torch.equal(v2.view(torch.int16), v.view(torch.int16)) and torch.equal(i2, i)
    # exact round trip
    back = nm.nm_unpack(v, i, K, N, M)
    assert np.array_equal(host_bits(back), orc.apply_mask(W, m))
    assert nm.nm_mask_check(mask, K, N, M) == 0


@pytest.mark.parametrize("N,M", LEVELS)
def test_prune_and_pack_bit_exact_general_shapes(N, M):
    # K not a multiple of 32, padded index rows, a leading dimension larger than K
    rng = np.random.default_rng(2000 + N * 17 + M)
    O, K = 23, 5 * M if M < 16 else 3 * M
    big = wl.tie_heavy_weights(rng, O, K + 16)
    W = np.ascontiguousarray(big[:, :K])
    m, vals, idx = oracle_pack(W, N, M)
    Wd = dev_bf16(big)[:, :K]  # ldw = K + 16
    mask = nm.nm_prune(Wd, N, M)
    assert np.array_equal(host_words(mask), orc.mask_to_words(m))
    v, i = nm.nm_pack(Wd, N, M)
    assert np.array_equal(host_bits(v), vals)
    assert np.array_equal(host_words(i), idx)
    v2, i2 = nm.nm_pack(Wd, N, M, mask=mask)
    assert torch.equal(v2.view(torch.int16), v.view(torch.int16)) and torch.equal(i2, i)
    back = nm.nm_unpack(v, i, K, N, M)
    assert np.array_equal(host_bits(back), orc.apply_mask(W, m))


def test_in_place_pruning():
    rng = np.random.default_rng(5)
    W = wl.draw_weights(rng, 64, 256)
    Wd = dev_bf16(W)
    nm.nm_prune(Wd, 2, 8, W_masked=Wd)
    assert np.array_equal(host_bits(Wd), orc.apply_mask(W, orc.nm_mask(W, 2, 8)))


@pytest.mark.parametrize("N,M", [(2, 4), (1, 8), (3, 8), (4, 16)])
@pytest.mark.parametrize("K", [256, 40 if False else 48])
def test_pack_with_a_callers_mask(N, M, K):
    # any saliency may produce the mask (Section 3.1): here a random legal one
    rng = np.random.default_rng(77 + N + M + K)
    O = 50
    W = wl.draw_weights(rng, O, K)
    m = np.zeros((O, K // M, M), dtype=bool)
    for o in range(O):
        for g in range(K // M):
            m[o, g, rng.choice(M, size=N, replace=False)] = True
    m = m.reshape(O, K)
    vals, idx = orc.nm_pack(W, m, N, M)
    mask_dev = dev_words(orc.mask_to_words(m))
    assert nm.nm_mask_check(mask_dev, K, N, M) == 0
    v, i = nm.nm_pack(dev_bf16(W), N, M, mask=mask_dev)
    assert np.array_equal(host_bits(v), vals) and np.array_equal(host_words(i), idx)


def test_mask_check_counts_bad_groups_and_pack_completes_them():
    rng = np.random.default_rng(9)
    O, K, N, M = 8, 64, 2, 4
    W = wl.draw_weights(rng, O, K)
    m = orc.nm_mask(W, N, M)
    m[0, 0:4] = [True, True, True, False]    # three set: the lowest two are used
    m[1, 4:8] = [False, False, True, False]  # one set: completed with the lowest unset position, value +0
    m[2, 8:12] = False                       # none set
    mask_dev = dev_words(orc.mask_to_words(m))
    assert nm.nm_mask_check(mask_dev, K, N, M) == 3
    v, i = nm.nm_pack(dev_bf16(W), N, M, mask=mask_dev)
    back = host_bits(nm.nm_unpack(v, i, K, N, M))
    expect = orc.apply_mask(W, m)
    expect[0, 2] = 0
    assert np.array_equal(back, expect)
    idx = host_words(i)
    assert (int(idx[0, 0]) & 0xF) == 0b0100          # positions 0,1
    assert ((int(idx[1, 0]) >> 4) & 0xF) == 0b1000   # positions 0 (filler),2
    assert ((int(idx[2, 0]) >> 8) & 0xF) == 0b0100   # positions 0,1 (fillers)


def test_pack_batched_equals_single_calls():
    rng = np.random.default_rng(13)
    specs = [(96, 128, 1, 4), (64, 256, 2, 4), (40, 384, 1, 8), (33, 128, 2, 8), (70, 256, 4, 8), (20, 512, 1, 16),
             (17, 256, 2, 16), (50, 128, 4, 16), (9, 40, 2, 8), (12, 128, 3, 8)]  # last two: per-matrix fallbacks
    Ws = [dev_bf16(wl.tie_heavy_weights(rng, O, K)) for (O, K, _, _) in specs]
    outs = nm.nm_pack_batched([(W, N, M) for W, (_, _, N, M) in zip(Ws, specs)])
    for W, (O, K, N, M), (v, i) in zip(Ws, specs, outs):
        v1, i1 = nm.nm_pack(W, N, M)
        assert torch.equal(v.view(torch.int16), v1.view(torch.int16)) and torch.equal(i, i1), (O, K, N, M)
        _, vals, idx = oracle_pack(host_bits(W), N, M)
        assert np.array_equal(host_bits(v), vals) and np.array_equal(host_words(i), idx)


def test_non_finite_weights_follow_the_key_order():
    W = np.array([[0x3F80, 0x7F80, 0x7FC0, 0x4000, 0x8000, 0x0000, 0x0001, 0x8001] * 4], dtype=np.uint16)
    W = np.repeat(W, 2, axis=0)
    for N, M in [(1, 4), (2, 4), (2, 8), (4, 8)]:
        m, vals, idx = oracle_pack(W, N, M)
        v, i = nm.nm_pack(dev_bf16(W), N, M)
        assert np.array_equal(host_bits(v), vals) and np.array_equal(host_words(i), idx)


# ------------------------------------------------------------------ sparse product

def run_layer(X, W, N, M, out_dtype, bias=None):
    v, i = nm.nm_pack(dev_bf16(W), N, M)
    b = None if bias is None else torch.from_numpy(bias).cuda()
    Y = nm.nm_linear_forward(v, i, W.shape[1], N, M, dev_bf16(X), bias=b, out_dtype=out_dtype)
    torch.cuda.synchronize()
    return Y


@pytest.mark.parametrize("N,M", LEVELS)
@pytest.mark.parametrize("out_dtype", [torch.float32, torch.bfloat16])
def test_spmm_parity_tiled_kernels(N, M, out_dtype):
    # several tiles in both directions with ragged tails: T = 3*197 = 591, O = 328, K = 320 (5 K steps)
    rng = np.random.default_rng(3000 + N * 17 + M)
    T, K, O = 591, 320, 328
    X = wl.draw_activations(rng, T, K)
    W = wl.draw_weights(rng, O, K)
    Yref, B = orc.nm_linear_from_bits(X, W, N, M)
    Y = host_output(run_layer(X, W, N, M, out_dtype))
    check_output(Y, Yref, B, K // M * N, out_dtype == torch.float32, (N, M))


@pytest.mark.parametrize("N,M", BENCH_LEVELS)
def test_spmm_parity_large_tile_path(N, M):
    # enough tiles (>= 256 of 256x256) to take the large-tile kernel, with ragged edges
    rng = np.random.default_rng(3500 + N * 17 + M)
    T, K, O = 16 * 256 + 37, 128, 16 * 256 + 36
    X = wl.draw_activations(rng, T, K)
    W = wl.draw_weights(rng, O, K)
    Yref, B = orc.nm_linear_from_bits(X, W, N, M)
    Y = host_output(run_layer(X, W, N, M, torch.float32))
    check_output(Y, Yref, B, K // M * N, True, (N, M))


@pytest.mark.parametrize("N,M", [(2, 4), (1, 8), (4, 8)])
def test_spmm_parity_large_tile_path_bf16_output(N, M):
    # the same path writing bfloat16: ragged in both directions (the last token tile is shifted back and stores
    # only its own rows; the last out-feature tile stores only its own columns), three K steps, with a bias
    rng = np.random.default_rng(3600 + N * 17 + M)
    T, K, O = 16 * 256 + 37, 192, 16 * 256 + 40
    X = wl.draw_activations(rng, T, K)
    W = wl.draw_weights(rng, O, K)
    bias = rng.standard_normal(O).astype(np.float32)
    Yref, B = orc.nm_linear_from_bits(X, W, N, M, bias=bias)
    v, i = nm.nm_pack(dev_bf16(W), N, M)
    out = torch.full((T + 2, O + 8), 7.0, dtype=torch.bfloat16, device="cuda")
    nm.nm_linear_forward(v, i, K, N, M, dev_bf16(X), bias=torch.from_numpy(bias).cuda(), out=out[1:T + 1, :O])
    check_output(host_output(out[1:T + 1, :O]), Yref, B + np.abs(bias)[None, :], K // M * N + 1, False, (N, M))
    guard = out.float()
    assert bool((guard[0] == 7).all()) and bool((guard[T + 1] == 7).all()) and bool((guard[:, O:] == 7).all())


@pytest.mark.parametrize("N,M", [(2, 4), (1, 8), (4, 8), (2, 16)])
def test_spmm_with_bias_and_strided_views(N, M):
    rng = np.random.default_rng(3700 + N + M)
    T, K, O = 200, 192, 136
    Xbig = wl.draw_activations(rng, T, K + 64)
    X = np.ascontiguousarray(Xbig[:, :K])
    W = wl.draw_weights(rng, O, K)
    bias = rng.standard_normal(O).astype(np.float32)
    Yref, B = orc.nm_linear_from_bits(X, W, N, M, bias=bias)
    B = B + np.abs(bias)[None, :]
    v, i = nm.nm_pack(dev_bf16(W), N, M)
    out_big = torch.zeros((T, O + 8), dtype=torch.float32, device="cuda")
    nm.nm_linear_forward(v, i, K, N, M, dev_bf16(Xbig)[:, :K], bias=torch.from_numpy(bias).cuda(), out=out_big[:, :O])
    Y = out_big.cpu().numpy().astype(np.float64)
    check_output(Y[:, :O], Yref, B, K // M * N + 1, True, (N, M))
    assert np.all(Y[:, O:] == 0)  # nothing written past the row


@pytest.mark.parametrize("N,M", [(1, 4), (2, 4), (3, 4), (2, 8), (3, 8), (4, 16), (16, 16)])
def test_spmm_parity_general_kernel(N, M):
    # K % 64 != 0 and odd O: the plain gather kernel
    rng = np.random.default_rng(4000 + N * 17 + M)
    T, K, O = 37, 3 * 16, 29
    X = wl.draw_activations(rng, T, K)
    W = wl.draw_weights(rng, O, K)
    Yref, B = orc.nm_linear_from_bits(X, W, N, M)
    for dt in (torch.float32, torch.bfloat16):
        Y = host_output(run_layer(X, W, N, M, dt))
        check_output(Y, Yref, B, K // M * N, dt == torch.float32, (N, M))


@pytest.mark.parametrize("N,M", BENCH_LEVELS + [(3, 8), (8, 8)])
def test_identity_activations_reproduce_the_masked_weight_exactly(N, M):
    # X = I  =>  Y = W_s^T exactly, also in bf16 output: ties the product to pack/unpack bit for bit
    rng = np.random.default_rng(4500 + N + M)
    K = O = 128
    W = wl.draw_weights(rng, O, K)
    X = wl.f32_to_bf16_bits(np.eye(K, dtype=np.float32))
    Ws = orc.apply_mask(W, orc.nm_mask(W, N, M))
    Y = run_layer(X, W, N, M, torch.bfloat16)
    def canon(b):  # -0 and +0 are the same value
        return np.where((b & 0x7FFF) == 0, np.uint16(0), b)

    assert np.array_equal(canon(host_bits(Y)), canon(Ws.T))
    Y32 = run_layer(X, W, N, M, torch.float32).cpu().numpy().astype(np.float64)
    assert np.array_equal(Y32, orc.bf16_bits_to_f64(Ws).T)


def test_config_single_2to4_linear():
    # X 197x384 ~N(0,1), W 384x384 ~N(0,0.02), 2:4, seed 0, fp32 out
    (L, X, W), = list(wl.draw_layers(wl.single_2to4(), seed=0))
    m, vals, idx = oracle_pack(W, 2, 4)
    v, i = nm.nm_pack(dev_bf16(W), 2, 4)
    assert np.array_equal(host_bits(v), vals) and np.array_equal(host_words(i), idx)
    Yref, B = orc.nm_linear(X, W, m)
    Y = nm.nm_spmm(v, i, L.K, 2, 4, dev_bf16(X))
    check_output(host_output(Y), Yref, B, L.K // 2, True, "config 1")


def test_small_batch_shapes():
    # batch 1 (197 tokens) DeiT-B fc1 / fc2 at 1:8 and 2:4
    for (L, X, W) in wl.draw_layers(wl.small_batch(), seed=0):
        Yref, B = orc.nm_linear_from_bits(X, W, L.N, L.M)
        for dt in (torch.float32, torch.bfloat16):
            Y = host_output(run_layer(X, W, L.N, L.M, dt))
            check_output(Y, Yref, B, L.K // L.M * L.N, dt == torch.float32, L.name)


def test_one_token_and_one_row_edges():
    rng = np.random.default_rng(8)
    for (T, K, O, N, M) in [(1, 64, 4, 2, 4), (3, 128, 1, 1, 8), (1, 16, 1, 4, 16), (17, 64, 20, 4, 8)]:
        X = wl.draw_activations(rng, T, K)
        W = wl.draw_weights(rng, O, K)
        Yref, B = orc.nm_linear_from_bits(X, W, N, M)
        Y = host_output(run_layer(X, W, N, M, torch.float32))
        check_output(Y, Yref, B, K // M * N, True, (T, K, O, N, M))


@pytest.mark.parametrize("N,M", [(2, 4), (1, 8), (2, 16), (4, 8), (3, 4), (8, 8)])
@pytest.mark.parametrize("shape", [(197, 3072, 768), (197, 768, 3072), (50, 1024, 200), (130, 704, 72), (16, 4096, 1024)])
def test_few_tokens_long_k(N, M, shape):
    # few output tiles and a long K (the batch-1 shapes of a transformer block and a decode-like one): the small
    # tiles over many more K steps than the load pipeline has stages (48, 12, 16, 11, 64), ragged in both
    # directions
    T, K, O = shape
    rng = np.random.default_rng(5200 + N * 17 + M + T + O)
    X = wl.draw_activations(rng, T, K)
    W = wl.draw_weights(rng, O, K)
    bias = rng.standard_normal(O).astype(np.float32)
    Yref, B = orc.nm_linear_from_bits(X, W, N, M, bias=bias)
    B = B + np.abs(bias)[None, :]
    Xd, bd = dev_bf16(X), torch.from_numpy(bias).cuda()
    v, i = nm.nm_pack(dev_bf16(W), N, M)
    whole = nm.nm_linear_forward(v, i, K, N, M, Xd, bias=bd)
    check_output(host_output(whole), Yref, B, K // M * N + 1, True, (N, M, shape))
    ws = nm.nm_spmm_prepare(v, i, K, N, M, T)
    for _ in range(2):
        assert torch.equal(whole, nm.nm_linear_forward_prepared(v, i, K, N, M, Xd, ws, bias=bd))
    y16 = nm.nm_linear_forward_prepared(v, i, K, N, M, Xd, ws, bias=bd, out_dtype=torch.bfloat16)
    check_output(host_output(y16), Yref, B, K // M * N + 1, False, (N, M, shape))
    # an output view whose rows do not split into 16-byte pieces takes the element-wise write-out
    wide = torch.zeros((T, O + 3), dtype=torch.float32, device="cuda")
    nm.nm_linear_forward_prepared(v, i, K, N, M, Xd, ws, bias=bd, out=wide[:, 1:O + 1])
    assert torch.equal(wide[:, 1:O + 1], whole)
    assert int(wide[:, 0].count_nonzero()) == 0 and int(wide[:, O + 1:].count_nonzero()) == 0


@pytest.mark.parametrize("N,M", [(2, 4), (1, 4), (2, 8), (1, 16), (4, 8), (8, 8)])
def test_prepare_then_prepared_equals_the_single_call(N, M):
    rng = np.random.default_rng(4700 + N + M)
    T, K, O = 300, 256, 272
    X = dev_bf16(wl.draw_activations(rng, T, K))
    v, i = nm.nm_pack(dev_bf16(wl.draw_weights(rng, O, K)), N, M)
    bias = torch.from_numpy(rng.standard_normal(O).astype(np.float32)).cuda()
    whole = nm.nm_linear_forward(v, i, K, N, M, X, bias=bias)
    ws = nm.nm_spmm_prepare(v, i, K, N, M, T)
    assert (ws is None) == (nm.nm_spmm_workspace_bytes(O, K, N, M, T) == 0)
    snapshot = None if ws is None else ws.clone()
    for _ in range(2):  # the prepared workspace serves any number of calls and is not modified
        part = nm.nm_linear_forward_prepared(v, i, K, N, M, X, ws, bias=bias)
        assert torch.equal(whole, part)
    if ws is not None:
        assert torch.equal(ws, snapshot)


def test_batched_call_groups_small_products_into_shared_launches():
    # Products too small for the persistent kernel: the batched call runs all layers of one operand form and tile
    # size in one launch of the tiled kernel.  Both forms and both tile sizes, levels with and without a workspace,
    # bias, both output types, ragged shapes, an unaligned output view (element-wise write-out), more layers than
    # one launch's table holds (40 of one class), and a layer the gather kernel takes.  Every output must hold the
    # bytes of the single call, and one layer of each class is checked against the oracle.
    rng = np.random.default_rng(5151)
    specs = []  # (T, K, O, N, M, out dtype, bias)
    for n in range(40):  # 2:4 form, 64 x 64 tiles
        specs.append((197 if n % 2 else 50 + n, 64 * (1 + n % 5), 64 + 24 * (n % 7), (1, 2)[n % 2], (4, 8, 16)[n % 3],
                      torch.bfloat16 if n % 3 else torch.float32, n % 4 == 0))
    specs += [(197, 768, 3072, 2, 4, torch.bfloat16, False), (197, 3072, 768, 1, 8, torch.float32, True),   # batch-1 block
              (197, 768, 768, 4, 8, torch.bfloat16, True), (130, 704, 72, 3, 4, torch.float32, False),      # dense form, 64 x 64
              (197, 256, 200, 8, 8, torch.bfloat16, False),
              (2048, 128, 2048, 2, 8, torch.bfloat16, False), (2048, 192, 2048, 2, 4, torch.float32, True),  # 128 x 128 tiles
              (2048, 128, 2048, 4, 16, torch.bfloat16, True),
              (64, 48, 40, 1, 8, torch.float32, False)]                                                       # gather kernel
    entries, singles, keep = [], [], {}
    for n, (T, K, O, N, M, dt, with_bias) in enumerate(specs):
        Xh, Wh = wl.draw_activations(rng, T, K), wl.draw_weights(rng, O, K)
        X = dev_bf16(Xh)
        v, i = nm.nm_pack(dev_bf16(Wh), N, M)
        ws = nm.nm_spmm_prepare(v, i, K, N, M, T)
        bh = rng.standard_normal(O).astype(np.float32) if with_bias else None
        bias = torch.from_numpy(bh).cuda() if with_bias else None
        singles.append(nm.nm_linear_forward_prepared(v, i, K, N, M, X, ws, bias=bias, out_dtype=dt))
        entries.append((v, i, K, N, M, X, ws, bias, torch.zeros((T, O), dtype=dt, device="cuda")))
        if n in (1, 40, 41, 42, 45, 47):
            keep[n] = (Xh, Wh, bh)
    # an output view whose rows are not whole 16-byte pieces
    T, K, O, N, M = 100, 128, 70, 2, 4
    X = dev_bf16(wl.draw_activations(rng, T, K))
    v, i = nm.nm_pack(dev_bf16(wl.draw_weights(rng, O, K)), N, M)
    singles.append(nm.nm_linear_forward_prepared(v, i, K, N, M, X, None))
    wide = torch.zeros((T, O + 3), dtype=torch.float32, device="cuda")
    entries.append((v, i, K, N, M, X, None, None, wide[:, 1:O + 1]))
    nm.nm_linear_forward_prepared_batched(entries)
    torch.cuda.synchronize()
    for n, (e, ref) in enumerate(zip(entries, singles)):
        if n < len(specs) and specs[n][1] >= 1024 and specs[n][0] <= 208:
            # few tiles and a long K: alone the reduction is cut into ranges, inside this call (which fills the
            # chip) it is not; same sums in another order
            tol = 2.0 ** -7 if e[-1].dtype == torch.bfloat16 else 2.0 ** -18
            scale = ref.float().abs().max().item()
            assert (e[-1].float() - ref.float()).abs().max().item() <= tol * scale, (n, specs[n])
            continue
        assert torch.equal(e[-1], ref), (n, specs[n] if n < len(specs) else "view")
    assert int(wide[:, 0].count_nonzero()) == 0 and int(wide[:, O + 1:].count_nonzero()) == 0
    # a call with few small layers keeps their own (smaller) tiles: same bytes again
    few = entries[:6] + entries[40:43]
    for e in few:
        e[-1].zero_()
    nm.nm_linear_forward_prepared_batched(few)
    for e, ref in zip(few, singles[:6] + singles[40:43]):
        assert torch.equal(e[-1], ref)
    for n, (Xh, Wh, bh) in keep.items():
        T, K, O, N, M, dt, _ = specs[n]
        Yref, B = orc.nm_linear_from_bits(Xh, Wh, N, M, bias=bh)
        if bh is not None:
            B = B + np.abs(bh)[None, :]  # the bias is one more term of the sum (it dominates these short sums)
        check_output(host_output(entries[n][-1]), Yref, B, K // M * N + 1, dt == torch.float32, specs[n])
