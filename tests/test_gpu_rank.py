"""GPU parity of the nested-level calls (ranks inside groups, Section 3 "Subset-Superset Relationship"):
ranks, the masks taken from them and the packed bytes taken from them must be bit-exact against the CPU
checker, and must agree with the library's own single-level calls."""
import numpy as np
import pytest
import torch

import paper_2409_09708_amd as nm
from oracle import nm_oracle as orc
from paper_2409_09708_amd import workloads as wl
from gpu_util import dev_bf16, host_bits, host_words

pytestmark = pytest.mark.gpu


def host_bytes(t):
    return t.contiguous().cpu().numpy()


@pytest.mark.parametrize("M", [4, 8, 16])
@pytest.mark.parametrize("kind", ["gauss", "ties"])
def test_rank_bit_exact_and_every_level_follows(M, kind):
    # contiguous: the fast kernels; 301 x 384 weights = 7224 chunks = 29 blocks with a ragged last one
    rng = np.random.default_rng(4000 + M)
    O, K = 301, 384
    W = wl.tie_heavy_weights(rng, O, K) if kind == "ties" else wl.draw_weights(rng, O, K)
    Wd = dev_bf16(W)
    rank = nm.nm_rank(Wd, M)
    assert rank.shape == (O, K // 2) and rank.numel() == nm.nm_rank_bytes(O, K)
    ref = orc.nm_rank(W, M)
    assert np.array_equal(host_bytes(rank), orc.rank_nibbles(ref))
    for N in sorted({1, 2, 3, M // 2, M}):
        mask = nm.nm_rank_mask(rank, K, N, M)
        m = orc.nm_mask(W, N, M)
        assert np.array_equal(host_words(mask), orc.mask_to_words(m)), (N, M)
        assert torch.equal(mask, nm.nm_prune(Wd, N, M))
        v, i = nm.nm_pack_ranked(Wd, rank, N, M)
        vals, idx = orc.nm_pack(W, m, N, M)
        assert np.array_equal(host_bits(v), vals), (N, M)
        assert np.array_equal(host_words(i), idx), (N, M)
        v2, i2 = nm.nm_pack(Wd, N, M)
        assert torch.equal(v.view(torch.int16), v2.view(torch.int16)) and torch.equal(i, i2)


@pytest.mark.parametrize("M", [4, 8, 16])
def test_rank_general_shapes(M):
    # K not a multiple of 32, a leading dimension larger than K, an unaligned start: the general kernels
    rng = np.random.default_rng(4100 + M)
    O, K = 23, 5 * M if M < 16 else 3 * M
    big = wl.tie_heavy_weights(rng, O, K + 16)
    W = np.ascontiguousarray(big[:, 8:8 + K])
    Wd = dev_bf16(big)[:, 8:8 + K]
    rank = nm.nm_rank(Wd, M)
    assert np.array_equal(host_bytes(rank), orc.rank_nibbles(orc.nm_rank(W, M)))
    for N in (1, 2, M):
        m = orc.nm_mask(W, N, M)
        assert np.array_equal(host_words(nm.nm_rank_mask(rank, K, N, M)), orc.mask_to_words(m))
        v, i = nm.nm_pack_ranked(Wd, rank, N, M)
        vals, idx = orc.nm_pack(W, m, N, M)
        assert np.array_equal(host_bits(v), vals) and np.array_equal(host_words(i), idx)


def test_rank_edge_values():
    # +-0, equal magnitudes of both signs, Inf and NaN patterns keep the order of the selection rule
    bits = np.array([[0x0000, 0x8000, 0x3F80, 0xBF80, 0x7F80, 0xFF80, 0x7FC0, 0x0001,
                      0x3F80, 0x3F80, 0x3F80, 0x3F80, 0x0000, 0x0000, 0x0000, 0x0000]], dtype=np.uint16)
    for M in (4, 8, 16):
        rank = nm.nm_rank(dev_bf16(bits), M)
        assert np.array_equal(host_bytes(rank), orc.rank_nibbles(orc.nm_rank(bits, M))), M


def test_rank_of_a_benchmark_matrix_serves_all_its_levels():
    # fc1 of DeiT-B (3072 x 768): one ranking per M, every level of the benchmark's set from it
    rng = np.random.default_rng(4200)
    W = wl.draw_weights(rng, 3072, 768)
    Wd = dev_bf16(W)
    for M, Ns in ((4, (1, 2)), (8, (1, 2, 4)), (16, (1, 2, 4))):
        rank = nm.nm_rank(Wd, M)
        assert np.array_equal(host_bytes(rank), orc.rank_nibbles(orc.nm_rank(W, M)))
        for N in Ns:
            v, i = nm.nm_pack_ranked(Wd, rank, N, M)
            v2, i2 = nm.nm_pack(Wd, N, M)
            assert torch.equal(v.view(torch.int16), v2.view(torch.int16)) and torch.equal(i, i2), (N, M)


def test_rank_batched_equals_single_calls():
    # a mix of shapes and group sizes, one of them not contiguous-friendly (goes through its own launch)
    rng = np.random.default_rng(4300)
    shapes = [(768, 768, 4), (2304, 768, 8), (301, 384, 16), (23, 40, 8), (3072, 768, 16)]
    Ws = [dev_bf16(wl.tie_heavy_weights(rng, O, K) if i % 2 else wl.draw_weights(rng, O, K))
          for i, (O, K, _) in enumerate(shapes)]
    ranks = nm.nm_rank_batched([(w, M) for w, (_, _, M) in zip(Ws, shapes)])
    for w, (O, K, M), r in zip(Ws, shapes, ranks):
        assert torch.equal(r, nm.nm_rank(w, M)), (O, K, M)
        assert np.array_equal(host_bytes(r), orc.rank_nibbles(orc.nm_rank(host_bits(w), M))), (O, K, M)


def test_pack_ranked_batched_equals_the_oracle_and_single_calls():
    # a sampled configuration packed from stored ranks in one call: fast-kernel shapes at the sampler's levels,
    # a level outside the batched kernel's set (3:8), a shape the fast kernel does not take (own launches),
    # and more matrices than one launch's table holds
    rng = np.random.default_rng(4400)
    specs = [(768, 768, 2, 4), (2304, 768, 1, 8), (301, 384, 4, 16), (23, 40, 2, 8), (3072, 768, 1, 16),
             (64, 128, 3, 8), (768, 3072, 4, 8), (128, 64, 1, 4), (96, 256, 2, 16)]
    specs += [(32 + 16 * (i % 3), 64, (1, 2)[i % 2], (4, 8, 16)[i % 3]) for i in range(60)]
    Wn = [wl.tie_heavy_weights(rng, O, K) if i % 2 else wl.draw_weights(rng, O, K)
          for i, (O, K, _, _) in enumerate(specs)]
    Ws = [dev_bf16(w) for w in Wn]
    ranks = nm.nm_rank_batched([(w, M) for w, (_, _, _, M) in zip(Ws, specs)])
    outs = nm.nm_pack_ranked_batched([(w, r, N, M) for w, r, (_, _, N, M) in zip(Ws, ranks, specs)])
    for n, (w, wd, r, (O, K, N, M), (v, i)) in enumerate(zip(Wn, Ws, ranks, specs, outs)):
        v1, i1 = nm.nm_pack_ranked(wd, r, N, M)
        assert torch.equal(v.view(torch.int16), v1.view(torch.int16)) and torch.equal(i, i1), (O, K, N, M)
        if n < 12:
            vals, idx = orc.nm_pack(w, orc.nm_mask(w, N, M), N, M)
            assert np.array_equal(host_bits(v), vals) and np.array_equal(host_words(i), idx), (O, K, N, M)


@pytest.mark.parametrize("N,M", [(1, 4), (2, 4), (3, 8), (4, 8), (4, 16), (16, 16)])
def test_mask_from_a_supplied_saliency(N, M):
    # Section 3.1: any saliency may rank the weights.  Random scores with many ties, signed zeros, infinities and
    # NaN; K not a multiple of 32; a leading dimension larger than the row
    rng = np.random.default_rng(900 + N + M)
    O, K = 37, 5 * M if M < 16 else 3 * M
    s = rng.integers(-4, 5, size=(O, K + 8)).astype(np.float32)
    s[rng.random(s.shape) < 0.05] = np.nan
    s[rng.random(s.shape) < 0.05] = -0.0
    s[rng.random(s.shape) < 0.03] = np.inf
    s[rng.random(s.shape) < 0.03] = -np.inf
    ref = orc.nm_mask_from_scores(s[:, :K], N, M)
    words = nm.nm_prune_scored(torch.from_numpy(s).cuda()[:, :K], N, M)
    assert np.array_equal(host_words(words), orc.mask_to_words(ref))
    assert nm.nm_mask_check(words, K, N, M) == 0


def test_taylor_saliency_mask_feeds_the_packing_call():
    # first-order Taylor saliency |w * g| (Section 3.1 names it as an alternative to the magnitude): the mask
    # it gives packs to the bytes the checker packs with the same mask, and with score = |w| it is nm_prune's mask
    rng = np.random.default_rng(901)
    O, K, N, M = 64, 256, 2, 8
    W = wl.draw_weights(rng, O, K)
    g = rng.standard_normal((O, K)).astype(np.float32)
    wf = orc.bf16_bits_to_f64(W).astype(np.float32)
    score = np.abs(wf * g)
    ref = orc.nm_mask_from_scores(score, N, M)
    words = nm.nm_prune_scored(torch.from_numpy(score).cuda(), N, M)
    assert np.array_equal(host_words(words), orc.mask_to_words(ref))
    v, i = nm.nm_pack(dev_bf16(W), N, M, mask=words)
    vals, idx = orc.nm_pack(W, ref, N, M)
    assert np.array_equal(host_bits(v), vals) and np.array_equal(host_words(i), idx)
    same = nm.nm_prune_scored(torch.from_numpy(np.abs(wf)).cuda(), N, M)
    assert torch.equal(same, nm.nm_prune(dev_bf16(W), N, M))
