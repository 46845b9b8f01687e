"""Host-side checks of the C ABI that need no GPU: the library loads, exports what the header
declares, sizes follow the packed layout, and every argument error is reported before a launch."""
import ctypes
import os
import re

import pytest

from oracle import nm_oracle as orc
from paper_2409_09708_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x1000  # a non-NULL, well aligned address that is never dereferenced on the error paths


@pytest.fixture(scope="module")
def lib():
    return binding.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "nm_sparse.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(nm_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported(lib):
    names = declared_functions()
    assert {"nm_prune", "nm_pack", "nm_spmm", "nm_linear_forward", "nm_unpack", "nm_pack_batched"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(binding.EXPORTS)


@pytest.mark.parametrize("N,M", [(1, 4), (2, 4), (4, 4), (1, 8), (2, 8), (3, 8), (4, 8), (1, 16), (2, 16), (4, 16)])
@pytest.mark.parametrize("O,K", [(1, 16), (5, 80), (768, 768), (3072, 768), (7, 48)])
def test_sizes_follow_the_layout(lib, N, M, O, K):
    if K % M:
        assert lib.nm_values_bytes(O, K, N, M) == 0
        return
    assert lib.nm_values_bytes(O, K, N, M) == O * orc.values_per_row(K, N, M) * 2
    assert lib.nm_index_bytes(O, K, N, M) == O * orc.index_words_per_row(K, N, M) * 4
    assert lib.nm_mask_bytes(O, K) == O * orc.mask_words_per_row(K) * 4


def test_sizes_of_illegal_requests_are_zero(lib):
    assert lib.nm_values_bytes(4, 16, 0, 4) == 0
    assert lib.nm_values_bytes(4, 16, 5, 4) == 0
    assert lib.nm_values_bytes(4, 16, 1, 32) == 0
    assert lib.nm_index_bytes(0, 16, 1, 4) == 0
    assert lib.nm_mask_bytes(-1, 16) == 0
    assert lib.nm_spmm_workspace_bytes(4, 64, 2, 4, 0) == 0


def test_workspace_sizes(lib):
    assert lib.nm_spmm_workspace_bytes(768, 768, 2, 4, 100) == 0       # packed 2:4 is the operand layout
    assert lib.nm_spmm_workspace_bytes(768, 768, 8, 8, 100) == 0       # dense level
    assert lib.nm_spmm_workspace_bytes(768, 768, 1, 8, 100) == 768 * 768 + 768 * 768 // 8
    assert lib.nm_spmm_workspace_bytes(768, 768, 4, 8, 100) == 768 * 768 * 2
    assert lib.nm_spmm_workspace_bytes(8, 24, 1, 8, 100) == 0          # general kernel, no scratch
    # the persistent kernel (long token counts) reads every level in stream order, rows padded to whole
    # 256-row tiles (768 -> 768, 700 -> 768)
    assert lib.nm_spmm_workspace_bytes(768, 768, 2, 4, 50432) == 768 * 768 + 768 * 768 // 8
    assert lib.nm_spmm_workspace_bytes(700, 768, 1, 16, 50432) == 768 * 768 + 768 * 768 // 8
    assert lib.nm_spmm_workspace_bytes(768, 768, 4, 8, 50432) == 768 * 768 * 2
    assert lib.nm_spmm_workspace_bytes(768, 768, 8, 8, 50432) == 768 * 768 * 2


def test_workspace_of_a_cut_reduction(lib):
    # few tiles and a long reduction: the fp32 partial sums of 2 .. 8 ranges lie behind the (256-aligned) operand copy
    T, K, O = 197, 4096, 1024
    planes = lib.nm_spmm_workspace_bytes(O, K, 2, 4, T)              # 2:4 needs no operand copy
    assert planes % (T * O * 4) == 0 and 2 <= planes // (T * O * 4) <= 8
    operand = O * K + O * K // 8
    with_copy = lib.nm_spmm_workspace_bytes(O, K, 1, 8, T)
    assert with_copy == (operand + 255) // 256 * 256 + planes       # the same ranges whatever the level of the form
    # a short reduction, or enough tiles to fill the chip, is never cut
    assert lib.nm_spmm_workspace_bytes(O, 1024, 2, 4, T) == 0
    assert lib.nm_spmm_workspace_bytes(O, K, 2, 4, 50432) == O * K + O * K // 8
    # ranges never come out empty: every count of steps from 64 up gives whole planes
    for steps in range(64, 100):
        b = lib.nm_spmm_workspace_bytes(256, steps * 64, 2, 4, 64)
        n = b // (64 * 256 * 4)
        assert b == n * 64 * 256 * 4 and 2 <= n <= 8
        per = -(-steps // n)
        assert (n - 1) * per < steps


def test_status_strings(lib):
    seen = set()
    for s in range(0, 8):
        txt = lib.nm_status_string(s).decode()
        assert txt and txt != "unknown status"
        seen.add(txt)
    assert len(seen) == 8
    assert lib.nm_status_string(99).decode() == "unknown status"
    assert lib.nm_last_hip_error() == 0


def test_prune_argument_errors(lib):
    assert lib.nm_prune(None, 4, 16, 16, 2, 4, FAKE, None, None) == 1
    assert lib.nm_prune(FAKE, 4, 16, 16, 2, 4, None, None, None) == 1
    assert lib.nm_prune(FAKE, 4, 16, 16, 0, 4, FAKE, None, None) == 3
    assert lib.nm_prune(FAKE, 4, 16, 16, 3, 2, FAKE, None, None) == 3
    assert lib.nm_prune(FAKE, 4, 16, 16, 1, 5, FAKE, None, None) == 3
    assert lib.nm_prune(FAKE, 4, 12, 12, 2, 8, FAKE, None, None) == 2   # K % M != 0
    assert lib.nm_prune(FAKE, 0, 16, 16, 2, 4, FAKE, None, None) == 2
    assert lib.nm_prune(FAKE, 4, 16, 8, 2, 4, FAKE, None, None) == 2    # ldw < K
    assert lib.nm_prune(FAKE + 1, 4, 16, 16, 2, 4, FAKE, None, None) == 4
    assert lib.nm_prune(FAKE, 4, 16, 16, 2, 4, FAKE + 2, None, None) == 4


def test_pack_unpack_argument_errors(lib):
    assert lib.nm_pack(None, 4, 16, 16, 2, 4, None, FAKE, FAKE, None) == 1
    assert lib.nm_pack(FAKE, 4, 16, 16, 2, 4, None, None, FAKE, None) == 1
    assert lib.nm_pack(FAKE, 4, 16, 16, 2, 4, None, FAKE, None, None) == 1
    assert lib.nm_pack(FAKE, 4, 16, 16, 9, 8, None, FAKE, FAKE, None) == 3
    assert lib.nm_pack(FAKE, 4, 20, 20, 2, 8, None, FAKE, FAKE, None) == 2
    assert lib.nm_pack(FAKE, 4, 16, 16, 2, 4, FAKE + 1, FAKE, FAKE, None) == 4
    assert lib.nm_unpack(None, FAKE, 4, 16, 2, 4, FAKE, 16, None) == 1
    assert lib.nm_unpack(FAKE, FAKE, 4, 16, 2, 4, FAKE, 15, None) == 2
    assert lib.nm_unpack(FAKE, FAKE, 4, 16, 2, 6, FAKE, 16, None) == 3
    assert lib.nm_mask_check(FAKE, 4, 16, 2, 4, None, None) == 1
    assert lib.nm_mask_check(FAKE, 4, 18, 2, 4, FAKE, None) == 2


def test_rank_argument_errors_and_sizes(lib):
    assert lib.nm_rank_bytes(8, 64) == 8 * 32
    assert lib.nm_rank_bytes(0, 64) == 0 and lib.nm_rank_bytes(8, 6) == 0
    assert lib.nm_rank(None, 4, 16, 16, 4, FAKE, None) == 1
    assert lib.nm_rank(FAKE, 4, 16, 16, 4, None, None) == 1
    assert lib.nm_rank(FAKE, 4, 16, 16, 5, FAKE, None) == 3
    assert lib.nm_rank(FAKE, 4, 12, 12, 8, FAKE, None) == 2
    assert lib.nm_rank(FAKE, 4, 16, 8, 4, FAKE, None) == 2
    assert lib.nm_rank(FAKE + 1, 4, 16, 16, 4, FAKE, None) == 4
    assert lib.nm_rank_mask(None, 4, 16, 2, 4, FAKE, None) == 1
    assert lib.nm_rank_mask(FAKE, 4, 16, 5, 4, FAKE, None) == 3
    assert lib.nm_rank_mask(FAKE, 4, 16, 2, 4, FAKE + 2, None) == 4
    assert lib.nm_pack_ranked(FAKE, None, 4, 16, 16, 2, 4, FAKE, FAKE, None) == 1
    assert lib.nm_pack_ranked(FAKE, FAKE, 4, 16, 16, 0, 4, FAKE, FAKE, None) == 3
    assert lib.nm_pack_ranked(FAKE, FAKE, 4, 16, 15, 2, 4, FAKE, FAKE, None) == 2
    assert lib.nm_pack_ranked(FAKE, FAKE, 4, 16, 16, 2, 4, FAKE, FAKE + 2, None) == 4


def test_rank_batched_argument_errors(lib):
    from paper_2409_09708_amd.binding import RankDesc
    lib.nm_rank_batched.argtypes = [ctypes.POINTER(RankDesc), ctypes.c_int32, ctypes.c_void_p]
    lib.nm_rank_batched.restype = ctypes.c_int32
    d = (RankDesc * 1)()
    assert lib.nm_rank_batched(None, 1, None) == 1
    assert lib.nm_rank_batched(d, 0, None) == 2
    d[0] = RankDesc(FAKE, None, 8, 64, 4, 0)
    assert lib.nm_rank_batched(d, 1, None) == 1
    d[0] = RankDesc(FAKE, FAKE, 8, 64, 6, 0)
    assert lib.nm_rank_batched(d, 1, None) == 3
    d[0] = RankDesc(FAKE, FAKE, 8, 60, 8, 0)
    assert lib.nm_rank_batched(d, 1, None) == 2


def test_pack_batched_argument_errors(lib):
    assert lib.nm_pack_batched(None, 1, None) == 1
    d = (binding.PackDesc * 2)()
    d[0] = binding.PackDesc(FAKE, FAKE, FAKE, 4, 16, 2, 4)
    d[1] = binding.PackDesc(FAKE, FAKE, FAKE, 4, 16, 2, 4)
    assert lib.nm_pack_batched(d, 0, None) == 2
    d[1] = binding.PackDesc(FAKE, None, FAKE, 4, 16, 2, 4)
    assert lib.nm_pack_batched(d, 2, None) == 1
    d[1] = binding.PackDesc(FAKE, FAKE, FAKE, 4, 16, 3, 2)
    assert lib.nm_pack_batched(d, 2, None) == 3
    d[1] = binding.PackDesc(FAKE, FAKE, FAKE, 4, 24, 1, 16)
    assert lib.nm_pack_batched(d, 2, None) == 2


def test_pack_ranked_batched_argument_errors(lib):
    assert lib.nm_pack_ranked_batched(None, 1, None) == 1
    d = (binding.PackRankedDesc * 2)()
    d[0] = binding.PackRankedDesc(FAKE, FAKE, FAKE, FAKE, 4, 16, 2, 4)
    d[1] = binding.PackRankedDesc(FAKE, FAKE, FAKE, FAKE, 4, 16, 2, 4)
    assert lib.nm_pack_ranked_batched(d, 0, None) == 2
    d[1] = binding.PackRankedDesc(FAKE, None, FAKE, FAKE, 4, 16, 2, 4)
    assert lib.nm_pack_ranked_batched(d, 2, None) == 1
    d[1] = binding.PackRankedDesc(FAKE, FAKE, FAKE, None, 4, 16, 2, 4)
    assert lib.nm_pack_ranked_batched(d, 2, None) == 1
    d[1] = binding.PackRankedDesc(FAKE, FAKE, FAKE, FAKE, 4, 16, 0, 4)
    assert lib.nm_pack_ranked_batched(d, 2, None) == 3
    d[1] = binding.PackRankedDesc(FAKE, FAKE, FAKE, FAKE, 4, 24, 1, 16)
    assert lib.nm_pack_ranked_batched(d, 2, None) == 2
    d[1] = binding.PackRankedDesc(FAKE, FAKE, FAKE, FAKE + 2, 4, 16, 2, 4)
    assert lib.nm_pack_ranked_batched(d, 2, None) == 4


def test_spmm_argument_errors(lib):
    ok = dict(values=FAKE, indices=FAKE, O=64, K=64, N=2, M=4, X=FAKE, T=16, ldx=64, Y=FAKE, ldy=64, dt=0,
              ws=None, wsb=0)

    def call(**kw):
        a = dict(ok, **kw)
        return lib.nm_spmm(a["values"], a["indices"], a["O"], a["K"], a["N"], a["M"], a["X"], a["T"], a["ldx"],
                           a["Y"], a["ldy"], a["dt"], a["ws"], a["wsb"], None)

    assert call(values=None) == 1 and call(indices=None) == 1 and call(X=None) == 1 and call(Y=None) == 1
    assert call(N=3, M=2) == 3 and call(M=32) == 3
    assert call(K=66) == 2 and call(T=0) == 2 and call(ldx=32) == 2 and call(ldy=8) == 2
    assert call(dt=2) == 5
    assert call(X=FAKE + 1) == 4 and call(Y=FAKE + 2) == 4
    # a level that needs scratch: missing, short and misaligned workspaces are refused before any launch (above 208
    # tokens; with fewer the product runs straight from the packed format when no workspace is given)
    assert call(N=1, M=8, T=300) == 6
    need = lib.nm_spmm_workspace_bytes(64, 64, 1, 8, 300)
    assert need == 256 * 64 + 256 * 64 // 8  # stream order: rows padded to a whole 256-row tile
    assert call(N=1, M=8, T=300, ws=FAKE, wsb=need - 1) == 6
    assert call(N=1, M=8, T=300, ws=FAKE + 16, wsb=need) == 6
    assert call(N=4, M=8, T=300, ws=None, wsb=0) == 6
    lf = lib.nm_linear_forward(FAKE, FAKE, 64, 64, 2, 4, FAKE, 16, 64, FAKE + 2, FAKE, 64, 0, None, 0, None)
    assert lf == 4  # bias must be 4-byte aligned


def test_prepare_and_prepared_argument_errors(lib):
    need = lib.nm_spmm_workspace_bytes(64, 64, 1, 8, 300)
    assert lib.nm_spmm_prepare(None, FAKE, 64, 64, 1, 8, 300, FAKE, need, None) == 1
    assert lib.nm_spmm_prepare(FAKE, FAKE, 64, 64, 9, 8, 300, FAKE, need, None) == 3
    assert lib.nm_spmm_prepare(FAKE, FAKE, 64, 60, 1, 8, 300, FAKE, need, None) == 2
    assert lib.nm_spmm_prepare(FAKE, FAKE, 64, 64, 1, 8, 0, FAKE, need, None) == 2
    assert lib.nm_spmm_prepare(FAKE, FAKE, 64, 64, 1, 8, 300, None, 0, None) == 6
    assert lib.nm_spmm_prepare(FAKE, FAKE, 64, 64, 1, 8, 300, FAKE, need - 1, None) == 6
    assert lib.nm_spmm_prepare(FAKE, FAKE, 64, 64, 2, 4, 300, None, 0, None) == 0   # nothing to prepare at 2:4
    assert lib.nm_spmm_prepare(FAKE, FAKE, 8, 24, 1, 8, 300, None, 0, None) == 0    # general kernel: no scratch
    args = (FAKE, FAKE, 64, 64, 1, 8, FAKE, 300, 64, None, FAKE, 64, 0)
    assert lib.nm_linear_forward_prepared(*args, None, 0, None) == 6
    assert lib.nm_linear_forward_prepared(FAKE, FAKE, 64, 64, 1, 8, None, 300, 64, None, FAKE, 64, 0, FAKE, need, None) == 1
    assert lib.nm_linear_forward_prepared(FAKE, FAKE, 64, 64, 1, 8, FAKE, 300, 32, None, FAKE, 64, 0, FAKE, need, None) == 2


def test_pack_prepare_batched_argument_errors(lib):
    from paper_2409_09708_amd.binding import LayerDesc
    lib.nm_pack_prepare_batched.argtypes = [ctypes.POINTER(LayerDesc), ctypes.c_int32, ctypes.c_void_p]
    lib.nm_pack_prepare_batched.restype = ctypes.c_int32
    d = (LayerDesc * 1)()
    assert lib.nm_pack_prepare_batched(None, 1, None) == 1
    assert lib.nm_pack_prepare_batched(d, 0, None) == 2
    d[0] = LayerDesc(FAKE, FAKE, None, 768, 768, 2, 4, 50432, None, 0)
    assert lib.nm_pack_prepare_batched(d, 1, None) == 1
    d[0] = LayerDesc(FAKE, FAKE, FAKE, 768, 768, 3, 2, 50432, None, 0)
    assert lib.nm_pack_prepare_batched(d, 1, None) == 3
    d[0] = LayerDesc(FAKE, FAKE, FAKE, 768, 768, 2, 4, 0, None, 0)
    assert lib.nm_pack_prepare_batched(d, 1, None) == 2
    d[0] = LayerDesc(FAKE, FAKE, FAKE, 768, 768, 2, 4, 50432, None, 0)   # a large layer needs its workspace
    assert lib.nm_pack_prepare_batched(d, 1, None) == 6
    d[0] = LayerDesc(FAKE, FAKE, FAKE, 768, 768, 2, 4, 50432, FAKE, 16)
    assert lib.nm_pack_prepare_batched(d, 1, None) == 6


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_LIB", None)
    monkeypatch.setattr(binding, "_PKG_DIR", str(tmp_path))
    with pytest.raises(RuntimeError, match="missing"):
        binding.load_library()


def test_backward_argument_errors(lib):
    def dx(**kw):
        a = dict(Ws=FAKE, O=64, K=64, ldw=64, dY=FAKE, T=16, ldy=64, dX=FAKE, ldx=64, dt=0)
        a.update(kw)
        return lib.nm_linear_backward_input(a["Ws"], a["O"], a["K"], a["ldw"], a["dY"], a["T"], a["ldy"], a["dX"],
                                            a["ldx"], a["dt"], a.get("ws"), a.get("wsb", 0), None)

    assert dx(Ws=None) == 1 and dx(dY=None) == 1 and dx(dX=None) == 1
    assert dx(O=0) == 2 and dx(K=-1) == 2 and dx(T=0) == 2
    assert dx(ldw=32) == 2 and dx(ldy=63) == 2 and dx(ldx=8) == 2
    assert dx(dt=3) == 5
    assert dx(Ws=FAKE + 1) == 4 and dx(dX=FAKE + 2) == 4 and dx(dX=FAKE + 2, dt=1) != 4
    # large layers go through the forward path's kernel with the weight transposed into the scratch
    big = dict(O=768, K=3072, ldw=3072, T=50432, ldy=768, ldx=3072)
    need = lib.nm_backward_input_workspace_bytes(768, 3072, 50432)
    assert need == 3072 * 768 * 2
    assert lib.nm_backward_input_workspace_bytes(768, 3000, 50432) == 3072 * 768 * 2  # columns padded to whole tiles
    assert lib.nm_backward_input_workspace_bytes(768, 3072, 197) == 0                 # few tokens: tiled kernel
    assert lib.nm_backward_input_workspace_bytes(800, 3072, 50432) == 0               # O % 64 != 0: tiled kernel
    assert dx(**big) == 6 and dx(ws=FAKE, wsb=need - 1, **big) == 6 and dx(ws=FAKE + 16, wsb=need, **big) == 6

    def dw(**kw):
        a = dict(dY=FAKE, T=16, O=64, ldy=64, X=FAKE, K=64, ldx=64, mask=None, dW=FAKE, lddw=64, dt=0, ws=None, wsb=0)
        a.update(kw)
        return lib.nm_linear_backward_weight(a["dY"], a["T"], a["O"], a["ldy"], a["X"], a["K"], a["ldx"], a["mask"],
                                             a["dW"], a["lddw"], a["dt"], a["ws"], a["wsb"], None)

    assert dw(dY=None) == 1 and dw(X=None) == 1 and dw(dW=None) == 1
    assert dw(T=0) == 2 and dw(O=0) == 2 and dw(K=0) == 2
    assert dw(ldy=32) == 2 and dw(ldx=63) == 2 and dw(lddw=8) == 2
    assert dw(dt=-1) == 5
    assert dw(X=FAKE + 1) == 4 and dw(mask=FAKE + 2) == 4 and dw(dW=FAKE + 2) == 4
    # the split reduction needs its scratch: missing, short and misaligned workspaces are refused before any launch
    need = lib.nm_backward_weight_workspace_bytes(64, 64, 16)
    assert need == 128 * 256 * 4  # one tile, one range
    assert dw() == 6 and dw(ws=FAKE, wsb=need - 1) == 6 and dw(ws=FAKE + 16, wsb=need) == 6


def test_backward_weight_workspace_sizes(lib):
    f = lib.nm_backward_weight_workspace_bytes
    tile = 128 * 256 * 4
    assert f(0, 64, 16) == 0 and f(64, 64, 0) == 0
    assert f(30, 64, 100) == 0 and f(64, 52, 100) == 0  # the general kernel needs no scratch
    # DeiT-B at batch 256 (T = 50432: 1576 steps of 32 tokens), 512 blocks at once: 768 x 768 -> 6 x 3 tiles,
    # 26 ranges (468 blocks, 91 % of a round); 3072 x 768 -> 72 tiles, 7 ranges (504); 2304 x 768 -> 54 tiles, 9
    assert f(768, 768, 50432) == 26 * 18 * tile
    assert f(3072, 768, 50432) == 7 * 72 * tile and f(768, 3072, 50432) == 7 * 72 * tile
    assert f(2304, 768, 50432) == 9 * 54 * tile
    # a reduction too short for four steps per range is not cut
    assert f(768, 768, 197) == 18 * tile


def test_int8_argument_errors_and_sizes(lib):
    f = lib.nm_i8_workspace_bytes
    assert f(768, 768, 2, 4, 197) == 768 * 768 // 2 + 768 * 768 // 8   # values + 2-bit selectors
    assert f(768, 768, 1, 16, 197) == 768 * 768 // 2 + 768 * 768 // 8  # every level with N <= 2 takes the 2:4 form
    assert f(768, 768, 4, 8, 197) == 768 * 768 and f(768, 768, 8, 8, 197) == 768 * 768  # masked dense copy
    assert f(64, 48, 1, 8, 197) == 0                                   # general kernel
    assert f(64, 64, 3, 2, 197) == 0 and f(0, 64, 2, 4, 197) == 0 and f(64, 128, 2, 4, 0) == 0
    # large layers: the persistent kernel's stream order, rows padded to whole 256-row tiles (700 -> 768)
    assert f(700, 768, 2, 4, 50432) == 768 * 768 // 2 + 768 * 768 // 8
    assert f(700, 768, 4, 8, 50432) == 768 * 768
    assert f(700, 256, 2, 4, 50432) == 700 * 256 // 2 + 700 * 256 // 8  # fewer than three K steps: tiled kernel

    def call(**kw):
        a = dict(Wq=FAKE, O=64, K=128, ldw=128, mask=FAKE, N=2, M=4, Xq=FAKE, T=16, ldx=128, Y=FAKE, ldy=64, dt=2,
                 ws=FAKE, wsb=1 << 20)
        a.update(kw)
        return lib.nm_linear_forward_i8(a["Wq"], a["O"], a["K"], a["ldw"], a["mask"], a["N"], a["M"], a["Xq"], a["T"],
                                        a["ldx"], 1.0, None, None, a["Y"], a["ldy"], a["dt"], a["ws"], a["wsb"], None)

    assert call(Wq=None) == 1 and call(mask=None) == 1 and call(Xq=None) == 1 and call(Y=None) == 1
    assert call(N=5, M=4) == 3 and call(M=2) == 3
    assert call(K=130) == 2 and call(T=0) == 2 and call(ldw=64) == 2 and call(ldx=64) == 2 and call(ldy=8) == 2
    assert call(dt=3) == 5
    assert call(mask=FAKE + 2) == 4 and call(Y=FAKE + 2) == 4 and call(Y=FAKE + 2, dt=1) != 4
    need = lib.nm_i8_workspace_bytes(64, 128, 2, 4, 16)
    assert call(ws=None, wsb=0) == 6 and call(wsb=need - 1) == 6 and call(ws=FAKE + 16) == 6
    assert lib.nm_i8_prepare(None, 64, 128, 128, FAKE, 2, 4, 16, FAKE, need, None) == 1
    assert lib.nm_i8_prepare(FAKE, 64, 128, 128, FAKE, 2, 4, 16, None, 0, None) == 6
    assert lib.nm_i8_prepare(FAKE, 64, 128, 128, FAKE, 2, 4, 0, FAKE, need, None) == 2
    assert lib.nm_i8_prepare(FAKE, 64, 48, 48, FAKE, 1, 8, 16, None, 0, None) == 0  # nothing to prepare


def test_int8_compressed_form_argument_errors_and_sizes(lib):
    assert lib.nm_values_i8_bytes(768, 768, 2, 8) == 768 * 768 // 4
    assert lib.nm_values_i8_bytes(768, 770, 2, 8) == 0 and lib.nm_values_i8_bytes(768, 768, 9, 8) == 0
    pk = lib.nm_pack_i8
    assert pk(None, 4, 16, 16, 2, 4, FAKE, FAKE, FAKE, None) == 1 and pk(FAKE, 4, 16, 16, 2, 4, None, FAKE, FAKE, None) == 1
    assert pk(FAKE, 4, 16, 16, 2, 4, FAKE, None, FAKE, None) == 1 and pk(FAKE, 4, 16, 16, 2, 4, FAKE, FAKE, None, None) == 1
    assert pk(FAKE, 4, 16, 8, 2, 4, FAKE, FAKE, FAKE, None) == 2 and pk(FAKE, 4, 18, 18, 2, 4, FAKE, FAKE, FAKE, None) == 2
    assert pk(FAKE, 4, 16, 16, 5, 4, FAKE, FAKE, FAKE, None) == 3 and pk(FAKE, 4, 16, 16, 2, 4, FAKE + 2, FAKE, FAKE, None) == 4
    up = lib.nm_unpack_i8
    assert up(None, FAKE, 4, 16, 2, 4, FAKE, 16, None) == 1 and up(FAKE, FAKE, 4, 16, 2, 4, FAKE, 8, None) == 2
    assert up(FAKE, FAKE + 1, 4, 16, 2, 4, FAKE, 16, None) == 4

    def call(fn=lib.nm_linear_forward_i8_packed, **kw):
        a = dict(v=FAKE, i=FAKE, O=64, K=128, N=1, M=8, Xq=FAKE, T=16, ldx=128, Y=FAKE, ldy=64, dt=2, ws=FAKE, wsb=1 << 20)
        a.update(kw)
        return fn(a["v"], a["i"], a["O"], a["K"], a["N"], a["M"], a["Xq"], a["T"], a["ldx"], 1.0, None, None, a["Y"],
                  a["ldy"], a["dt"], a["ws"], a["wsb"], None)

    for fn in (lib.nm_linear_forward_i8_packed, lib.nm_linear_forward_i8_packed_prepared):
        assert call(fn, v=None) == 1 and call(fn, i=None) == 1 and call(fn, Xq=None) == 1 and call(fn, Y=None) == 1
        assert call(fn, N=0) == 3 and call(fn, K=132) == 2 and call(fn, T=0) == 2 and call(fn, ldx=64) == 2
        assert call(fn, dt=7) == 5 and call(fn, i=FAKE + 2) == 4
        assert call(fn, ws=None, wsb=0) == 6
    need = lib.nm_i8_workspace_bytes(64, 128, 1, 8, 16)
    assert lib.nm_i8_prepare_packed(FAKE, FAKE, 64, 128, 1, 8, 16, FAKE, need - 1, None) == 6
    assert lib.nm_i8_prepare_packed(None, FAKE, 64, 128, 1, 8, 16, FAKE, need, None) == 1
    assert lib.nm_i8_prepare_packed(FAKE, FAKE, 64, 48, 1, 8, 16, None, 0, None) == 0  # general kernel: nothing to prepare


def test_prune_scored_argument_errors(lib):
    f = lib.nm_prune_scored
    assert f(None, 4, 16, 16, 2, 4, FAKE, None) == 1 and f(FAKE, 4, 16, 16, 2, 4, None, None) == 1
    assert f(FAKE, 4, 16, 16, 5, 4, FAKE, None) == 3 and f(FAKE, 4, 16, 16, 2, 5, FAKE, None) == 3
    assert f(FAKE, 4, 18, 18, 2, 4, FAKE, None) == 2 and f(FAKE, 0, 16, 16, 2, 4, FAKE, None) == 2
    assert f(FAKE, 4, 16, 12, 2, 4, FAKE, None) == 2
    assert f(FAKE + 2, 4, 16, 16, 2, 4, FAKE, None) == 4 and f(FAKE, 4, 16, 16, 2, 4, FAKE + 2, None) == 4


def test_forward_batched_argument_errors(lib):
    D = binding.ForwardDesc
    ok = dict(values=FAKE, indices=FAKE, O=64, K=64, N=2, M=4, X=FAKE, T=16, ldx=64, bias=None, Y=FAKE, ldy=64,
              out_dtype=0, reserved=0, workspace=None, workspace_bytes=0)

    def run(*overrides):
        d = (D * len(overrides))()
        for n, kw in enumerate(overrides):
            d[n] = D(**dict(ok, **kw))
        return lib.nm_linear_forward_prepared_batched(d, len(overrides), None)

    assert lib.nm_linear_forward_prepared_batched(None, 1, None) == 1
    d = (D * 1)()
    d[0] = D(**ok)
    assert lib.nm_linear_forward_prepared_batched(d, 0, None) == 2
    # the first offending descriptor decides, whatever follows it
    assert run({}, dict(values=None)) == 1 and run({}, dict(X=None)) == 1 and run({}, dict(Y=None)) == 1
    assert run({}, dict(N=3, M=2)) == 3 and run({}, dict(K=66)) == 2 and run({}, dict(ldy=8)) == 2
    assert run({}, dict(out_dtype=2)) == 5 and run({}, dict(Y=FAKE + 2)) == 4
    assert run({}, dict(N=1, M=8, T=300)) == 6  # a level that needs a prepared workspace at this token count
    assert run({}, dict(N=1, M=8, T=300, workspace=FAKE, workspace_bytes=16)) == 6


def test_static_scratch_entry_argument_errors(lib):
    # the entry point for callers that cannot allocate: argument errors and the size limit come before any
    # device call, so they are checked here without a GPU
    cap = lib.nm_static_scratch_bytes()
    assert cap == 8 << 20
    ok = (FAKE, FAKE, 64, 64, 1, 8, FAKE, 16, 64, None, FAKE, 64, 0, None)
    bad = lambda i, v: lib.nm_linear_forward_static(*(ok[:i] + (v,) + ok[i + 1:]))
    assert bad(0, None) == 1 and bad(1, None) == 1 and bad(6, None) == 1 and bad(10, None) == 1
    assert bad(4, 9) == 3 and bad(3, 60) == 2 and bad(7, 0) == 2 and bad(8, 32) == 2 and bad(11, 8) == 2
    assert bad(12, 2) == 5 and bad(6, FAKE + 1) == 4 and bad(9, FAKE + 2) == 4
    # a layer whose operand-order copy does not fit the fixed scratch is refused (dense form of 4096 x 4096 at
    # 65536 tokens: 32 MiB)
    assert lib.nm_spmm_workspace_bytes(4096, 4096, 4, 8, 65536) > cap
    assert lib.nm_linear_forward_static(FAKE, FAKE, 4096, 4096, 4, 8, FAKE, 65536, 4096, None, FAKE, 4096, 1, None) == 6


def test_weights_beyond_the_grid_limit_are_refused(lib):
    # O * K above 2^40: some launcher's grid would not fit; reported as a shape error, nothing launched
    big = 1 << 21
    assert lib.nm_values_bytes(big, big, 2, 4) == 0
    assert lib.nm_prune(FAKE, big, big, big, 2, 4, FAKE, None, None) == 2
    assert lib.nm_unpack(FAKE, FAKE, big, big, 2, 4, FAKE, big, None) == 2
    assert lib.nm_values_bytes(1 << 20, 1 << 20, 2, 4) == (1 << 40)
