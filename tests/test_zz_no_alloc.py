"""The entry point that allocates nothing (fixed scratch inside the library) against the entry point it is a
variant of, nm_linear_forward with a caller's workspace: same bytes in Y, on two calls in a row, the second on a
smaller layer (the scratch keeps the first call's contents), and both within tolerance of the CPU checker."""
import numpy as np
import pytest
import torch

import paper_2409_09708_amd as nm
from oracle import nm_oracle as orc
from paper_2409_09708_amd import workloads as wl
from gpu_util import check_output, dev_bf16, host_output

pytestmark = pytest.mark.gpu


def run_pair(T, K, O, N, M, out_dtype, with_bias, rng):
    X, W = wl.draw_activations(rng, T, K), wl.draw_weights(rng, O, K)
    bias = rng.standard_normal(O).astype(np.float32) if with_bias else None
    bias_d = torch.from_numpy(bias).cuda() if with_bias else None
    Xd = dev_bf16(X)
    v, i = nm.nm_pack(dev_bf16(W), N, M)
    need = nm.nm_spmm_workspace_bytes(O, K, N, M, T)
    assert need <= nm.nm_static_scratch_bytes()
    ws = torch.empty((max(need, 256),), dtype=torch.uint8, device="cuda")
    ref = nm.nm_linear_forward(v, i, K, N, M, Xd, bias=bias_d, out_dtype=out_dtype, workspace=ws)
    out = torch.full((T, O), float("nan"), dtype=out_dtype, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    # raw C ABI call: no workspace argument, nothing allocated
    lib = nm.load_library()
    st = lib.nm_linear_forward_static(v.data_ptr(), i.data_ptr(), O, K, N, M, Xd.data_ptr(), T, Xd.stride(0),
                                      bias_d.data_ptr() if with_bias else None, out.data_ptr(), out.stride(0),
                                      1 if out_dtype == torch.bfloat16 else 0, torch.cuda.current_stream().cuda_stream)
    assert st == 0, nm.nm_status_string(st)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(out.view(torch.int16 if out_dtype == torch.bfloat16 else torch.int32),
                       ref.view(torch.int16 if out_dtype == torch.bfloat16 else torch.int32)), (T, K, O, N, M)
    Yref, B = orc.nm_linear_from_bits(X, W, N, M, bias=bias)
    if with_bias:
        B = B + np.abs(bias)[None, :]
    check_output(host_output(out), Yref, B, K // M * N + (1 if with_bias else 0), out_dtype == torch.float32,
                 f"static {T}x{K}x{O} {N}:{M}")


def test_static_scratch_matches_workspace_call_two_calls_second_smaller():
    rng = np.random.default_rng(20240)
    # first: a layer on the persistent kernel (stream-order scratch, dense form, 2 x 129 tiles), then smaller
    # ones: tiled kernel with a re-coded 1:8 weight, then a level that needs no scratch at all
    run_pair(129 * 256 - 19, 192, 500, 4, 8, torch.bfloat16, True, rng)
    run_pair(197, 768, 384, 1, 8, torch.float32, False, rng)
    run_pair(64, 128, 96, 2, 4, torch.float32, True, rng)


def test_static_scratch_sparse_form_then_smaller_sparse_form():
    rng = np.random.default_rng(20241)
    run_pair(128 * 256 + 5, 256, 512, 2, 16, torch.bfloat16, False, rng)
    run_pair(300, 128, 200, 1, 4, torch.bfloat16, True, rng)


def test_layer_too_large_for_the_static_scratch_is_refused():
    lib = nm.load_library()
    x = torch.zeros((8,), dtype=torch.bfloat16, device="cuda")
    st = lib.nm_linear_forward_static(x.data_ptr(), x.data_ptr(), 4096, 4096, 4, 8, x.data_ptr(), 65536, 4096, None,
                                      x.data_ptr(), 4096, 1, None)
    assert st == 6
