"""The library's calls are kernel launches and nothing else (no allocation, no memset, no synchronisation), so a
step of the path (select + pack + operand order of all layers, then all products) can be recorded into a HIP
graph once and replayed.  Every replay is checked against the same calls issued eagerly on the data the buffers
hold at that moment, with eager work and synchronisations between the replays, and once against the oracle."""
import numpy as np
import pytest
import torch

import paper_2409_09708_amd as nm
from oracle import nm_oracle as orc
from paper_2409_09708_amd import workloads as wl
from gpu_util import check_output, dev_bf16, host_bits, host_output, host_words

pytestmark = pytest.mark.gpu


def test_a_recorded_step_replays_like_the_eager_calls():
    rng = np.random.default_rng(777)
    T = 1300  # persistent kernel for the wide layers (five token tiles and a ragged sixth), tiled kernel for the small one
    specs = [(768, 768, 2, 4, torch.bfloat16), (768, 1024, 1, 8, torch.float32), (1024, 768, 4, 8, torch.bfloat16),
             (256, 128, 2, 8, torch.float32)]  # (K, O, N, M, output type)
    W_host = [wl.draw_weights(rng, O, K) for (K, O, _, _, _) in specs]
    X_host = [wl.draw_activations(rng, T, K) for (K, _, _, _, _) in specs]
    Ws = [dev_bf16(w) for w in W_host]
    Xs = [dev_bf16(x) for x in X_host]
    layers = [(W, N, M, T) for W, (_, _, N, M, _) in zip(Ws, specs)]
    # buffers of the recorded step and of the eager step
    packed_g, ws_g = nm.nm_pack_prepare_batched(layers)
    packed_e, ws_e = nm.nm_pack_prepare_batched(layers)
    Yg = [torch.zeros((T, O), dtype=dt, device="cuda") for (_, O, _, _, dt) in specs]
    Ye = [torch.zeros((T, O), dtype=dt, device="cuda") for (_, O, _, _, dt) in specs]

    def entries(packed, wss, Ys):
        return [(v, i, K, N, M, X, ws, None, Y)
                for (v, i), ws, X, Y, (K, _, N, M, _) in zip(packed, wss, Xs, Ys, specs)]

    descs_g = nm.forward_descs(entries(packed_g, ws_g, Yg))
    descs_e = nm.forward_descs(entries(packed_e, ws_e, Ye))

    def step(packed, wss, descs, stream):
        nm.nm_pack_prepare_batched(layers, stream=stream, out=packed, workspaces=wss)
        nm.nm_linear_forward_prepared_batched(descs, stream=stream)

    step(packed_e, ws_e, descs_e, torch.cuda.current_stream())  # first launches raise the kernels' LDS limits
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.graph(graph, stream=side):
        step(packed_g, ws_g, descs_g, torch.cuda.current_stream())
    torch.cuda.synchronize()

    for replay in range(4):
        if replay:  # new weights and activations in the same buffers: the graph must read what is there now
            for n, (K, O, _, _, _) in enumerate(specs):
                W_host[n] = wl.draw_weights(rng, O, K)
                X_host[n] = wl.draw_activations(rng, T, K)
                Ws[n].copy_(dev_bf16(W_host[n]))
                Xs[n].copy_(dev_bf16(X_host[n]))
        for y in Yg + Ye:
            y.fill_(7.0)
        for (v, i) in packed_g:
            v.zero_()
            i.zero_()
        torch.cuda.synchronize()
        graph.replay()
        step(packed_e, ws_e, descs_e, torch.cuda.current_stream())
        torch.cuda.synchronize()
        for n in range(len(specs)):
            assert torch.equal(packed_g[n][0].view(torch.int16), packed_e[n][0].view(torch.int16)), (replay, n)
            assert torch.equal(packed_g[n][1], packed_e[n][1]), (replay, n)
            assert torch.equal(Yg[n], Ye[n]), (replay, n)

    # the last replay against the oracle
    for n, (K, O, N, M, dt) in enumerate(specs):
        mask = orc.nm_mask(W_host[n], N, M)
        vals, idx = orc.nm_pack(W_host[n], mask, N, M)
        assert np.array_equal(host_bits(packed_g[n][0]), vals) and np.array_equal(host_words(packed_g[n][1]), idx)
        Yref, B = orc.nm_linear(X_host[n], W_host[n], mask)
        check_output(host_output(Yg[n]), Yref, B, K // M * N, dt == torch.float32, f"layer {n}")


def test_the_entry_point_on_the_fixed_scratch_replays_like_its_eager_calls():
    # the calls that cannot allocate are the ones a caller records: three layers in a row on the library's scratch
    rng = np.random.default_rng(31000)
    lib = nm.load_library()
    # (T, K, O, N, M): a re-coded level on the tiled kernel, a dense-form level, a 2:4 layer
    shapes = [(197, 768, 384, 1, 8), (300, 256, 512, 4, 8), (64, 128, 96, 2, 4)]
    layers = []
    for (T, K, O, N, M) in shapes:
        X = dev_bf16(wl.draw_activations(rng, T, K))
        v, i = nm.nm_pack(dev_bf16(wl.draw_weights(rng, O, K)), N, M)
        bias = torch.from_numpy(rng.standard_normal(O).astype(np.float32)).cuda()
        eager = nm.nm_linear_forward(v, i, K, N, M, X, bias=bias, out_dtype=torch.bfloat16)
        out = torch.zeros((T, O), dtype=torch.bfloat16, device="cuda")
        layers.append((T, K, O, N, M, X, v, i, bias, eager, out))

    def static_calls(stream):
        for (T, K, O, N, M, X, v, i, bias, _, out) in layers:
            st = lib.nm_linear_forward_static(v.data_ptr(), i.data_ptr(), O, K, N, M, X.data_ptr(), T, X.stride(0),
                                              bias.data_ptr(), out.data_ptr(), out.stride(0), 1, stream)
            assert st == 0, nm.nm_status_string(st)

    # first use outside the capture: kernel attributes and the scratch address are set up once per device
    static_calls(torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        static_calls(torch.cuda.current_stream().cuda_stream)
    for rep in range(4):
        for layer in layers:
            layer[-1].fill_(3.0)          # eager work between the replays; the replay must overwrite it
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for (T, K, O, N, M, X, v, i, bias, eager, out) in layers:
            assert torch.equal(out.view(torch.int16), eager.view(torch.int16)), (rep, T, K, O, N, M)
        # an eager call of the same entry point between replays (it shares the scratch)
        static_calls(torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
