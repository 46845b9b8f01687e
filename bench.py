#!/usr/bin/env python3
"""Benchmark of the N:M-sparse linear hot path on one MI355X.

One step = one pass of the whole path over the DeiT-B batch-256 linear stack (50432 tokens, 12 blocks
x {qkv, proj, fc1, fc2}, layer-wise level drawn with seed 0 from {1:4,2:4,1:8,2:8,4:8,1:16,4:16}):
magnitude N:M selection + packing of all 48 weights (one batched launch), then the 48 sparse-weight x
dense-activation products from the packed form (bf16 in, fp32 accumulate, bf16 out).  All inputs are
resident in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_DENSE_TFLOPS = 2500.0  # MI355X dense bf16 matrix-core peak
PEAK_HBM_GBS = 8000.0            # MI355X HBM3E
PEAK_INT8_DENSE_TOPS = 5000.0    # MI355X dense int8 matrix-core peak
PEAK_HBM_GBS = 8000.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def build_inputs(layers, torch, wl, seed=0):
    """Weights: one Gaussian draw per layer.  Activations: one Gaussian draw per input width (768 and
    3072); every layer gets its own copy (rolled by its index along the token axis) so that no two layers
    share HBM lines or cache contents."""
    from paper_2409_09708_amd import bf16_tensor as dev_bf16
    rng = np.random.default_rng(seed)
    base = {}
    for L in layers:
        if L.K not in base:
            base[L.K] = dev_bf16(wl.draw_activations(rng, L.T, L.K))
    Ws, Xs = [], []
    for i, L in enumerate(layers):
        Ws.append(dev_bf16(wl.draw_weights(rng, L.O, L.K)))
        Xs.append(torch.roll(base[L.K], shifts=i, dims=0).contiguous())
    return Ws, Xs


def algorithmic_bytes(L, out_bytes=2):
    """HBM bytes one product launch has to move: X once, the operand-order weight once, Y once."""
    b = {4: 2, 8: 3, 16: 4}[L.M]
    if L.N <= 2:
        w = L.O * L.K * (2 + 2 / 8) / 2  # 2:4 operand form: half the values + 2-bit selectors
    else:
        w = L.O * L.K * 2                # dense operand form
    del b
    return 2.0 * L.T * L.K + w + out_bytes * L.T * L.O


def ceiling_ms(L):
    """Time below which one product cannot go on nominal peaks: the matrix-core roof (a level with N <= 2 runs
    on the 2:4 sparse instruction at half the dense instruction count, the others on the dense one) or the HBM
    roof of its algorithmic bytes, whichever is later."""
    math = L.dense_flops * (0.5 if L.N <= 2 else 1.0) / (PEAK_BF16_DENSE_TFLOPS * 1e12)
    hbm = algorithmic_bytes(L) / (PEAK_HBM_GBS * 1e9)
    return max(math, hbm) * 1e3


def measured_traffic(schedule):
    """HBM bytes per launch of the dominant kernel, in the given launch schedule, from the committed rocprofv3
    counter summary, or None when the kernel source has changed since the counters were taken."""
    import hashlib
    path = os.path.join(ROOT, "profiles", "hbm_traffic_bench_deit_b256.txt")
    src = os.path.join(ROOT, "paper_2409_09708_amd", "csrc", "nm_spmm.hip")
    try:
        text = open(path).read()
        now = hashlib.sha256(open(src, "rb").read()).hexdigest()[:16]
    except OSError:
        return None
    if f"nm_spmm.hip {now}" not in text:
        return None
    key = "sparse_gemm_hbm_bytes_per_launch_" + ("batched" if schedule == "batched" else "single")
    for line in text.splitlines():
        if line.startswith(key + " "):
            return int(line.split()[1])
    return None


def cpu_baseline(wl, seed=0, blocks=12):
    """The CPU checker as it stands, timed on this host on the same workload, once: the 4*blocks layers at their
    drawn levels and all 50432 tokens: select + pack + fp64 product (about 15-20 s on the benchmark host).  As in
    the GPU step one activation matrix is drawn per input width; only the checker's own calls are timed."""
    from oracle import nm_oracle as orc
    layers = wl.deit_b_stack()[:4 * blocks]
    tokens = layers[0].T
    rng = np.random.default_rng(seed)
    xs = {}
    for L in layers:
        if L.K not in xs:
            xs[L.K] = wl.draw_activations(rng, tokens, L.K)
    dt, useful = 0.0, 0.0
    for L in layers:
        W = wl.draw_weights(rng, L.O, L.K)
        t0 = time.perf_counter()
        m = orc.nm_mask(W, L.N, L.M)
        orc.nm_pack(W, m, L.N, L.M)
        Xf = orc.bf16_bits_to_f64(xs[L.K])
        Ws = orc.bf16_bits_to_f64(orc.apply_mask(W, m))
        _ = Xf @ Ws.T
        dt += time.perf_counter() - t0
        useful += 2.0 * tokens * L.O * L.K * L.N / L.M
        del Xf, Ws, _
    cores = len(os.sched_getaffinity(0))
    return {"value": useful / dt / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "sample": f"{len(layers)} of the 48 layers at their drawn levels on all {tokens} tokens, once: "
                      f"numpy select + pack + fp64 dense product, {dt:.2f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--schedule", default="batched", choices=("batched", "streams", "single"),
                    help="how the 48 independent products of a step are launched")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--report", action="store_true", help="per-layer table on stderr")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (a known HBM traffic, for scaling profiler byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: the library has no multi-GPU path (--gpus must be 1)", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2409_09708_amd as nm
    from paper_2409_09708_amd import workloads as wl

    nm.load_library()  # no fallback: fails here if the HIP library is missing
    if not torch.cuda.is_available():
        print("no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    layers = wl.deit_b_stack(batch=256, seed=0)
    T = layers[0].T
    t_gen = time.perf_counter()
    Ws, Xs = build_inputs(layers, torch, wl)
    log(f"inputs ready in {time.perf_counter() - t_gen:.1f} s")

    packed = [(torch.empty((L.O, L.K // L.M * L.N), dtype=torch.bfloat16, device=dev),
               torch.empty((L.O, nm.nm_index_bytes(L.O, L.K, L.N, L.M) // (4 * L.O)), dtype=torch.int32, device=dev))
              for L in layers]
    Ys = [torch.empty((L.T, L.O), dtype=torch.bfloat16, device=dev) for L in layers]
    # one operand-order workspace per layer (a deployed model keeps them; here they are rewritten every step)
    workspaces = [torch.empty((max(nm.nm_spmm_workspace_bytes(L.O, L.K, L.N, L.M, L.T), 256),), dtype=torch.uint8,
                              device=dev) for L in layers]
    stream = torch.cuda.current_stream()
    pack_args = [(W, L.N, L.M, L.T) for W, L in zip(Ws, layers)]

    # The 48 products of a step are independent (every layer has its own input).  A persistent product kernel
    # ends with a partial round of tiles (591 tiles on 256 compute units = 2.3 rounds for the 768-wide layers,
    # which then cost 3), so the step hands all of them to the library at once: layers of one operand form share
    # a launch whose blocks walk the tiles of all of them as one list (2 launches instead of 48).
    # --schedule streams: one launch per layer, alternating between two streams of equal priority, so that the
    # next kernel's blocks start on the compute units that fall idle.  --schedule single: one launch per layer,
    # one stream.
    side = torch.cuda.Stream(device=dev) if args.schedule == "streams" else None
    packed_ready, side_done = torch.cuda.Event(), torch.cuda.Event()
    descs = nm.forward_descs([(v, i, L.K, L.N, L.M, X, ws, None, Y)
                              for L, (v, i), X, Y, ws in zip(layers, packed, Xs, Ys, workspaces)])

    def step():
        # the whole path: select + pack all 48 weights and write their operand-order forms (one launch), then
        # the 48 products at each layer's own level
        nm.nm_pack_prepare_batched(pack_args, stream=stream, out=packed, workspaces=workspaces)
        if args.schedule == "batched":
            nm.nm_linear_forward_prepared_batched(descs, stream=stream)
            return
        if side is not None:
            packed_ready.record(stream)
            side.wait_event(packed_ready)
        for n, (L, (v, i), X, Y, ws) in enumerate(zip(layers, packed, Xs, Ys, workspaces)):
            on = side if (side is not None and n % 2) else stream
            nm.nm_linear_forward_prepared(v, i, L.K, L.N, L.M, X, ws, out=Y, stream=on)
        if side is not None:
            side_done.record(side)
            stream.wait_event(side_done)

    if args.calibrate_copy:
        src = torch.empty((256 << 20,), dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / args.steps

    useful = sum(L.useful_flops for L in layers)
    dense = sum(L.dense_flops for L in layers)

    # ---- kernel durations with HIP events on the launch stream: a second pass over the same step with events
    # around the batched pack and around every product launch.  In the batched schedule the library launches the
    # persistent kernel once per operand form; the pass hands it the two groups one after the other, so each event
    # pair brackets exactly one kernel.  Otherwise (and for the per-layer report) every layer is its own launch.
    reps = max(3, min(args.steps, 10))
    sp = [j for j, L in enumerate(layers) if L.N <= 2]
    dn = [j for j, L in enumerate(layers) if L.N > 2]
    sp_useful = sum(layers[j].useful_flops for j in sp)
    pk = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    layer_ms = None
    if args.schedule == "batched":
        entries = [(v, i, L.K, L.N, L.M, X, ws, None, Y) for L, (v, i), X, Y, ws in zip(layers, packed, Xs, Ys, workspaces)]
        descs_sp = nm.forward_descs([entries[j] for j in sp])
        descs_dn = nm.forward_descs([entries[j] for j in dn])
        gv = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(reps)]
        for r in range(reps):
            pk[r][0].record(stream)
            nm.nm_pack_prepare_batched(pack_args, stream=stream, out=packed, workspaces=workspaces)
            pk[r][1].record(stream)
            gv[r][0].record(stream)
            nm.nm_linear_forward_prepared_batched(descs_sp, stream=stream)
            gv[r][1].record(stream)
            nm.nm_linear_forward_prepared_batched(descs_dn, stream=stream)
            gv[r][2].record(stream)
        torch.cuda.synchronize()
        sp_ms = float(np.median([g[0].elapsed_time(g[1]) for g in gv]))
        dn_ms = float(np.median([g[1].elapsed_time(g[2]) for g in gv]))
        sp_launches = 1
    if args.schedule != "batched" or args.report:
        ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in layers]
              for _ in range(reps)]
        for r in range(reps):
            if args.schedule != "batched":
                pk[r][0].record(stream)
            nm.nm_pack_prepare_batched(pack_args, stream=stream, out=packed, workspaces=workspaces)
            if args.schedule != "batched":
                pk[r][1].record(stream)
            for j, (L, (v, i), X, Y, ws) in enumerate(zip(layers, packed, Xs, Ys, workspaces)):
                ev[r][j][0].record(stream)
                nm.nm_linear_forward_prepared(v, i, L.K, L.N, L.M, X, ws, out=Y, stream=stream)
                ev[r][j][1].record(stream)
        torch.cuda.synchronize()
        layer_ms = [float(np.median([ev[r][j][0].elapsed_time(ev[r][j][1]) for r in range(reps)]))
                    for j in range(len(layers))]
        if args.schedule != "batched":
            sp_ms = sum(layer_ms[j] for j in sp)
            dn_ms = sum(layer_ms[j] for j in dn)
            sp_launches = len(sp)
    pack_ms = float(np.median([a.elapsed_time(b) for a, b in pk]))

    # dominant kernel: the sparse matrix-core product (the 36 layers with N <= 2): one launch for all of them in
    # the batched schedule, one per layer otherwise
    achieved = sp_useful / (sp_ms * 1e-3) / 1e12
    roofline = {"bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_DENSE_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved / PEAK_BF16_DENSE_TFLOPS, "traffic": measured_traffic(args.schedule),
                "kernel": "nm_stream_kernel<sparse> (v_smfmac_f32_16x16x64_bf16); useful FLOPs 2*T*O*K*N/M summed over the "
                          f"{len(sp)} layers with N <= 2, {sp_launches} launch(es) per step",
                "launches_per_step": sp_launches, "avg_launch_ms": sp_ms / sp_launches,
                "useful_flops_per_launch": sp_useful / sp_launches,
                "dense_equivalent_tflops": sum(layers[j].dense_flops for j in sp) / (sp_ms * 1e-3) / 1e12,
                "algorithmic_hbm_bytes_per_launch": sum(algorithmic_bytes(layers[j]) for j in sp) / sp_launches,
                "dense_form_kernel_ms_per_step": dn_ms}

    # ---- nested levels (ranks inside groups): rank the 48 weights once for their M, then take each layer's
    # level from the ranks.  Streaming kernels: algorithmic bytes = 2 read + 1/2 written per weight for the
    # ranking; 2.5 read + packed bytes written for the ranked pack.
    ranks = [torch.empty((L.O, L.K // 2), dtype=torch.uint8, device=dev) for L in layers]
    rank_args = [(W, L.M) for W, L in zip(Ws, layers)]

    def rank_all():
        nm.nm_rank_batched(rank_args, stream=stream, out=ranks)

    ranked_args = [(W, r, L.N, L.M) for W, r, L in zip(Ws, ranks, layers)]

    def pack_ranked_all():
        nm.nm_pack_ranked_batched(ranked_args, stream=stream, out=packed)

    def timed(fn):
        fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        for _ in range(reps):
            fn()
        b.record(stream)
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    n_weights = sum(L.O * L.K for L in layers)
    packed_bytes = sum(v.numel() * 2 + i.numel() * 4 for v, i in packed)
    rank_ms, pr_ms = timed(rank_all), timed(pack_ranked_all)
    nested = {"workload": "48 DeiT-B weight matrices: ranking in one launch, packing from the ranks in one launch",
              "rank": {"ms": rank_ms, "algorithmic_bytes": 2.5 * n_weights,
                       "roofline": {"bound": "hbm", "achieved": 2.5 * n_weights / rank_ms / 1e6, "peak": 8000.0,
                                    "unit": "GB/s", "frac": 2.5 * n_weights / rank_ms / 1e6 / 8000.0}},
              "pack_ranked": {"ms": pr_ms, "algorithmic_bytes": 2.5 * n_weights + packed_bytes,
                              "roofline": {"bound": "hbm", "achieved": (2.5 * n_weights + packed_bytes) / pr_ms / 1e6,
                                           "peak": 8000.0, "unit": "GB/s",
                                           "frac": (2.5 * n_weights + packed_bytes) / pr_ms / 1e6 / 8000.0}}}

    # ---- training products of one transformer block (its four layers at their levels): dX = dY (W.m) and
    # dW = (dY^T X).m, dense matrix-core products of 2*T*O*K FLOPs each; the forward outputs stand in for dY
    train_layers = list(range(4))
    masked, words, dXs, dWs, gws = [], [], [], [], []
    for j in train_layers:
        L = layers[j]
        wm = torch.empty_like(Ws[j])
        words.append(nm.nm_prune(Ws[j], L.N, L.M, W_masked=wm))
        masked.append(wm)
        dXs.append(torch.empty((L.T, L.K), dtype=torch.bfloat16, device=dev))
        dWs.append(torch.empty((L.O, L.K), dtype=torch.float32, device=dev))
        gws.append(torch.empty((max(nm.nm_backward_weight_workspace_bytes(L.O, L.K, L.T), 256),), dtype=torch.uint8,
                               device=dev))

    def grad_inputs():
        for n, j in enumerate(train_layers):
            nm.nm_linear_backward_input(masked[n], Ys[j], out=dXs[n], stream=stream)

    def grad_weights():
        for n, j in enumerate(train_layers):
            nm.nm_linear_backward_weight(Ys[j], Xs[j], mask=words[n], out=dWs[n], workspace=gws[n], stream=stream)

    dx_ms, dw_ms = timed(grad_inputs), timed(grad_weights)
    block_flops = sum(layers[j].dense_flops for j in train_layers)

    def mfma_roofline(ms):
        tf = block_flops / ms / 1e9
        return {"bound": "mfma", "achieved": tf, "peak": PEAK_BF16_DENSE_TFLOPS, "unit": "TFLOP/s",
                "frac": tf / PEAK_BF16_DENSE_TFLOPS}

    training = {"workload": "one DeiT-B block at batch 256 (qkv, proj, fc1, fc2; T=50432): input gradients in bf16, "
                            "masked weight gradients in fp32; 2*T*O*K FLOPs per product",
                "input_gradient": {"ms": dx_ms, "roofline": mfma_roofline(dx_ms)},
                "weight_gradient": {"ms": dw_ms, "roofline": mfma_roofline(dw_ms)}}
    del masked, words, dXs, dWs, gws

    # ---- int8 form of the same block (8-bit quantisation on top of the sparse weights): the masks are those of
    # the float weights, the int8 operands synthetic; useful operations 2*T*O*K*N/M per product, bf16 output
    q_masks = [nm.nm_prune(Ws[j], layers[j].N, layers[j].M) for j in train_layers]
    gen = torch.Generator(device=dev)
    gen.manual_seed(1234)
    q_w = [torch.randint(-127, 128, (layers[j].O, layers[j].K), device=dev, dtype=torch.int8, generator=gen)
           for j in train_layers]
    q_x = [torch.randint(-127, 128, (layers[j].T, layers[j].K), device=dev, dtype=torch.int8, generator=gen)
           for j in train_layers]
    q_scale = [torch.full((layers[j].O,), 1e-4, dtype=torch.float32, device=dev) for j in train_layers]
    q_ws = [nm.nm_i8_prepare(q_w[n], q_masks[n], layers[j].N, layers[j].M, layers[j].T)
            for n, j in enumerate(train_layers)]

    def int8_products():
        for n, j in enumerate(train_layers):
            L = layers[j]
            nm.nm_linear_forward_i8_prepared(q_w[n], q_masks[n], L.N, L.M, q_x[n], q_ws[n], x_scale=0.02,
                                             w_scale=q_scale[n], out=Ys[j], stream=stream)

    q_ms = timed(int8_products)
    q_useful = sum(layers[j].useful_flops for j in train_layers)
    q_tops = q_useful / q_ms / 1e9
    int8 = {"workload": "one DeiT-B block at batch 256 (qkv, proj, fc1, fc2 at their seed-0 levels), int8 operands, "
                        "int32 sums rescaled to bf16; useful operations 2*T*O*K*N/M",
            "ms": q_ms, "dense_equivalent_tops": block_flops / q_ms / 1e9,
            "roofline": {"bound": "mfma", "achieved": q_tops, "peak": PEAK_INT8_DENSE_TOPS, "unit": "TOP/s",
                         "frac": q_tops / PEAK_INT8_DENSE_TOPS}}
    del q_masks, q_w, q_x, q_scale, q_ws

    # ---- the same stack at batch 1 (197 tokens): products of a few tiles each, bound by streaming the weights; all
    # 48 go to the library in one call, which runs the layers of one operand form in one launch of the tiled kernel
    Ts = 197
    small_layers = [(W, L.N, L.M, Ts) for W, L in zip(Ws, layers)]
    small_packed, small_ws = nm.nm_pack_prepare_batched(small_layers, stream=stream)
    small_Y = [torch.empty((Ts, L.O), dtype=torch.bfloat16, device=dev) for L in layers]
    small_descs = nm.forward_descs([(v, i, L.K, L.N, L.M, X[:Ts], ws, None, Y) for (v, i), ws, X, Y, L in
                                    zip(small_packed, small_ws, Xs, small_Y, layers)])

    def small_products():
        nm.nm_linear_forward_prepared_batched(small_descs, stream=stream)

    small_ms = timed(small_products)
    small_bytes = sum((ws.numel() if ws is not None else v.numel() * 2 + i.numel() * 4) + 2 * Ts * (L.K + L.O)
                      for (v, i), ws, L in zip(small_packed, small_ws, layers))
    small_batch = {"workload": "the 48 linears at batch 1 (T=197), bf16 out, one batched call; bytes = operand-form weights "
                               "+ X + Y of every layer",
                   "ms": small_ms, "algorithmic_bytes": small_bytes,
                   "useful_tflops": sum(2.0 * Ts * L.O * L.K * L.N / L.M for L in layers) / small_ms / 1e9,
                   "roofline": {"bound": "hbm", "achieved": small_bytes / small_ms / 1e6, "peak": PEAK_HBM_GBS,
                                "unit": "GB/s", "frac": small_bytes / small_ms / 1e6 / PEAK_HBM_GBS}}
    del small_packed, small_ws, small_Y, small_descs

    # ---- context, not part of the path: the vendor library's dense bf16 product (torch.matmul) on the same four
    # shapes with unpruned weights, i.e. what the block costs without any sparsity
    try:
        def dense_library():
            for j in train_layers:
                torch.matmul(Xs[j], Ws[j].t(), out=Ys[j])

        lib_ms = timed(dense_library)
        sparse_block_ms = None
        if layer_ms:
            sparse_block_ms = sum(layer_ms[j] for j in train_layers)
        dense_library_reference = {
            "workload": "torch.matmul (vendor dense bf16 GEMM) on the four products of one DeiT-B block at batch 256, "
                        "unpruned weights, bf16 out",
            "ms": lib_ms, "tflops": block_flops / lib_ms / 1e9}
        if sparse_block_ms:
            dense_library_reference["this_library_block_ms_at_seed0_levels"] = sparse_block_ms
    except Exception as e:  # the comparison is optional
        dense_library_reference = {"error": str(e)[:200]}

    if args.report:
        log(f"training products of one block: dX {dx_ms:.3f} ms ({training['input_gradient']['roofline']['achieved']:.0f} "
            f"TFLOP/s), dW {dw_ms:.3f} ms ({training['weight_gradient']['roofline']['achieved']:.0f} TFLOP/s)")
        log(f"int8 products of one block: {q_ms:.3f} ms ({q_tops:.0f} useful TOP/s, "
            f"{int8['dense_equivalent_tops']:.0f} dense-equivalent)")
        log(f"batch 1 (T=197), 48 products in one call: {small_ms * 1e3:.1f} us "
            f"({small_batch['roofline']['achieved']:.0f} GB/s of weights + activations)")
        if "ms" in dense_library_reference:
            log(f"for scale, the vendor library's dense bf16 product on the block's four shapes: "
                f"{dense_library_reference['ms']:.3f} ms ({dense_library_reference['tflops']:.0f} TFLOP/s)")
        log(f"nested levels: rank 48 matrices {rank_ms:.3f} ms ({nested['rank']['roofline']['achieved']:.0f} GB/s), "
            f"pack from ranks {pr_ms:.3f} ms ({nested['pack_ranked']['roofline']['achieved']:.0f} GB/s)")
        log(f"{'layer':<12}{'N:M':>6}{'ms':>9}{'useful TF/s':>13}{'dense-eq TF/s':>15}{'% bf16 peak':>13}{'% of ceiling':>14}")
        for L, ms in zip(layers, layer_ms or []):
            u = L.useful_flops / ms / 1e9
            log(f"{L.name:<12}{L.N:>3}:{L.M:<3}{ms:>8.3f}{u:>13.1f}{L.dense_flops / ms / 1e9:>15.1f}{100 * u / PEAK_BF16_DENSE_TFLOPS:>12.1f}%"
                f"{100 * ceiling_ms(L) / ms:>13.1f}%")
        wbytes = sum(L.O * L.K * 2 for L in layers)
        obytes = sum(v.numel() * 2 + i.numel() * 4 for v, i in packed)
        sbytes = sum(nm.nm_spmm_workspace_bytes(L.O, L.K, L.N, L.M, L.T) for L in layers)
        log(f"select + pack + operand order (48 matrices, one launch): {pack_ms:.3f} ms, "
            f"{(wbytes + obytes + sbytes) / pack_ms / 1e6:.0f} GB/s ({wbytes / 1e6:.0f} MB read, "
            f"{obytes / 1e6:.0f} MB packed + {sbytes / 1e6:.0f} MB operand order written)")

    out = {
        "metric": "N:M sparse-linear useful TFLOP/s (% bf16 MFMA peak), DeiT-B b=256",
        "value": useful / dt / 1e12,
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": dt * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "deit_b_linear_stack_batch256: 48 linears, T=50432, layer-wise N:M seed 0 from "
                               "{1:4,2:4,1:8,2:8,4:8,1:16,4:16}; step = select + pack 48 weights (one launch) + 48 sparse products, bf16 out",
                   "tokens": T, "layers": len(layers), "product_schedule": args.schedule},
        "pct_of_bf16_dense_peak": 100.0 * useful / dt / 1e12 / PEAK_BF16_DENSE_TFLOPS,
        "dense_equivalent_tflops": dense / dt / 1e12,
        "pack_ms": pack_ms,
        # the stack's time if every product ran at its own roof (nominal matrix-core or HBM peak), over the step
        "fraction_of_ceiling": sum(ceiling_ms(L) for L in layers) / (dt * 1e3),
        "roofline": roofline,
        "nested_levels": nested,
        "training_products": training,
        "int8_products": int8,
        "small_batch_products": small_batch,
        "dense_library_reference": dense_library_reference,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
