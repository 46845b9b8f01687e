#!/usr/bin/env python3
"""Benchmark of the N:M-sparse linear hot path on one MI355X.

One step = one pass of the whole path over the DeiT-B batch-256 linear stack (50432 tokens, 12 blocks
x {qkv, proj, fc1, fc2}, layer-wise level drawn with seed 0 from {1:4,2:4,1:8,2:8,4:8,1:16,4:16}):
magnitude N:M selection + packing of all 48 weights (one batched launch), then the 48 sparse-weight x
dense-activation products from the packed form (bf16 in, fp32 accumulate, bf16 out).  All inputs are
resident in HBM before the timed region.  Prints ONE JSON line; besides the headline it carries the
other workloads (single 2:4 layer, DeiT-B block at batch 64, Swin-B-shaped stages, batch 1), the rates
measured on the device in the same process, and the parity of the timed buffers with the CPU checker.

    python bench.py [--gpus 1] [--steps K] [--warmup W]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_DENSE_TFLOPS = 2500.0  # MI355X dense bf16 matrix-core peak
PEAK_HBM_GBS = 8000.0            # MI355X HBM3E
PEAK_INT8_DENSE_TOPS = 5000.0    # MI355X dense int8 matrix-core peak
INDEX_BITS = {4: 2, 8: 3, 16: 4}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


# ------------------------------------------------------------------------------------------------------
# bytes and floors of one layer
# ------------------------------------------------------------------------------------------------------
def packed_weight_bytes(L):
    """The packed form: kept values (2 bytes) + log2(M)-bit positions, index rows padded to 32 bits."""
    fields = L.K // L.M * L.N
    return L.O * (fields * 2 + (fields * INDEX_BITS[L.M] + 31) // 32 * 4)


def algorithmic_bytes(L, out_bytes=2):
    """HBM bytes one product has to move: X once, the packed weight once, Y once."""
    return 2.0 * L.T * L.K + packed_weight_bytes(L) + out_bytes * L.T * L.O


def floors_ms(L, out_bytes=2):
    """(matrix-core floor, HBM floor) of one product on nominal peaks.  A level with N <= 2 runs on the 2:4
    sparse instruction at half the dense instruction count, the others on the dense one."""
    math = L.dense_flops * (0.5 if L.N <= 2 and L.N < L.M else 1.0) / (PEAK_BF16_DENSE_TFLOPS * 1e12)
    hbm = algorithmic_bytes(L, out_bytes) / (PEAK_HBM_GBS * 1e9)
    return math * 1e3, hbm * 1e3


def ceiling_ms(L, out_bytes=2):
    return max(floors_ms(L, out_bytes))


def hbm_roofline(nbytes, ms, **extra):
    gbs = nbytes / ms / 1e6
    return dict({"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS,
                 "traffic": None}, **extra)


def mfma_roofline(flops, ms, peak=PEAK_BF16_DENSE_TFLOPS, unit="TFLOP/s", **extra):
    tf = flops / ms / 1e9
    return dict({"bound": "mfma", "achieved": tf, "peak": peak, "unit": unit, "frac": tf / peak, "traffic": None}, **extra)


# ------------------------------------------------------------------------------------------------------
# inputs
# ------------------------------------------------------------------------------------------------------
def build_inputs(layers, torch, wl, seed=0):
    """Weights: one Gaussian draw per layer.  Activations: one Gaussian draw per input width (768 and 3072);
    every layer gets its own device copy, rolled by its index along the token axis, so that no two layers share
    HBM lines or cache contents.  Returns the device tensors and the host bit patterns they were made from."""
    from paper_2409_09708_amd import bf16_tensor as dev_bf16
    rng = np.random.default_rng(seed)
    x_host, base = {}, {}
    for L in layers:
        if L.K not in base:
            x_host[L.K] = wl.draw_activations(rng, L.T, L.K)
            base[L.K] = dev_bf16(x_host[L.K])
    Ws, Xs, w_host = [], [], []
    for i, L in enumerate(layers):
        w_host.append(wl.draw_weights(rng, L.O, L.K))
        Ws.append(dev_bf16(w_host[-1]))
        Xs.append(torch.roll(base[L.K], shifts=i, dims=0).contiguous())
    return Ws, Xs, w_host, x_host


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


# ------------------------------------------------------------------------------------------------------
# parity of timed buffers with the CPU checker
# ------------------------------------------------------------------------------------------------------
def compare_output(y_host, Yref, B, workers):
    """max |Y - Yref| / B over all elements and the relative Frobenius error, in row chunks on `workers`
    threads.  y_host: bf16 bit patterns (uint16) or float32, [T, O]."""
    T = Yref.shape[0]
    step = max(256, (T + 4 * workers - 1) // (4 * workers))

    def part(r0):
        r1 = min(T, r0 + step)
        y = y_host[r0:r1]
        if y.dtype == np.uint16:
            y = (y.astype(np.uint32) << 16).view(np.float32)
        d = y.astype(np.float64) - Yref[r0:r1]
        finite = bool(np.isfinite(d).all())
        ratio = float((np.abs(d) / (B[r0:r1] + 1e-30)).max())
        return ratio, float((d * d).sum()), float((Yref[r0:r1] ** 2).sum()), finite

    with ThreadPoolExecutor(max_workers=workers) as pool:
        parts = list(pool.map(part, range(0, T, step)))
    ratio = max(p[0] for p in parts)
    fro = (sum(p[1] for p in parts) / max(sum(p[2] for p in parts), 1e-300)) ** 0.5
    if not all(p[3] for p in parts):
        ratio = float("inf")
    return ratio, fro


def oracle_stack(wl, layers, w_host, x_host, timed_outputs):
    """The CPU checker as it stands on the whole step, once: per layer select + pack + fp64 product with its
    bound, timed; and (untimed) the comparison of the GPU's packed bytes and outputs of the timed step with
    them, every element.  timed_outputs[j] = (values bits, index words, Y bits rolled back to the base
    activation order), or None to time only."""
    from oracle import nm_oracle as orc
    cores = len(os.sched_getaffinity(0))
    dt, useful = 0.0, 0.0
    worst_ratio, worst_fro, bytes_equal, checked = 0.0, 0.0, True, 0
    for j, L in enumerate(layers):
        t0 = time.perf_counter()
        m = orc.nm_mask(w_host[j], L.N, L.M)
        vals, idx = orc.nm_pack(w_host[j], m, L.N, L.M)
        Yref, B = orc.nm_linear(x_host[L.K], w_host[j], m)
        dt += time.perf_counter() - t0
        useful += L.useful_flops
        if timed_outputs is not None:
            v, i, y = timed_outputs[j]
            bytes_equal = bytes_equal and np.array_equal(v, vals) and np.array_equal(i, idx)
            ratio, fro = compare_output(y, Yref, B, cores)
            worst_ratio, worst_fro = max(worst_ratio, ratio), max(worst_fro, fro)
            checked += 1
            timed_outputs[j] = None
        del Yref, B, m
    base = {"value": useful / dt / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "sample": f"all {len(layers)} layers at their drawn levels on all {layers[0].T} tokens, once: numpy select + "
                      f"pack + fp64 dense product and its bound product, {dt:.2f} s"}
    parity = None
    if timed_outputs is not None:
        parity = {"checked_layers": checked, "elements": "all", "packed_bytes_equal": bool(bytes_equal),
                  "max_err_over_bound": worst_ratio, "max_fro": worst_fro,
                  "pass": bool(bytes_equal and worst_ratio <= 1e-2 and worst_fro <= 5e-3)}
    return base, parity


# ------------------------------------------------------------------------------------------------------
# one layer at a time: the other workloads
# ------------------------------------------------------------------------------------------------------
def time_call(torch, stream, fn, reps, warm=3):
    """Median and minimum duration (ms) of fn, each repetition bracketed by events on the launch stream."""
    for _ in range(warm):
        fn()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for a, b in ev:
        a.record(stream)
        fn()
        b.record(stream)
    torch.cuda.synchronize()
    ts = [a.elapsed_time(b) for a, b in ev]
    return float(np.median(ts)), float(min(ts))


def measure_layers(nm, torch, wl, layers, seed, stream, reps, out_dtype, check, dense_reference=True):
    """Each layer of a workload as its own prepared product call: duration (events around the call, median of
    `reps`), rates, floors; the vendor library's dense product on the same shape for scale; and the timed output
    compared with the CPU checker, every element."""
    from oracle import nm_oracle as orc
    from paper_2409_09708_amd import bf16_tensor as dev_bf16
    cores = len(os.sched_getaffinity(0))
    out_bytes = 2 if out_dtype == torch.bfloat16 else 4
    rows = []
    for L, Xh, Wh in wl.draw_layers(layers, seed=seed):
        X, W = dev_bf16(Xh), dev_bf16(Wh)
        (packed,), (ws,) = nm.nm_pack_prepare_batched([(W, L.N, L.M, L.T)], stream=stream)
        Y = torch.full((L.T, L.O), float("nan"), dtype=out_dtype, device=X.device)
        call = lambda: nm.nm_linear_forward_prepared(packed[0], packed[1], L.K, L.N, L.M, X, ws, out=Y, stream=stream)
        ms, ms_min = time_call(torch, stream, call, reps)
        math_ms, hbm_ms = floors_ms(L, out_bytes)
        row = {"layer": L.name, "T": L.T, "K": L.K, "O": L.O, "level": f"{L.N}:{L.M}", "ms": ms, "ms_min": ms_min,
               "useful_tflops": L.useful_flops / ms / 1e9, "dense_equivalent_tflops": L.dense_flops / ms / 1e9,
               "hbm_gbs": algorithmic_bytes(L, out_bytes) / ms / 1e6,
               "bound": "hbm" if hbm_ms >= math_ms else "mfma", "frac_of_ceiling": max(math_ms, hbm_ms) / ms}
        if dense_reference:
            Yd = torch.empty((L.T, L.O), dtype=torch.bfloat16, device=X.device)
            row["dense_library_ms"] = time_call(torch, stream, lambda: torch.matmul(X, W.t(), out=Yd), reps)[0]
            del Yd
        if check:
            y_host = Y.cpu().numpy() if out_dtype == torch.float32 else nm.bf16_bits(Y)
            Yref, B = orc.nm_linear_from_bits(Xh, Wh, L.N, L.M)
            ratio, fro = compare_output(y_host, Yref, B, cores)
            row["max_err_over_bound"], row["fro"] = ratio, fro
            row["parity_pass"] = bool(ratio <= 1e-2 and fro <= 5e-3)
            del Yref, B
        rows.append(row)
        del X, W, Y, packed, ws
    return rows


def measured_peaks(nm, torch, stream):
    """Rates measured on this device in this process: loops of nothing but matrix instructions (2:4 sparse and
    dense bf16), and a plain streaming copy of 1 GiB."""
    out = {}
    sink = None
    for kind, name in ((0, "smfmac_f32_16x16x64_bf16"), (1, "mfma_f32_16x16x32_bf16")):
        ops = 0

        def run():
            nonlocal sink, ops
            sink, ops = nm.nm_probe_matrix_rate(kind, 4000, sink=sink, stream=stream)

        ms, ms_min = time_call(torch, stream, run, 5, warm=2)
        out[name] = {"dense_equivalent_tflops": ops / ms / 1e9, "best": ops / ms_min / 1e9, "ms": ms}
    src = torch.empty((1 << 30,), dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    ms, ms_min = time_call(torch, stream, lambda: nm.nm_probe_copy(src, dst, stream=stream), 5, warm=2)
    out["copy_1GiB"] = {"read_plus_write_gbs": 2 * src.numel() / ms / 1e6, "best": 2 * src.numel() / ms_min / 1e6, "ms": ms}
    del src, dst
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--schedule", default="batched", choices=("batched", "streams", "single"),
                    help="how the 48 independent products of a step are launched")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the CPU checker (no cpu_baseline, no parity)")
    ap.add_argument("--headline-only", action="store_true", help="skip the other workloads and the side measurements")
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
    Ws, Xs, w_host, x_host = build_inputs(layers, torch, wl)
    log(f"inputs ready in {time.perf_counter() - t_gen:.1f} s")

    packed = [(torch.empty((L.O, L.K // L.M * L.N), dtype=torch.bfloat16, device=dev),
               torch.empty((L.O, nm.nm_index_bytes(L.O, L.K, L.N, L.M) // (4 * L.O)), dtype=torch.int32, device=dev))
              for L in layers]
    # outputs start as NaN: a tile the product never wrote fails the comparison below
    Ys = [torch.full((L.T, L.O), float("nan"), dtype=torch.bfloat16, device=dev) for L in layers]
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
    # one stream (what a model whose layers depend on each other issues).
    side = torch.cuda.Stream(device=dev) if args.schedule == "streams" else None
    packed_ready, side_done = torch.cuda.Event(), torch.cuda.Event()
    entries = [(v, i, L.K, L.N, L.M, X, ws, None, Y) for L, (v, i), X, Y, ws in zip(layers, packed, Xs, Ys, workspaces)]
    descs = nm.forward_descs(entries)

    def step(schedule):
        # the whole path: select + pack all 48 weights and write their operand-order forms (one launch), then
        # the 48 products at each layer's own level
        nm.nm_pack_prepare_batched(pack_args, stream=stream, out=packed, workspaces=workspaces)
        if schedule == "batched":
            nm.nm_linear_forward_prepared_batched(descs, stream=stream)
            return
        if schedule == "streams":
            packed_ready.record(stream)
            side.wait_event(packed_ready)
        for n, (L, (v, i), X, Y, ws) in enumerate(zip(layers, packed, Xs, Ys, workspaces)):
            on = side if (schedule == "streams" and n % 2) else stream
            nm.nm_linear_forward_prepared(v, i, L.K, L.N, L.M, X, ws, out=Y, stream=on)
        if schedule == "streams":
            side_done.record(side)
            stream.wait_event(side_done)

    def timed_steps(schedule, warmup, steps):
        for _ in range(warmup):
            step(schedule)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step(schedule)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    if args.calibrate_copy:
        src = torch.empty((256 << 20,), dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        nm.nm_probe_copy(src, dst, stream=stream)
        torch.cuda.synchronize()
        del src, dst
    dt = timed_steps(args.schedule, args.warmup, args.steps)

    useful = sum(L.useful_flops for L in layers)
    dense = sum(L.dense_flops for L in layers)

    # ---- the outputs of the timed step, brought to the host for the comparison with the CPU checker further down
    # (every later pass over the step rewrites the same bytes; nothing else writes into these buffers)
    timed_outputs = None
    if not args.no_cpu_baseline:
        timed_outputs = []
        for j, ((v, i), Y) in enumerate(zip(packed, Ys)):
            y = np.roll(nm.bf16_bits(Y), -j, axis=0)  # row t of layer j's input is row t - j of the base draw
            timed_outputs.append((nm.bf16_bits(v), i.cpu().numpy().view(np.uint32), y))

    # ---- kernel durations with HIP events on the launch stream: a second pass over the same step with events
    # around the batched pack and around every product launch.  In the batched schedule the library launches the
    # persistent kernel once per operand form; the pass hands it the two groups one after the other, so each event
    # pair brackets exactly one kernel.
    reps = max(3, min(args.steps, 10))
    sp = [j for j, L in enumerate(layers) if L.N <= 2]
    dn = [j for j, L in enumerate(layers) if L.N > 2]
    sp_useful = sum(layers[j].useful_flops for j in sp)
    pk = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    if args.schedule == "batched":
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
    # every layer as its own launch (per-layer durations; the sums are the dominant kernel's time in the other
    # schedules)
    ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in layers] for _ in range(reps)]
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
    layer_ms = [float(np.median([ev[r][j][0].elapsed_time(ev[r][j][1]) for r in range(reps)])) for j in range(len(layers))]
    if args.schedule != "batched":
        sp_ms = sum(layer_ms[j] for j in sp)
        dn_ms = sum(layer_ms[j] for j in dn)
        sp_launches = len(sp)
    pack_ms = float(np.median([a.elapsed_time(b) for a, b in pk]))
    # the same step with one launch per layer on one stream
    seq_dt = dt if args.schedule == "single" else timed_steps("single", 1, max(3, args.steps // 2))

    # ---- dominant kernel: the persistent product in the 2:4 form (the 36 layers with N <= 2): one launch for all of
    # them in the batched schedule, one per layer otherwise.  Which roof binds it is decided on nominal peaks: the
    # later of the matrix-core floor (half the dense instruction count at the dense peak's rate x 2) and the HBM
    # floor of its algorithmic bytes (X + packed W + Y of every layer).
    sp_bytes = sum(algorithmic_bytes(layers[j]) for j in sp)
    sp_dense = sum(layers[j].dense_flops for j in sp)
    math_floor = sum(floors_ms(layers[j])[0] for j in sp)
    hbm_floor = sp_bytes / (PEAK_HBM_GBS * 1e9) * 1e3
    traffic = measured_traffic(args.schedule)
    launch_ms = sp_ms / sp_launches
    common = {"traffic": traffic, "traffic_source": "profiles/hbm_traffic_bench_deit_b256.txt (rocprofv3 FETCH_SIZE, WRITE_SIZE; "
                                                    "null when nm_spmm.hip has changed since)",
              "kernel": "nm_stream_kernel<sparse> (v_smfmac_f32_16x16x64_bf16) over the "
                        f"{len(sp)} layers with N <= 2, {sp_launches} launch(es) per step",
              "launches_per_step": sp_launches, "avg_launch_ms": launch_ms,
              "algorithmic_hbm_bytes_per_launch": sp_bytes / sp_launches,
              "useful_flops_per_launch": sp_useful / sp_launches,
              "hbm_floor_ms_per_launch": hbm_floor / sp_launches, "mfma_floor_ms_per_launch": math_floor / sp_launches,
              "hbm": {"achieved_gbs": sp_bytes / sp_ms / 1e6, "frac": sp_bytes / sp_ms / 1e6 / PEAK_HBM_GBS},
              "mfma": {"useful_tflops": sp_useful / sp_ms / 1e9, "frac_useful": sp_useful / sp_ms / 1e9 / PEAK_BF16_DENSE_TFLOPS,
                       "dense_equivalent_tflops": sp_dense / sp_ms / 1e9,
                       "frac_of_sparse_instruction_rate": sp_dense / sp_ms / 1e9 / (2 * PEAK_BF16_DENSE_TFLOPS)},
              "dense_form_kernel_ms_per_step": dn_ms}
    if hbm_floor >= math_floor:
        roofline = hbm_roofline(sp_bytes, sp_ms, **common)
    else:
        roofline = mfma_roofline(sp_useful, sp_ms, **common)

    per_layer = []
    for L, ms in zip(layers, layer_ms):
        m_ms, h_ms = floors_ms(L)
        per_layer.append({"layer": L.name, "level": f"{L.N}:{L.M}", "ms": ms, "useful_tflops": L.useful_flops / ms / 1e9,
                          "hbm_gbs": algorithmic_bytes(L) / ms / 1e6, "bound": "hbm" if h_ms >= m_ms else "mfma",
                          "frac_of_ceiling": max(m_ms, h_ms) / ms})

    # ---- select + pack: the step's launch also writes each layer's operand-order copy for the product kernel;
    # the packing alone (nm_pack_batched) is timed beside it.  Algorithmic bytes: 2 read per weight + the packed
    # bytes written.
    def timed(fn, n=reps):
        fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        for _ in range(n):
            fn()
        b.record(stream)
        torch.cuda.synchronize()
        return a.elapsed_time(b) / n

    n_weights = sum(L.O * L.K for L in layers)
    packed_bytes = sum(packed_weight_bytes(L) for L in layers)
    operand_bytes = sum(nm.nm_spmm_workspace_bytes(L.O, L.K, L.N, L.M, L.T) for L in layers)
    pack_only_args = [(W, L.N, L.M) for W, L in zip(Ws, layers)]
    pack_warm_ms = timed(lambda: nm.nm_pack_batched(pack_only_args, stream=stream, out=packed))
    # The 224 MB the packing moves fit the 256 MB memory-side cache, so calls in a row on the same weights are
    # served from it.  The HBM figure: 512 MB of other data read between the calls, events around each call.
    sweep = torch.zeros((64 << 20,), dtype=torch.int64, device=dev)
    cold = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for a, b in cold:
        sweep.max()  # reads 512 MB: what the cache held is gone, and nothing dirty is left behind
        a.record(stream)
        nm.nm_pack_batched(pack_only_args, stream=stream, out=packed)
        b.record(stream)
    torch.cuda.synchronize()
    pack_only_ms = float(np.median([a.elapsed_time(b) for a, b in cold]))
    del sweep
    pack = {"workload": "magnitude selection + packing of the 48 DeiT-B weight matrices (84.9 M weights), one launch",
            "algorithmic_bytes": 2.0 * n_weights + packed_bytes,
            "pack_only": {"ms": pack_only_ms, "ms_same_buffers": pack_warm_ms,
                          "note": "ms: the weights come from HBM (512 MB of other data read in between); ms_same_buffers: calls in "
                                  "a row, served by the memory-side cache",
                          "roofline": hbm_roofline(2.0 * n_weights + packed_bytes, pack_only_ms)},
            "pack_and_operand_order": {"ms": pack_ms, "operand_order_bytes_written": operand_bytes,
                                       "note": "the step's launch: also writes the product kernel's operand-order copy",
                                       "roofline": hbm_roofline(2.0 * n_weights + packed_bytes, pack_ms),
                                       "moved_gbs": (2.0 * n_weights + packed_bytes + operand_bytes) / pack_ms / 1e6}}

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
        "sequential": {"schedule": "one launch per layer on one stream", "ms_per_step": seq_dt * 1e3,
                       "value": useful / seq_dt / 1e12, "fraction_of_ceiling": sum(ceiling_ms(L) for L in layers) / (seq_dt * 1e3)},
        "roofline": roofline,
        "layers": per_layer,
        "pack": pack,
    }

    if not args.headline_only:
        # ---- nested levels (ranks inside groups): rank the 48 weights once for their M, then take each layer's
        # level from the ranks.  Streaming kernels: 2 read + 1/2 written per weight for the ranking; 2.5 read +
        # packed bytes written for the ranked pack.
        ranks = [torch.empty((L.O, L.K // 2), dtype=torch.uint8, device=dev) for L in layers]
        rank_args = [(W, L.M) for W, L in zip(Ws, layers)]
        ranked_args = [(W, r, L.N, L.M) for W, r, L in zip(Ws, ranks, layers)]
        rank_ms = timed(lambda: nm.nm_rank_batched(rank_args, stream=stream, out=ranks))
        pr_ms = timed(lambda: nm.nm_pack_ranked_batched(ranked_args, stream=stream, out=packed))
        out["nested_levels"] = {
            "workload": "48 DeiT-B weight matrices: ranking in one launch, packing from the ranks in one launch",
            "rank": {"ms": rank_ms, "algorithmic_bytes": 2.5 * n_weights, "roofline": hbm_roofline(2.5 * n_weights, rank_ms)},
            "pack_ranked": {"ms": pr_ms, "algorithmic_bytes": 2.5 * n_weights + packed_bytes,
                            "roofline": hbm_roofline(2.5 * n_weights + packed_bytes, pr_ms)}}
        del ranks

        # ---- training products of one transformer block (its four layers at their levels): dX = dY (W.m) and
        # dW = (dY^T X).m, dense matrix-core products of 2*T*O*K FLOPs each; a bf16 copy of the forward outputs
        # stands in for dY
        train_layers = list(range(4))
        dYs = [Ys[j].clone() for j in train_layers]
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
            for n in range(len(train_layers)):
                nm.nm_linear_backward_input(masked[n], dYs[n], out=dXs[n], stream=stream)

        def grad_weights():
            for n, j in enumerate(train_layers):
                nm.nm_linear_backward_weight(dYs[n], Xs[j], mask=words[n], out=dWs[n], workspace=gws[n], stream=stream)

        dx_ms, dw_ms = timed(grad_inputs), timed(grad_weights)
        block_flops = sum(layers[j].dense_flops for j in train_layers)
        out["training_products"] = {
            "workload": "one DeiT-B block at batch 256 (qkv, proj, fc1, fc2; T=50432): input gradients in bf16, "
                        "masked weight gradients in fp32; 2*T*O*K FLOPs per product",
            "input_gradient": {"ms": dx_ms, "roofline": mfma_roofline(block_flops, dx_ms)},
            "weight_gradient": {"ms": dw_ms, "roofline": mfma_roofline(block_flops, dw_ms)}}
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
                                                 w_scale=q_scale[n], out=dYs[n], stream=stream)

        q_ms = timed(int8_products)
        q_useful = sum(layers[j].useful_flops for j in train_layers)
        # floors of the four products: int8 X once, the compressed int8 weight (values + positions) once, bf16 Y
        # once; matrix instructions at the int8 dense rate, twice that on the 2:4 form
        q_bytes = q_math_ms = 0.0
        for j in train_layers:
            L = layers[j]
            fields = L.K // L.M * L.N
            q_bytes += L.T * L.K + L.O * (fields + (fields * INDEX_BITS[L.M] + 31) // 32 * 4) + 2.0 * L.T * L.O
            q_math_ms += L.dense_flops * (0.5 if L.N <= 2 and L.N < L.M else 1.0) / (PEAK_INT8_DENSE_TOPS * 1e12) * 1e3
        q_hbm_ms = q_bytes / (PEAK_HBM_GBS * 1e9) * 1e3
        q_mfma = mfma_roofline(q_useful, q_ms, peak=PEAK_INT8_DENSE_TOPS, unit="TOP/s", floor_ms=q_math_ms)
        q_hbm = hbm_roofline(q_bytes, q_ms, floor_ms=q_hbm_ms)
        out["int8_products"] = {
            "workload": "one DeiT-B block at batch 256 (qkv, proj, fc1, fc2 at their seed-0 levels), int8 operands, "
                        "int32 sums rescaled to bf16; useful operations 2*T*O*K*N/M; bound = the later floor",
            "ms": q_ms, "dense_equivalent_tops": block_flops / q_ms / 1e9, "algorithmic_bytes": q_bytes,
            "roofline": q_hbm if q_hbm_ms >= q_math_ms else q_mfma,
            "other_roof": q_mfma if q_hbm_ms >= q_math_ms else q_hbm}
        del q_masks, q_w, q_x, q_scale, q_ws

        # ---- context, not part of the path: the vendor library's dense bf16 product (torch.matmul) on the same four
        # shapes with unpruned weights, i.e. what the block costs without any sparsity
        try:
            def dense_library():
                for n, j in enumerate(train_layers):
                    torch.matmul(Xs[j], Ws[j].t(), out=dYs[n])

            lib_ms = timed(dense_library)
            out["dense_library_reference"] = {
                "workload": "torch.matmul (vendor dense bf16 GEMM) on the four products of one DeiT-B block at batch 256, "
                            "unpruned weights, bf16 out",
                "ms": lib_ms, "tflops": block_flops / lib_ms / 1e9,
                "this_library_block_ms_at_seed0_levels": sum(layer_ms[j] for j in train_layers)}
        except Exception as e:  # the comparison is optional
            out["dense_library_reference"] = {"error": str(e)[:200]}
        del dYs

        # ---- the same stack at batch 1 (197 tokens): products of a few tiles each, bound by streaming the weights;
        # all 48 go to the library in one call.  Algorithmic bytes: packed weights + X + Y of every layer.
        Ts = 197
        small_layers = [(W, L.N, L.M, Ts) for W, L in zip(Ws, layers)]
        small_packed, small_ws = nm.nm_pack_prepare_batched(small_layers, stream=stream)
        small_Y = [torch.empty((Ts, L.O), dtype=torch.bfloat16, device=dev) for L in layers]
        small_descs = nm.forward_descs([(v, i, L.K, L.N, L.M, X[:Ts], ws, None, Y) for (v, i), ws, X, Y, L in
                                        zip(small_packed, small_ws, Xs, small_Y, layers)])
        small_warm_ms = timed(lambda: nm.nm_linear_forward_prepared_batched(small_descs, stream=stream), n=20)
        # The 170 MB a call reads fit the 256 MB memory-side cache, so repeated calls on one set of buffers are
        # served from it.  The HBM figure comes from three sets of weights (packed + operand order, 510 MB) taken
        # in turn: a set has left the cache when its turn comes again.
        rot_sets = [(small_packed, small_ws)] + [nm.nm_pack_prepare_batched(small_layers, stream=stream) for _ in range(2)]
        rot_descs = [nm.forward_descs([(v, i, L.K, L.N, L.M, X[:Ts], ws, None, Y) for (v, i), ws, X, Y, L in
                                       zip(pk, wss, Xs, small_Y, layers)]) for (pk, wss) in rot_sets]
        turn = [0]

        def rotated_call():
            nm.nm_linear_forward_prepared_batched(rot_descs[turn[0] % 3], stream=stream)
            turn[0] += 1

        small_ms = timed(rotated_call, n=21)
        small_bytes = sum(packed_weight_bytes(L) + 2 * Ts * (L.K + L.O) for L in layers)
        operand_small = sum((ws.numel() if ws is not None else v.numel() * 2 + i.numel() * 4) + 2 * Ts * (L.K + L.O)
                            for (v, i), ws, L in zip(small_packed, small_ws, layers))
        # the same call without workspaces: the kernel that reads the packed format itself (2:4 layers need no
        # workspace either way)
        packed_descs = nm.forward_descs([(v, i, L.K, L.N, L.M, X[:Ts], None, None, Y) for (v, i), X, Y, L in
                                         zip(small_packed, Xs, small_Y, layers)])
        packed_ms = timed(lambda: nm.nm_linear_forward_prepared_batched(packed_descs, stream=stream), n=20)
        out["small_batch_products"] = {
            "workload": "the 48 linears at batch 1 (T=197), bf16 out, one batched call; algorithmic bytes = packed weights "
                        "+ X + Y of every layer; three sets of weight buffers (510 MB) taken in turn, so every call "
                        "reads its weights from HBM (ms_same_buffers: one set again and again, served by the 256 MB "
                        "memory-side cache)",
            "ms": small_ms, "ms_same_buffers": small_warm_ms, "algorithmic_bytes": small_bytes, "bytes_read_in_operand_form": operand_small,
            "useful_tflops": sum(2.0 * Ts * L.O * L.K * L.N / L.M for L in layers) / small_ms / 1e9,
            "roofline": hbm_roofline(small_bytes, small_ms),
            "without_workspace": {"note": "the kernel that decodes the packed format in registers: reads the algorithmic "
                                          "bytes, nothing to prepare", "ms": packed_ms,
                                  "roofline": hbm_roofline(small_bytes, packed_ms)}}
        del small_packed, small_ws, small_Y, small_descs, packed_descs, rot_sets, rot_descs

    # free the stack before the other workloads
    del Ws, Xs, Ys, packed, workspaces, entries, descs
    torch.cuda.empty_cache()

    if not args.headline_only:
        check = not args.no_cpu_baseline
        # ---- the other workloads, one prepared product call per layer (events around each call), outputs compared
        # with the CPU checker on every element
        cfg1 = measure_layers(nm, torch, wl, wl.single_2to4(), 0, stream, 50, torch.float32, check)
        cfg2 = measure_layers(nm, torch, wl, wl.deit_b_block(batch=64, seed=0), 0, stream, 20, torch.bfloat16, check)
        cfg4 = measure_layers(nm, torch, wl, wl.swin_b_stages(batch=64, seed=0), 0, stream, 20, torch.bfloat16, check)
        cfg5 = measure_layers(nm, torch, wl, wl.small_batch(), 0, stream, 50, torch.bfloat16, check)
        out["single_layer_2to4"] = {"workload": "X 197x384, W 384x384 at 2:4, fp32 out: one call, launch-latency bound",
                                    "latency_us": cfg1[0]["ms"] * 1e3, "layers": cfg1}
        out["deit_b_block_batch64"] = {
            "workload": "the four linears of a DeiT-B block at 12608 tokens, levels 4:8, 2:8, 1:8, 2:4 (seed 0), bf16 out",
            "ms": sum(r["ms"] for r in cfg2), "useful_tflops": sum(L.useful_flops for L in wl.deit_b_block(64, 0)) /
            sum(r["ms"] for r in cfg2) / 1e9, "layers": cfg2}
        out["swin_b_stages_batch64"] = {
            "workload": "one block per stage of a Swin-B-shaped hierarchy at batch 64 (C = 128 / 256 / 512 / 1024 with 200704 / "
                        "50176 / 12544 / 3136 tokens), level per stage from {2:4,1:8,2:8,2:16} (seed 0), bf16 out; stages "
                        "C = 128 and 256 are HBM-bound (hbm_gbs), C = 512 and 1024 nearer the matrix roof (useful_tflops)",
            "layers": cfg4,
            "slower_than_dense_library": [r["layer"] for r in cfg4 if r["ms"] > r.get("dense_library_ms", float("inf"))]}
        out["batch1_fc_layers"] = {"workload": "DeiT-B fc1 768->3072 and fc2 3072->768 at 197 tokens, 1:8 and 2:4, one call each",
                                   "layers": cfg5,
                                   "slower_than_dense_library": [r["layer"] for r in cfg5 if r["ms"] > r.get("dense_library_ms", float("inf"))]}
        out["measured_peaks"] = measured_peaks(nm, torch, stream)
        mp = out["measured_peaks"]
        out["roofline"]["frac_of_measured_peaks"] = {
            "hbm": roofline["hbm"]["achieved_gbs"] / mp["copy_1GiB"]["read_plus_write_gbs"],
            "sparse_instruction_rate": roofline["mfma"]["dense_equivalent_tflops"] / mp["smfmac_f32_16x16x64_bf16"]["dense_equivalent_tflops"]}

    if args.report:
        log(f"{'layer':<12}{'N:M':>6}{'ms':>9}{'useful TF/s':>13}{'GB/s':>9}{'bound':>7}{'% of ceiling':>14}")
        for r in per_layer:
            log(f"{r['layer']:<12}{r['level']:>6}{r['ms']:>9.3f}{r['useful_tflops']:>13.1f}{r['hbm_gbs']:>9.0f}{r['bound']:>7}"
                f"{100 * r['frac_of_ceiling']:>13.1f}%")
        log(f"step {dt * 1e3:.3f} ms batched, {seq_dt * 1e3:.3f} ms one launch per layer; 2:4-form launch {sp_ms:.3f} ms, "
            f"dense-form {dn_ms:.3f} ms, pack+operand order {pack_ms:.3f} ms, pack alone {pack_only_ms:.3f} ms")
        for key in ("single_layer_2to4", "deit_b_block_batch64", "swin_b_stages_batch64", "batch1_fc_layers"):
            for r in out.get(key, {}).get("layers", []):
                log(f"{key[:10]:<11}{r['layer']:<12}{r['level']:>6} T={r['T']:<7}{r['ms'] * 1e3:>9.1f} us {r['useful_tflops']:>8.1f} TF/s "
                    f"{r['hbm_gbs']:>7.0f} GB/s  ceiling {100 * r['frac_of_ceiling']:>5.1f}%  dense lib "
                    f"{r.get('dense_library_ms', 0) * 1e3:>8.1f} us  err/bound {r.get('max_err_over_bound', -1):.2e}")
        for key in ("nested_levels", "training_products", "int8_products", "small_batch_products", "measured_peaks", "pack"):
            if key in out:
                log(key, json.dumps(out[key]))

    if not args.no_cpu_baseline:
        out["cpu_baseline"], out["parity"] = oracle_stack(wl, layers, w_host, x_host, timed_outputs)
        extra = [r.get("parity_pass", True) for key in ("single_layer_2to4", "deit_b_block_batch64", "swin_b_stages_batch64",
                                                        "batch1_fc_layers") for r in out.get(key, {}).get("layers", [])]
        out["parity"]["other_workloads_pass"] = bool(all(extra))
        out["parity"]["other_workloads_checked_layers"] = len(extra)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
