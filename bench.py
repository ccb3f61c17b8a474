#!/usr/bin/env python3
"""Benchmark of the k3 hot path on one MI355X.

Default workload ("cfg2"): the 3-D U-Net encoder block -- two 3x3x3 conv + ReLU layers
(32 -> 32 channels) and a 2x2x2 max-pool on a 1 x 64^3 volume, bf16 with fp32
accumulation, forward + backward (both weight gradients, both data gradients, pool
backward).  A step is one pass of that block; the step is captured in a HIP graph so the
~10 kernel launches are not bound by host launch latency.  The headline value is the
exact (in-bounds) convolution FLOPs of the step divided by the step time; the same K steps
are timed five more times and the spread (min / median / max) is reported beside it.

The default run also carries the rest of the metric (skipped with --quick):
"peaks_measured" -- this box's own matrix-core and HBM rates (a register-resident bf16 MFMA
loop, a device copy), against which every rate is printed beside the nominal peaks;
"layers" -- per-launch time and TFLOP/s of single 3x3x3 layers at the shapes that carry the
large U-Net steps; "unet" -- the base-64 U-Net step on 2 x 256^3 (workload config 4)
without swapping, with every stored encoder activation swapped, and under a device-memory
budget of three quarters of its unswapped footprint (refused without swapping, completed
with the planner's swap plan): voxels/s, overhead, overlap fraction and the link rates the
copies reached against the box's own pinned-memory copy rates.

Other workloads: "unet128" (full 4-level U-Net, base 32, 1 x 128^3, no swapping),
"unet256" (base 64, 2 x 256^3) and "unet320" (base 64, 4 x 320^3) print the unabridged
"unet" object (the plan listings included; --budget-gb sets the budget).  "bp64" / "bp96" time
the paper's second model (section 4.1: two conv+pool encoder layers, two conv+up-sampling
decoder layers, 128 channels, batch of 8 blocks, class-weighted loss) in training and inference.  "sweep" plans
and runs a row of resolutions under one fixed budget and reports the swap overhead of each.
--pmc-pass / --pmc-parse / --stats-md are the helpers the summaries under profiles/ were made with.

Prints ONE JSON line on stdout.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2516.6   # 256 CU x 4096 FLOP/clk x 2.4 GHz, dense
HBM_PEAK_GBS = 8000.0


def conv_flops(n, d, h, w, cin, cout):
    """Exact multiply-add FLOPs of one 3x3x3 pass: taps that fall into the zero padding are not counted."""
    return 2.0 * n * cin * cout * (3 * d - 2) * (3 * h - 2) * (3 * w - 2)


def time_calls(fn, iters, warm=3, graph=False):
    """Average duration (ms) of fn() over `iters` back-to-back calls, HIP events on the launch stream.
    graph=True: the calls are captured into one HIP graph first (as the benchmark step is), which
    takes the host's launch cost out of the gaps between the kernels."""
    import torch
    for _ in range(warm):
        fn()
    run = None
    if graph:
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for _ in range(iters):
                fn()
        g.replay()
        run = g.replay
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    if run is not None:
        run()
    else:
        for _ in range(iters):
            fn()
    e1.record()
    e1.synchronize()
    return e0.elapsed_time(e1) / iters


# ----------------------------------------------------------------------------- cfg2
def bench_cfg2(args):
    import numpy as np
    import torch
    import synth
    from paper_1811_12174_amd import k3

    N, S, C = 1, 64, 32
    bf = torch.bfloat16

    def dev(a):
        return torch.from_numpy(a).cuda().to(bf).contiguous()

    x = dev(synth.activations(1, (N, S, S, S, C), "bf16"))
    w1 = dev(synth.conv_weights(2, C, C, "bf16"))
    w2 = dev(synth.conv_weights(3, C, C, "bf16"))
    b1 = torch.zeros(C, device="cuda")
    b2 = torch.zeros(C, device="cuda")
    dyp = dev(synth.activations(4, (N, S // 2, S // 2, S // 2, C), "bf16"))
    pk1 = torch.empty(k3.conv3d_packed_bytes(C, C, k3.BF16), device="cuda", dtype=torch.uint8)
    pk2 = torch.empty_like(pk1)
    k3.conv3d_pack_weights(w1, pk1)
    k3.conv3d_pack_weights(w2, pk2)
    a1, a2, da2, da1, dx = (torch.empty_like(x) for _ in range(5))
    p = torch.empty_like(dyp)
    dW1, dW2 = torch.empty((3, 3, 3, C, C), device="cuda"), torch.empty((3, 3, 3, C, C), device="cuda")
    db1, db2 = torch.empty(C, device="cuda"), torch.empty(C, device="cuda")
    ws = torch.empty(k3.conv3d_bwd_weight_workspace_bytes(x, a1), device="cuda", dtype=torch.uint8)

    a1bits = torch.empty(k3.relu_bits_bytes(a1) // 2, device="cuda", dtype=torch.int16)
    a2route = torch.empty(k3.relu_bits_bytes(a2) // 2, device="cuda", dtype=torch.int16)

    def step():
        # conv1 also writes the one-bit-per-element ReLU mask of its output, which conv2's
        # backward-data pass applies to the gradient it produces
        k3.conv3d_fwd_bits(x, w1, pk1, b1, 1, a1, a1bits)
        k3.conv3d_fwd(a1, w2, pk2, b2, 1, a2)
        # the pooling layer keeps one routing bit per element of a2 (first maximum of its window
        # and > 0) and its backward pass reads those instead of a2
        k3.pool3d_fwd_bits(a2, p, a2route)
        # each producer of an activation gradient applies the ReLU mask of the tensor it
        # differentiates (pool backward: a2; conv2 backward-data: a1), so the conv backward
        # passes read no mask
        k3.pool3d_bwd_bits(a2route, dyp, da2)
        k3.conv3d_bwd_weight(a1, da2, None, dW2, db2, ws)
        k3.conv3d_bwd_data_bits(da2, None, w2, pk2, da1, a1bits)
        k3.conv3d_bwd_weight(x, da1, None, dW1, db1, ws)
        k3.conv3d_bwd_data(da1, None, w1, pk1, dx)

    for _ in range(3):
        step()
    torch.cuda.synchronize()
    run = step
    graph = None
    if not args.no_graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        run = graph.replay
    # per-call timings (events on the launch stream), same launch configuration as the step
    it = max(20, args.steps // 4)
    gr = not args.no_graph
    kern = {
        "conv3d_fwd": time_calls(lambda: k3.conv3d_fwd(a1, w2, pk2, b2, 1, a2), it, graph=gr),
        "conv3d_bwd_data": time_calls(lambda: k3.conv3d_bwd_data_bits(da2, None, w2, pk2, da1, a1bits), it, graph=gr),
        "conv3d_bwd_weight": time_calls(lambda: k3.conv3d_bwd_weight(a1, da2, None, dW2, db2, ws), it, graph=gr),
        # (the fused convolution + pool call saves a launch but lengthens the convolution by as much: not used in the step)
        "conv3d_fwd_pool": time_calls(lambda: k3.conv3d_fwd_pool(a1, w2, pk2, b2, 1, a2, p), it, graph=gr),
        "pool3d_fwd_bits": time_calls(lambda: k3.pool3d_fwd_bits(a2, p, a2route), it, graph=gr),
        "pool3d_bwd_bits": time_calls(lambda: k3.pool3d_bwd_bits(a2route, dyp, da2), it, graph=gr),
        # (the forms that keep and re-read a2 instead of the routing bits: not used in the step)
        "pool3d_fwd": time_calls(lambda: k3.pool3d_fwd(a2, p), it, graph=gr),
        "pool3d_bwd": time_calls(lambda: k3.pool3d_bwd(a2, dyp, None, da2, relu_mask=True), it, graph=gr),
    }

    def mix():   # the implicit-GEMM kernel as the step launches it: 2 forward + 2 backward-data passes
        k3.conv3d_fwd_bits(x, w1, pk1, b1, 1, a1, a1bits)
        k3.conv3d_fwd(a1, w2, pk2, b2, 1, a2)
        k3.conv3d_bwd_data_bits(da2, None, w2, pk2, da1, a1bits)
        k3.conv3d_bwd_data(da1, None, w1, pk1, dx)
    mfma_ms = time_calls(mix, it, graph=not args.no_graph) / 4.0
    # the step itself, timed last: the GPU has then been busy for a while and holds its steady clocks
    for _ in range(args.warmup):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    # the same K steps timed REPEATS more times: how much one box scatters (the value above is the first timing)
    rep = [ms]
    for _ in range(args.repeats):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            run()
        torch.cuda.synchronize()
        rep.append((time.perf_counter() - t0) * 1e3 / args.steps)
    rep.sort()

    f1 = conv_flops(N, S, S, S, C, C)
    step_flops = 6 * f1
    value = step_flops / (ms * 1e-3) / 1e12

    # (the weight-gradient call is two launches: the MFMA kernel and the small split-K reduction)
    wgrad_ms = kern["conv3d_bwd_weight"]
    share = {"conv_mfma_zs_kernel": 4 * mfma_ms, "conv_wgrad_pipe_kernel": 2 * wgrad_ms}
    dominant = max(share, key=share.get)
    dom_ms = mfma_ms if dominant == "conv_mfma_zs_kernel" else wgrad_ms
    achieved = f1 / (dom_ms * 1e-3) / 1e12
    roofline = {"bound": "mfma", "kernel": dominant, "achieved": round(achieved, 2), "peak": MFMA_BF16_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4),
                "flops_per_launch": f1, "avg_launch_ms": round(dom_ms, 5), "traffic": load_traffic(dominant, "cfg2")}
    out = {
        "metric": "3D conv fwd+bwd TFLOP/s", "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "cfg2: encoder block, 2x(conv3x3x3 32->32 + ReLU) + 2x2x2 max-pool, N=1, 64^3, fwd+bwd",
                   "hip_graph": graph is not None, "launches_per_step": 10, "conv_passes_per_step": 6, "flops_per_step": step_flops},
        "pct_mfma_peak": round(100 * value / MFMA_BF16_PEAK_TFLOPS, 2),
        "voxels_per_s": round(N * S ** 3 / (ms * 1e-3), 1),
        "ms_per_step_spread": {"repeats": len(rep), "min": round(rep[0], 5), "median": round(rep[len(rep) // 2], 5),
                               "max": round(rep[-1], 5)},
        "roofline": roofline,
        "call_ms": {k: round(v, 5) for k, v in kern.items()},
        "call_tflops": {k: round(f1 / (kern[k] * 1e-3) / 1e12, 2) for k in ("conv3d_fwd", "conv3d_bwd_data", "conv3d_bwd_weight")},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline_cfg2(step_flops)
    return out


def cpu_baseline_cfg2(step_flops):
    """The oracle, as it stands, on the same block (one full forward + backward), timed on the host cores."""
    import numpy as np
    import oracle
    import synth
    oracle.build(force=False)
    N, S, C = 1, 64, 32
    x = synth.activations(1, (N, S, S, S, C), "bf16").astype(np.float64)
    w1 = synth.conv_weights(2, C, C, "bf16").astype(np.float64)
    w2 = synth.conv_weights(3, C, C, "bf16").astype(np.float64)
    dyp = synth.activations(4, (N, S // 2, S // 2, S // 2, C), "bf16").astype(np.float64)
    def one_step():
        a1 = oracle.conv3d_fwd(x, w1, None, relu=True)
        a2 = oracle.conv3d_fwd(a1, w2, None, relu=True)
        oracle.pool3d_fwd(a2)
        g2 = oracle.relu_bwd(oracle.pool3d_bwd(a2, dyp), a2)
        oracle.conv3d_bwd_weight(a1, g2)
        g1 = oracle.relu_bwd(oracle.conv3d_bwd_data(g2, w2), a1)
        oracle.conv3d_bwd_weight(x, g1)
        oracle.conv3d_bwd_data(g1, w1)
    # whole steps until about ten seconds of CPU work have been timed (at least one, at most 40)
    t0 = time.perf_counter()
    n = 0
    while n < 1 or (time.perf_counter() - t0 < 10.0 and n < 40):
        one_step()
        n += 1
    dt = time.perf_counter() - t0
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    out = {"value": round(n * step_flops / dt / 1e12, 5), "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
           "seconds": round(dt, 2),
           "sample": f"{n} full cfg2 steps (6 conv passes + pool fwd/bwd each) in fp64 direct loops"}
    # the same loops on one thread: one forward pass over an eighth of the volume (about a second)
    try:
        import ctypes
        gomp = ctypes.CDLL("libgomp.so.1")
        gomp.omp_set_num_threads(1)
        xs = np.ascontiguousarray(x[:, :S // 2, :S // 2, :S // 2, :])
        t1 = time.perf_counter()
        oracle.conv3d_fwd(xs, w1, None, relu=True)
        d1 = time.perf_counter() - t1
        gomp.omp_set_num_threads(threads)
        out["one_thread"] = {"value": round(conv_flops(N, S // 2, S // 2, S // 2, C, C) / d1 / 1e12, 6), "unit": "TFLOP/s",
                             "sample": f"one conv3d_fwd pass, 1 x {S // 2}^3, {C}->{C}"}
    except OSError:
        pass
    return out


def measure_peaks():
    """The two machine rates of this very box: the register-resident bf16 MFMA loop (what the
    matrix cores sustain at the clock the chip holds under full matrix load) and a plain device
    copy (what a streaming kernel gets from HBM, bytes read + written).  Best of five launches."""
    import torch
    from paper_1811_12174_amd import k3
    blocks = 256 * 8
    sink = torch.empty(blocks * 256, device="cuda", dtype=torch.float32)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    k3.probe_mfma_bf16(200, blocks, sink)
    best = 0.0
    for _ in range(5):
        e0.record()
        fl = k3.probe_mfma_bf16(20000, blocks, sink)
        e1.record()
        e1.synchronize()
        best = max(best, fl / (e0.elapsed_time(e1) * 1e-3) / 1e12)
    src = torch.ones(1 << 30, device="cuda", dtype=torch.uint8)
    dst = torch.empty_like(src)
    k3.probe_copy(src, dst, 4096)
    copy = 0.0
    for grid in (1024, 2048, 4096, 8192, 1024):   # the best launch shape differs a little between boxes
        e0.record()
        k3.probe_copy(src, dst, grid)
        e1.record()
        e1.synchronize()
        copy = max(copy, 2.0 * src.numel() / (e0.elapsed_time(e1) * 1e-3) / 1e9)
    return {"mfma_bf16_tflops": round(best, 1), "mfma_pct_of_nominal": round(100 * best / MFMA_BF16_PEAK_TFLOPS, 1),
            "hbm_copy_gbs": round(copy, 1), "hbm_pct_of_nominal": round(100 * copy / HBM_PEAK_GBS, 1),
            "how": "register-resident 32x32x16 bf16 MFMA loop, 2048 workgroups x 4 waves; 1 GiB grid-stride device copy (read + write)"}


def bench_layers(args, mfma_measured):
    """Single 3x3x3 layers at the shapes that carry the base-64 U-Net step (cfg4 / cfg5) and the
    base-32 level 0 (cfg3): per launch time, TFLOP/s over the exact in-bounds FLOPs, fraction of
    the nominal and of the measured matrix-core peak.  Launches are captured in a HIP graph."""
    import torch
    import synth
    from paper_1811_12174_amd import k3
    bf = torch.bfloat16
    out = []
    for (n, s, c) in ((2, 128, 64), (2, 64, 128), (1, 128, 32)):
        t = layer_tensors(n, s, c)
        x, g, w, b, pk, y, dx, dW, db, ws = (t[k] for k in ("x", "g", "w", "b", "pk", "y", "dx", "dW", "db", "ws"))
        fl = conv_flops(n, s, s, s, c, c)
        it = 10 if n * s ** 3 * c > (1 << 26) else 20
        ms = {"fwd": time_calls(lambda: k3.conv3d_fwd(x, w, pk, b, 1, y), it, graph=True),
              "dgrad": time_calls(lambda: k3.conv3d_bwd_data(g, None, w, pk, dx), it, graph=True),
              "wgrad": time_calls(lambda: k3.conv3d_bwd_weight(x, g, None, dW, db, ws), it, graph=True)}
        row = {"shape": f"{n}x{s}^3 {c}->{c}", "gflop_per_pass": round(fl / 1e9, 2)}
        for k, v in ms.items():
            tf = fl / (v * 1e-3) / 1e12
            row[k] = {"ms": round(v, 4), "tflops": round(tf, 1), "frac": round(tf / MFMA_BF16_PEAK_TFLOPS, 4),
                      "frac_of_measured": round(tf / mfma_measured, 4) if mfma_measured else None}
        out.append(row)
        del t, x, g, y, dx, ws
    return out


def compact_unet(u):
    """The figures of a bench_unet result that the one-line record carries (the plan listings stay out)."""
    keep = ("ms_per_step", "voxels_per_s", "overhead_pct", "ms_copies_only", "overlap_fraction", "achieved_gbs_out",
            "achieved_gbs_in", "achieved_pct_of_one_direction_peak", "copies_only_pct_of_link", "accounted_peak_gb",
            "device_budget_gb", "no_swap_under_budget", "swap_under_budget")
    out = {k: u[k] for k in ("workload", "steps", "ms_per_step_no_swap", "voxels_per_s_no_swap", "conv_tflops_no_swap",
                             "pct_mfma_peak_no_swap", "accounted_peak_gb_no_swap", "link_gbs") if k in u}
    for leg in ("encoder_activations_swapped", "planned_for_budget"):
        if leg in u:
            o = {k: u[leg][k] for k in keep if k in u[leg]}
            if isinstance(o.get("no_swap_under_budget"), str):
                o["no_swap_under_budget"] = o["no_swap_under_budget"][:7]
            if "bytes_out_per_step" in u[leg]:
                o["gb_out"] = round(u[leg]["bytes_out_per_step"] / 1e9, 2)
                o["gb_in"] = round(u[leg]["bytes_in_per_step"] / 1e9, 2)
            if "plan" in u[leg]:
                o["tensors_swapped"] = len(u[leg]["plan"]["swapped_tensors"])
                o["predicted_ms"] = u[leg]["plan"]["predicted_ms"]
            out[leg] = o
    return out


def load_traffic(kernel, workload):
    """HBM bytes per launch (fetched + written) measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE and
    scaled by the same counters on a copy kernel of known size; null when not recorded."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        with open(path) as f:
            t = json.load(f)
        rec = t.get(workload, {}).get(kernel)
        return None if rec is None else rec.get("bytes_per_launch")
    except (OSError, ValueError):
        return None


# ----------------------------------------------------------------------------- HBM traffic counters
def layer_tensors(n, s, c):
    """Seeded tensors, packed weights and outputs of one n x s^3, c -> c layer."""
    import torch
    import synth
    from paper_1811_12174_amd import k3
    bf = torch.bfloat16
    t = {}
    if n * s ** 3 * c <= (1 << 28):
        t["x"] = torch.from_numpy(synth.activations(11, (n, s, s, s, c), "bf16")).cuda().to(bf)
        t["g"] = torch.from_numpy(synth.activations(12, (n, s, s, s, c), "bf16")).cuda().to(bf)
    else:   # the host generator would need minutes: seeded N(0,1) values made on the device
        gen = torch.Generator(device="cuda")
        gen.manual_seed(181112174)
        t["x"] = torch.empty((n, s, s, s, c), device="cuda", dtype=bf)
        t["g"] = torch.empty((n, s, s, s, c), device="cuda", dtype=bf)
        for i in range(n):
            t["x"][i] = torch.randn((s, s, s, c), device="cuda", generator=gen).to(bf)
            t["g"][i] = torch.randn((s, s, s, c), device="cuda", generator=gen).to(bf)
    t["w"] = torch.from_numpy(synth.conv_weights(13, c, c, "bf16")).cuda().to(bf)
    t["b"] = torch.zeros(c, device="cuda")
    t["pk"] = torch.empty(k3.conv3d_packed_bytes(c, c, k3.BF16), device="cuda", dtype=torch.uint8)
    k3.conv3d_pack_weights(t["w"], t["pk"])
    t["y"], t["dx"] = torch.empty_like(t["x"]), torch.empty_like(t["x"])
    t["dW"], t["db"] = torch.empty((3, 3, 3, c, c), device="cuda"), torch.empty(c, device="cuda")
    t["ws"] = torch.empty(k3.conv3d_bwd_weight_workspace_bytes(t["x"], t["g"]), device="cuda", dtype=torch.uint8)
    return t


def run_layer(t, reps):
    from paper_1811_12174_amd import k3
    for _ in range(reps):
        k3.conv3d_fwd(t["x"], t["w"], t["pk"], t["b"], 1, t["y"])
        k3.conv3d_bwd_data(t["g"], None, t["w"], t["pk"], t["dx"])
        k3.conv3d_bwd_weight(t["x"], t["g"], None, t["dW"], t["db"], t["ws"])


def pmc_pass(args):
    """Workload for `rocprofv3 --pmc FETCH_SIZE` / `--pmc WRITE_SIZE` (and for kernel traces of single
    layers): a device copy of known size (the calibration of the counter) followed by a few launches of
    every cfg2 call, or -- with --layer N,S,C -- of the forward, backward-data and backward-weight pass
    of one N x S^3, C -> C layer."""
    import torch
    import synth
    from paper_1811_12174_amd import k3
    N, S, C = 1, 64, 32
    bf = torch.bfloat16
    src = torch.ones(64 << 20, device="cuda", dtype=torch.float32)   # 256 MiB read + 256 MiB written
    dst = torch.empty_like(src)
    for _ in range(3):
        torch.add(src, 1.0, out=dst)   # a plain elementwise kernel: reads 256 MiB, writes 256 MiB
    if args.layer:
        n, s, c = args.layer
        run_layer(layer_tensors(n, s, c), args.layer_reps)
        torch.cuda.synchronize()
        print(json.dumps({"pmc_pass": "done", "layer": [n, s, c], "copy_bytes_read": src.numel() * 4,
                          "copy_bytes_written": src.numel() * 4}))
        return
    x = torch.from_numpy(synth.activations(1, (N, S, S, S, C), "bf16")).cuda().to(bf)
    w = torch.from_numpy(synth.conv_weights(2, C, C, "bf16")).cuda().to(bf)
    dyp = torch.from_numpy(synth.activations(4, (N, S // 2, S // 2, S // 2, C), "bf16")).cuda().to(bf)
    b = torch.zeros(C, device="cuda")
    pk = torch.empty(k3.conv3d_packed_bytes(C, C, k3.BF16), device="cuda", dtype=torch.uint8)
    k3.conv3d_pack_weights(w, pk)
    a1, a2, da2, da1 = (torch.empty_like(x) for _ in range(4))
    p = torch.empty_like(dyp)
    dW, db = torch.empty((3, 3, 3, C, C), device="cuda"), torch.empty(C, device="cuda")
    ws = torch.empty(k3.conv3d_bwd_weight_workspace_bytes(x, a1), device="cuda", dtype=torch.uint8)
    a1bits = torch.empty(k3.relu_bits_bytes(a1) // 2, device="cuda", dtype=torch.int16)
    a2route = torch.empty(k3.relu_bits_bytes(a2) // 2, device="cuda", dtype=torch.int16)
    for _ in range(3):
        k3.conv3d_fwd_bits(x, w, pk, b, 1, a1, a1bits)
        k3.conv3d_fwd(a1, w, pk, b, 1, a2)
        k3.pool3d_fwd_bits(a2, p, a2route)
        k3.pool3d_bwd_bits(a2route, dyp, da2)
        k3.conv3d_bwd_weight(a1, da2, None, dW, db, ws)
        k3.conv3d_bwd_data_bits(da2, None, w, pk, da1, a1bits)
        k3.conv3d_bwd_data(da1, None, w, pk, a2)
    torch.cuda.synchronize()
    print(json.dumps({"pmc_pass": "done", "copy_bytes_read": src.numel() * 4, "copy_bytes_written": src.numel() * 4}))


def pmc_parse(fetch_csv, write_csv, key="cfg2", path=None):
    """Turns the two counter_collection.csv files of a pair of pmc passes into the entry `key` of
    profiles/traffic.json (other entries of the file are kept)."""
    import csv
    import collections

    def per_kernel(path, counter):
        acc, cnt = collections.defaultdict(float), collections.Counter()
        with open(path) as f:
            for r in csv.DictReader(f):
                if r["Counter_Name"] != counter:
                    continue
                acc[r["Kernel_Name"]] += float(r["Counter_Value"])
                cnt[r["Kernel_Name"]] += 1
        return {k: acc[k] / cnt[k] for k in acc}

    fetch, write = per_kernel(fetch_csv, "FETCH_SIZE"), per_kernel(write_csv, "WRITE_SIZE")
    copy = [k for k in fetch if "FunctorOnSelf_add" in k][:1]   # the 256 MiB elementwise add of the pass
    if not copy:
        raise SystemExit("no copy kernel found in the counter files")
    known = float(64 << 20) * 4
    f_scale = known / (fetch[copy[0]] * 1024.0)    # counters are in KiB per dispatch
    w_scale = known / (write[copy[0]] * 1024.0)
    path = path or os.path.join(ROOT, "profiles", "traffic.json")
    try:
        with open(path) as f:
            out = json.load(f)
    except (OSError, ValueError):
        out = {}
    cal = {"copy_kernel": copy[0], "known_bytes_each_way": known, "fetch_counter_kib": fetch[copy[0]],
           "write_counter_kib": write[copy[0]], "fetch_scale": f_scale, "write_scale": w_scale}
    out.setdefault("_calibration", {})
    if "copy_kernel" in out["_calibration"]:      # older layout: one calibration for the file
        out["_calibration"] = {"cfg2": out["_calibration"]}
    out["_calibration"][key] = cal
    out[key] = {}
    for k in fetch:
        if "k3::" not in k:
            continue
        short = k.split("k3::")[1].split("<")[0].split("(")[0]
        fb, wb = fetch[k] * 1024.0 * f_scale, write.get(k, 0.0) * 1024.0 * w_scale
        rec = out[key].setdefault(short, {"variants": {}})
        rec["variants"][k] = {"fetch_bytes": round(fb), "write_bytes": round(wb)}
    for short, rec in out[key].items():
        v = list(rec["variants"].values())
        rec["fetch_bytes"] = round(sum(x["fetch_bytes"] for x in v) / len(v))
        rec["write_bytes"] = round(sum(x["write_bytes"] for x in v) / len(v))
        rec["bytes_per_launch"] = rec["fetch_bytes"] + rec["write_bytes"]
    with open(path, "w") as f:
        json.dump(out, f, indent=1, sort_keys=True)
    print("wrote", path, "entry", key)


def stats_md(csv_path, top=12):
    """rocprofv3's kernel_stats.csv as a markdown table (durations in microseconds), for profiles/*.md."""
    import csv
    import re
    rows = list(csv.DictReader(open(csv_path)))
    out = ["| kernel | calls | total us | avg us | min us | max us | % |", "|---|---|---|---|---|---|---|"]
    for r in rows[:top]:
        name = re.sub(r"\(.*$", "", r["Name"])[:110]
        out.append(f"| `{name}` | {r['Calls']} | {float(r['TotalDurationNs']) / 1e3:.1f} | {float(r['AverageNs']) / 1e3:.2f} | "
                   f"{float(r['MinNs']) / 1e3:.2f} | {float(r['MaxNs']) / 1e3:.2f} | {float(r['Percentage']):.2f} |")
    print("\n".join(out))


# ----------------------------------------------------------------------------- U-Net steps
def unet_flops(base, levels, n, size):
    """Exact conv FLOPs of one forward + backward U-Net step (3x3x3 layers only; no dgrad for the first layer)."""
    import synth
    total = 0.0
    res = {}
    for name, kind, ci, co in synth.unet_plan(base, 1, levels, 3):
        if kind != "conv":
            continue
        l = int(name[3])
        s = size // 2 ** l
        f = conv_flops(n, s, s, s, ci, co)
        total += f * (2 if name == "enc0.conv1" else 3)
    return total


def measure_link(nbytes=1 << 30, reps=4):
    """Rates (GB/s) of the swap engine's own copies (hipMemcpyAsync between device and page-locked
    host memory on its two copy streams) on this machine: each direction alone, and each direction
    with both busy."""
    import torch
    from paper_1811_12174_amd import k3
    dev_a = torch.empty(nbytes, device="cuda", dtype=torch.uint8)
    dev_b = torch.empty(nbytes, device="cuda", dtype=torch.uint8)
    ctx = k3.lms_create(0)
    h1, h2 = k3.lms_host_alloc(nbytes), k3.lms_host_alloc(nbytes)

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return round(nbytes * reps / (time.perf_counter() - t0) / 1e9, 1)
    try:
        def out():
            h = k3.lms_swap_out(ctx, dev_a.data_ptr(), nbytes, h1)
            k3.lms_sync(ctx)
            k3.lms_release(ctx, h)
        d2h = timed(out)
        hb = k3.lms_swap_out(ctx, dev_b.data_ptr(), nbytes, h2)
        k3.lms_sync(ctx)
        k3.lms_release_after(ctx, hb)

        def back():
            k3.lms_prefetch_start(ctx, hb, dev_b.data_ptr())
            k3.lms_sync(ctx)
            k3.lms_evict(ctx, hb)
        h2d = timed(back)

        def both():
            ha = k3.lms_swap_out(ctx, dev_a.data_ptr(), nbytes, h1)
            k3.lms_prefetch_start(ctx, hb, dev_b.data_ptr())
            k3.lms_sync(ctx)
            k3.lms_evict(ctx, hb)
            k3.lms_release(ctx, ha)
        each = timed(both)
        k3.lms_release(ctx, hb)
    finally:
        k3.lms_host_free(h1)
        k3.lms_host_free(h2)
        k3.lms_destroy(ctx)
    return {"d2h_alone": d2h, "h2d_alone": h2d, "each_direction_both_busy": each}


def bench_unet(args, base, size, n, swap, label, budget_gb=0.0):
    import numpy as np
    import torch
    import synth
    from paper_1811_12174_amd import k3, planner
    from paper_1811_12174_amd.executor import OutOfBudget
    from paper_1811_12174_amd.unet import UNet3D
    params = synth.unet_params(base=base, levels=4, dtype="bf16")
    x = torch.from_numpy(synth.volume_field(7, n, size, dtype="bf16")).cuda().to(torch.bfloat16)
    lab = torch.from_numpy(synth.ellipsoid_labels(8, n, size)).cuda()
    net = UNet3D(params, base=base, levels=4)
    steps, warm = max(1, args.unet_steps), 2
    prog = net.program(x.shape)
    fixed = net.fixed_bytes(prog)

    def run(**kw):
        for _ in range(warm):
            net.step(x, lab, **kw)
        torch.cuda.synchronize()
        if net.lms is not None:
            k3.lms_sync(net.lms)
        torch.cuda.reset_peak_memory_stats()
        t0 = time.perf_counter()
        for _ in range(steps):
            net.step(x, lab, **kw)
        torch.cuda.synchronize()
        if net.lms is not None:
            k3.lms_sync(net.lms)
        return (time.perf_counter() - t0) / steps

    def swap_leg(plan, budget):
        net.step(x, lab, swap=plan, budget=budget)       # creates the swap context on first use
        torch.cuda.synchronize()
        k3.lms_sync(net.lms)
        k3.lms_set_copy_timing(net.lms, True)
        busy0 = k3.lms_copy_busy_ms(net.lms)
        dt = run(swap=plan, budget=budget)
        busy1 = k3.lms_copy_busy_ms(net.lms)
        k3.lms_set_copy_timing(net.lms, False)
        r = net.last_run
        n_steps = warm + steps
        busy_out, busy_in = (busy1[0] - busy0[0]) / n_steps * 1e-3, (busy1[1] - busy0[1]) / n_steps * 1e-3
        # the same instruction stream with its copies but without its kernels: what the link alone needs
        net.copies_only = True
        try:
            t_copy = run(swap=plan, budget=budget)
        finally:
            net.copies_only = False
        shorter = min(t_noswap, t_copy)
        return {"ms_per_step": round(dt * 1e3, 3), "voxels_per_s": round(V / dt, 1),
                "overhead_pct": round(100 * (dt / t_noswap - 1), 2),
                "ms_compute_only": round(t_noswap * 1e3, 3), "ms_copies_only": round(t_copy * 1e3, 3),
                "overlap_fraction": round((t_noswap + t_copy - dt) / shorter, 3) if shorter > 0 else None,
                # achieved rate of the engine's copies inside the real step: bytes over the time the
                # copy stream of that direction was busy (timed event pairs around every copy)
                "copy_busy_ms_out": round(busy_out * 1e3, 2), "copy_busy_ms_in": round(busy_in * 1e3, 2),
                "achieved_gbs_out": round(r.bytes_out / busy_out / 1e9, 1) if busy_out > 0 else None,
                "achieved_gbs_in": round(r.bytes_in / busy_in / 1e9, 1) if busy_in > 0 else None,
                "achieved_pct_of_one_direction_peak": (round(100 * min(r.bytes_out / busy_out / 1e9 / link["d2h_alone"],
                                                                       r.bytes_in / busy_in / 1e9 / link["h2d_alone"]), 1)
                                                       if link and busy_out > 0 and busy_in > 0 else None),
                "link_gbs_out_copies_only": round(r.bytes_out / t_copy / 1e9, 1) if t_copy > 0 else None,
                "link_gbs_in_copies_only": round(r.bytes_in / t_copy / 1e9, 1) if t_copy > 0 else None,
                # the copies alone against the best the link could do with these byte counts: both
                # directions busy for the smaller count, one direction for the rest
                "copies_only_pct_of_link": (round(100 * link_seconds(r.bytes_out, r.bytes_in, link) / t_copy, 1)
                                            if link and t_copy > 0 else None),
                "accounted_peak_gb": round(r.peak / 1e9, 3), "allocator_peak_gb": round(torch.cuda.max_memory_allocated() / 1e9, 3),
                "bytes_out_per_step": int(r.bytes_out), "bytes_in_per_step": int(r.bytes_in),
                "copy_seconds_at_link_peak": round(max(r.bytes_out, r.bytes_in) / 57e9, 4),
                "device_copies_dropped": r.releases, "plan": plan.describe()}

    link = measure_link() if (swap or budget_gb) else None

    def link_seconds(b_out, b_in, rates):
        lo, hi = min(b_out, b_in), max(b_out, b_in)
        return lo / (rates["each_direction_both_busy"] * 1e9) + (hi - lo) / (min(rates["d2h_alone"], rates["h2d_alone"]) * 1e9)

    V = n * size ** 3
    t_noswap = run()
    need = net.last_run.peak      # accounted bytes the unswapped step holds
    fl = unet_flops(base, 4, n, size)
    res = {"workload": label, "steps": steps, "ms_per_step_no_swap": round(t_noswap * 1e3, 3),
           "voxels_per_s_no_swap": round(V / t_noswap, 1), "conv_tflops_no_swap": round(fl / t_noswap / 1e12, 2),
           "pct_mfma_peak_no_swap": round(100 * fl / t_noswap / 1e12 / MFMA_BF16_PEAK_TFLOPS, 2),
           "accounted_peak_gb_no_swap": round(net.last_run.peak / 1e9, 3),
           "allocator_peak_gb_no_swap": round(torch.cuda.max_memory_allocated() / 1e9, 3)}
    # weight update (SGD with momentum over the parameter arena + rebuild of the packed weights)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(5):
        net.sgd_step(0.0, 0.9, 0.0)   # lr = 0: same work, weights unchanged
    torch.cuda.synchronize()
    res["weight_update_ms"] = round((time.perf_counter() - t0) / 5 * 1e3, 3)
    res["parameters"] = int(net.n_params)
    # per-call GPU durations of this very workload feed the planner's simulator
    net.step(x, lab, timing=True)
    dur = net.call_seconds
    if link:
        res["link_gbs"] = link
    if swap:
        # every stored encoder activation spends its idle gaps in host memory (the paper's default:
        # swap the feature maps), in the smallest budget that selection can run in
        plan = planner.swap_all(prog, only=planner.is_encoder_activation, fixed_bytes=fixed, durations=dur)
        res["encoder_activations_swapped"] = swap_leg(plan, plan.budget)
        res["encoder_activations_swapped"]["device_budget_gb"] = round(plan.budget / 1e9, 3)
    if swap and not budget_gb:
        budget_gb = round(0.75 * need / 1e9, 3)   # default: three quarters of what the step needs unswapped
    if budget_gb:
        # The situation the paper's LMS exists for: a device-memory limit below what the step
        # needs without swapping.  The planner picks what leaves the GPU; the limit is enforced
        # by the step's own slab allocator; allocator_peak_gb is what torch's allocator really handed out.
        budget = int(budget_gb * 1e9)
        leg = {"device_budget_gb": budget_gb}
        try:
            net.step(x, lab, swap=False, budget=budget)
            torch.cuda.synchronize()
            leg["no_swap_under_budget"] = "completed"
        except OutOfBudget as e:
            leg["no_swap_under_budget"] = "refused: " + str(e)
        try:
            plan = planner.plan_for_budget(prog, budget, fixed_bytes=fixed, durations=dur)
        except OutOfBudget as e:
            leg["swap_under_budget"] = "no plan fits: " + str(e)
            plan = None
        if plan is not None:
            leg.update(swap_leg(plan, budget))
            leg["swap_under_budget"] = "completed"
        res["planned_for_budget"] = leg
    net.close()
    return res


def bench_bp(args, size):
    """The section-4.1 encoder / decoder: batch of 8 blocks of size^3 voxels, 128 channels,
    class-weighted loss; one step = forward + backward + SGD update.  Also the inference pass
    (forward + arg-max read-out)."""
    import torch
    import synth
    from paper_1811_12174_amd.unet import EncoderDecoder3D
    n, ch = 8, 128
    params = synth.bp_params(cin=1, channels=ch, dtype="bf16")
    x = torch.from_numpy(synth.volume_field(7, n, size, dtype="bf16")).cuda().to(torch.bfloat16)
    labh = synth.ellipsoid_labels(8, n, size)
    lab = torch.from_numpy(labh).cuda()
    net = EncoderDecoder3D(params, cin=1, channels=ch, class_weights=synth.inverse_frequency_class_weights(labh))
    steps, warm = max(1, args.unet_steps) * 5, 3

    def timed(fn):
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps

    def train():
        net.step(x, lab)
        net.sgd_step(0.0, 0.9, 0.0)   # lr = 0: the full update work, weights unchanged
    t_train = timed(train)
    t_infer = timed(lambda: net.classify(x))
    net.step(x, lab, timing=True)
    prog = net.program(x.shape)
    per_call = sorted(((d, f"{c.fn} {c.layer or ''}".strip()) for c, d in zip(prog.calls, net.call_seconds)), reverse=True)[:6]
    fl = sum(c.flops for c in prog.calls if c.fn.startswith("conv_"))
    V = n * size ** 3
    res = {"workload": f"section-4.1 encoder/decoder, 8 x {size}^3, 128 channels, class-weighted loss", "steps": steps,
           "ms_per_training_step": round(t_train * 1e3, 3), "training_voxels_per_s": round(V / t_train, 1),
           "conv_tflops": round(fl / t_train / 1e12, 2), "ms_per_inference_pass": round(t_infer * 1e3, 3),
           "inference_voxels_per_s": round(V / t_infer, 1), "accounted_peak_gb": round(net.last_run.peak / 1e9, 3),
           "slowest_calls_ms": [[name, round(d * 1e3, 3)] for d, name in per_call]}
    net.close()
    return res


def bench_sweep(args):
    """Swap overhead against resolution at a fixed device budget (the paper's section 3 reports
    the overhead of LMS growing with the image resolution on its 16 GB GPUs): base-64 U-Net, batch
    2, edge 192 ... 288, every step planned for the same budget."""
    out = []
    for size in args.sweep_edges:
        u = bench_unet(args, 64, size, 2, False, f"U-Net base 64, 2 x {size}^3", budget_gb=args.sweep_budget_gb)
        leg = u["planned_for_budget"]
        row = {"edge": size, "no_swap_ms": u["ms_per_step_no_swap"], "no_swap_peak_gb": u["accounted_peak_gb_no_swap"],
               "no_swap_under_budget": leg["no_swap_under_budget"][:7], "swap_under_budget": leg["swap_under_budget"][:12]}
        if leg["swap_under_budget"] == "completed":
            row.update({"planned_ms": leg["ms_per_step"], "overhead_pct": leg["overhead_pct"],
                        "predicted_ms": leg["plan"]["predicted_ms"], "peak_gb": leg["accounted_peak_gb"],
                        "gb_out": round(leg["bytes_out_per_step"] / 1e9, 2), "gb_in": round(leg["bytes_in_per_step"] / 1e9, 2),
                        "tensors_swapped": len(leg["plan"]["swapped_tensors"])})
        print("sweep", json.dumps(row), file=sys.stderr, flush=True)
        out.append(row)
        import gc
        import torch
        gc.collect()
        torch.cuda.synchronize()
        torch.cuda.empty_cache()   # every size starts from an empty block cache
    return {"device_budget_gb": args.sweep_budget_gb, "rows": out}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--workload", default="cfg2", choices=["cfg2", "unet128", "unet256", "unet320", "sweep", "bp64", "bp96"])
    ap.add_argument("--budget-gb", type=float, default=0.0,
                    help="U-Net workloads: also run under this device-memory limit, without and with swapping")
    ap.add_argument("--sweep-budget-gb", type=float, default=32.0, help="device budget of the sweep workload")
    ap.add_argument("--sweep-edges", type=int, nargs="+", default=[192, 208, 224, 240, 256, 272, 288, 304],
                    help="volume edges of the sweep workload (multiples of 8)")
    ap.add_argument("--unet-steps", type=int, default=2)
    ap.add_argument("--repeats", type=int, default=5, help="cfg2: further timings of the same K steps (spread)")
    ap.add_argument("--quick", action="store_true",
                    help="cfg2: the block only, without the single-layer list, the machine peaks and the cfg4 U-Net legs")
    ap.add_argument("--detail", default="", help="also write the full (unabridged) result as JSON to this path")
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--pmc-pass", action="store_true", help="run the short workload the HBM-traffic counters are collected on")
    ap.add_argument("--pmc-parse", nargs=2, metavar=("FETCH_CSV", "WRITE_CSV"),
                    help="write an entry of profiles/traffic.json from the counter files of two --pmc-pass runs")
    ap.add_argument("--pmc-key", default="cfg2", help="name of that entry (the workload the passes ran)")
    ap.add_argument("--layer", type=lambda v: tuple(int(x) for x in v.split(",")), default=None, metavar="N,S,C",
                    help="--pmc-pass: run the three passes of one N x S^3, C -> C layer instead of the cfg2 calls")
    ap.add_argument("--layer-reps", type=int, default=5)
    ap.add_argument("--stats-md", default="", metavar="KERNEL_STATS_CSV",
                    help="print rocprofv3's kernel_stats.csv as a markdown table and exit")
    args = ap.parse_args()
    if args.pmc_parse:
        pmc_parse(*args.pmc_parse, key=args.pmc_key)
        return
    if args.stats_md:
        stats_md(args.stats_md)
        return
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the paper's multi-GPU all-reduce is out of scope); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the k3 kernels have no CPU fallback", file=sys.stderr)
        sys.exit(1)
    from paper_1811_12174_amd import k3
    k3.lib()
    if args.pmc_pass:
        pmc_pass(args)
        return
    if args.workload == "cfg2":
        out = bench_cfg2(args)
        if not args.quick:
            # the rest of the metric: the machine's own peaks, the layers that carry the large steps,
            # and the cfg4 U-Net step without swapping, with every encoder activation swapped and
            # under a device budget of three quarters of its unswapped footprint
            pk = measure_peaks()
            out["peaks_measured"] = pk
            out["pct_of_measured_mfma_peak"] = round(100 * out["value"] / pk["mfma_bf16_tflops"], 2)
            out["roofline"]["frac_of_measured"] = round(out["roofline"]["achieved"] / pk["mfma_bf16_tflops"], 4)
            out["layers"] = bench_layers(args, pk["mfma_bf16_tflops"])
            import gc
            gc.collect()
            torch.cuda.empty_cache()
            full = bench_unet(args, 64, 256, 2, True, "cfg4: U-Net base 64, 2 x 256^3, fwd+bwd")
            out["unet"] = compact_unet(full)
            if args.detail:
                with open(args.detail, "w") as f:
                    json.dump({"line": out, "unet_full": full}, f, indent=1)
    elif args.workload in ("bp64", "bp96"):
        u = bench_bp(args, 64 if args.workload == "bp64" else 96)
        out = {"metric": "encoder/decoder training step voxels/s", "value": u["training_voxels_per_s"], "unit": "voxels/s",
               "n_gpus": 1, "steps": u["steps"], "warmup": 3, "ms_per_step": u["ms_per_training_step"], "higher_is_better": True,
               "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
               "config": {"workload": u["workload"]}, "encoder_decoder": u}
    elif args.workload == "sweep":
        sw = bench_sweep(args)
        done = [r for r in sw["rows"] if "planned_ms" in r]
        last = done[-1]
        out = {"metric": "U-Net step voxels/s under a device budget", "value": round(2 * last["edge"] ** 3 / (last["planned_ms"] * 1e-3), 1),
               "unit": "voxels/s", "n_gpus": 1, "steps": max(1, args.unet_steps), "warmup": 2, "ms_per_step": last["planned_ms"],
               "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
               "config": {"workload": f"swap-overhead sweep, U-Net base 64, batch 2, edge {sw['rows'][0]['edge']}..{sw['rows'][-1]['edge']}, "
                                      f"budget {sw['device_budget_gb']} GB; value is the largest edge that ran"},
               "sweep": sw}
    else:
        if args.workload == "unet128":
            u = bench_unet(args, 32, 128, 1, False, "cfg3: U-Net base 32, 1 x 128^3, no swapping")
        elif args.workload == "unet256":
            u = bench_unet(args, 64, 256, 2, True, "cfg4: U-Net base 64, 2 x 256^3, swap plan for a device budget",
                           budget_gb=args.budget_gb)
        else:
            u = bench_unet(args, 64, 320, 4, True, "cfg5: U-Net base 64, 4 x 320^3, swap plan for a device budget",
                           budget_gb=args.budget_gb)
        sw = u.get("planned_for_budget", {})
        value = sw.get("voxels_per_s", u["voxels_per_s_no_swap"])
        ms = sw.get("ms_per_step", u["ms_per_step_no_swap"])
        out = {"metric": "U-Net step voxels/s", "value": value, "unit": "voxels/s", "n_gpus": 1, "steps": u["steps"],
               "warmup": 2, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
               "dtype": "bf16", "data": "synthetic", "config": {"workload": u["workload"]}, "unet": u}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
