#!/usr/bin/env python3
"""Throughput of the GDWS layer forward pass on one MI355X.

One step = one pass of the whole hot path (generalized depthwise + pointwise + epilogue)
over one batch of synthetic input already resident in HBM.  Default workload: the bf16
layer with C = M = 128 on 16 x 16 feature maps at batch 256, g from the greedy 25 % MAC
budget (G = 269).  Prints ONE JSON line with images/s, the dominant kernel's roofline
figures and the CPU oracle timed on the host cores.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

HBM_PEAK_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default="config2",
                    choices=["config2", "config2_g9", "config2_g1", "vgg16", "resnet18", "resnet50"],
                    help="config2 (default, the headline layer) and its two sub-runs, or one of the network-shaped "
                         "workloads (VGG-16 fp16 batch 256, ResNet-18 bf16 batch 512 at 32x32; ResNet-50 bf16 batch 128 "
                         "at 224x224)")
    ap.add_argument("--batch", type=int, default=0, help="network workloads: batch size (0 = the workload's own)")
    ap.add_argument("--layout", default="nhwc", choices=["nhwc", "nchw"])
    ap.add_argument("--mode", default="auto", choices=["auto", "fused", "unfused"])
    ap.add_argument("--rotate", type=int, default=16,
                    help="number of distinct input/output buffer pairs cycled through (keeps the working set "
                         "larger than the 256 MB last-level cache so HBM is what is measured)")
    ap.add_argument("--ramp-ms", type=float, default=60.0,
                    help="untimed launches of the same step for this many milliseconds before the warm-up steps: "
                         "from idle the GPU's clock governor needs some 30 ms of load to reach its steady state, "
                         "and a launch is 13 %% slower until then")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="additionally run a plain device copy of this many MiB a few times (the known-size "
                         "kernel that scales the FETCH_SIZE / WRITE_SIZE counters of a --pmc run)")
    return ap.parse_args()


def clock_ramp(step, ramp_ms):
    """Keep the GPU busy with step(i) for about ramp_ms so that its clocks are at their steady state."""
    import torch
    i, t0 = 0, time.perf_counter()
    while (time.perf_counter() - t0) * 1e3 < ramp_ms:
        for _ in range(50):
            step(i)
            i += 1
        torch.cuda.synchronize()


def measured_traffic(workload, layout):
    """HBM bytes per launch from the committed counter summary of this workload, or None."""
    path = os.path.join(ROOT, "profiles", f"fused_{workload}_{layout}_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1])
    except OSError:
        pass
    return None


def run_network(a):
    """Whole-network forward of a VGG-16 / ResNet-18 / ResNet-50 shaped stack (every 3x3 convolution a GDWS layer)."""
    import numpy as np
    import torch
    import paper_2110_14871_amd as gd
    import workloads
    from gpu_util import empty_act, to_device
    from net_util import build_network

    torch.cuda.set_device(0)
    dtype, batch, size, maker = {"vgg16": ("f16", 256, 32, workloads.vgg16_shape),
                                 "resnet18": ("bf16", 512, 32, workloads.resnet18_shape),
                                 "resnet50": ("bf16", 128, 224, workloads.resnet50_shape)}[a.workload]
    N = a.batch or batch
    shapes = maker(size, size)
    net, _ = build_network(shapes, dtype, a.layout)
    x, _ = to_device(workloads.rng.normal(900, (N, 3, size, size)), dtype, a.layout)
    last = shapes[-1]
    y = empty_act(N, last.M, last.Ho, last.Wo, dtype, a.layout)
    ws = torch.empty(max(1, gd.gdws_net_workspace_bytes(net, N, size, size)), dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream()
    clock_ramp(lambda i: gd.gdws_network_forward(net, x, y, N, size, size, workspace=ws, stream=stream), a.ramp_ms)
    for _ in range(a.warmup):
        gd.gdws_network_forward(net, x, y, N, size, size, workspace=ws, stream=stream)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record(stream)
    for _ in range(a.steps):
        gd.gdws_network_forward(net, x, y, N, size, size, workspace=ws, stream=stream)
    ev1.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / a.steps
    dev_ms = ev0.elapsed_time(ev1) / a.steps
    # algorithmic traffic and work: every layer reads its input and writes its output once, plus the weights
    alg_bytes, flops = 0, 0.0
    for l in shapes:
        px_in, px_out = N * l.H * l.W, N * l.Ho * l.Wo
        alg_bytes += 2 * (px_in * l.C + px_out * l.M)
        if l.kind == "gdws":
            G = int(workloads.configs.draw_g(l, gd.gdws_budget_gamma).sum())
            flops += 2.0 * px_out * G * (l.K * l.K + l.M)
            alg_bytes += 2 * G * (l.K * l.K + l.M)
        elif l.kind == "dense":
            flops += 2.0 * px_out * l.M * l.C * l.K * l.K
            alg_bytes += 2 * l.M * l.C * l.K * l.K
    achieved = alg_bytes / (dev_ms * 1e-3) / 1e9
    print(json.dumps({
        "metric": "GDWS network images/sec", "value": N / (wall_ms * 1e-3), "unit": "images/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": wall_ms, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": dtype, "data": "synthetic",
        "config": {"workload": f"{a.workload}-shaped network, batch {N}, {size}x{size} input, {len(shapes)} layers",
                   "layout": a.layout, "clock_ramp_ms": a.ramp_ms},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None, "kernel_ms": dev_ms,
                     "tflops": flops / (dev_ms * 1e-3) / 1e12, "algorithmic_bytes": alg_bytes}}))


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path needs no collective; batch shards would "
              "each run this same kernel) -- use --gpus 1", file=sys.stderr)
        sys.exit(2)

    if a.workload in ("vgg16", "resnet18", "resnet50"):
        if a.steps == 2000:
            a.steps, a.warmup = 20, 3
        return run_network(a)

    import numpy as np
    import torch
    import paper_2110_14871_amd as gd
    import workloads
    from gpu_util import empty_act, from_device, rel_l2, to_device

    torch.cuda.set_device(0)
    c2 = workloads.config2(N=256)
    N, C, H, W, M, K = c2["N"], c2["C"], c2["H"], c2["W"], c2["M"], c2["K"]
    dtype, b = "bf16", 2
    if a.workload == "config2":
        s, r = gd.gdws_singular_values(c2["Wt"])
        g = gd.gdws_mego(s, r, gd.gdws_budget_gamma(c2["rho"], C, K, M), g_init=np.ones(C, np.int32), cap=9)
    else:
        g = np.full(C, 9 if a.workload == "config2_g9" else 1, np.int32)
    G = int(g.sum())
    desc = gd.make_desc(C, M, K, 1, 1, dtype, a.layout)
    plan = gd.gdws_plan(desc, g, W=c2["Wt"])
    mode = {"auto": gd.MODE_AUTO, "fused": gd.MODE_FUSED, "unfused": gd.MODE_UNFUSED}[a.mode]
    ws = torch.empty(max(1, gd.gdws_workspace_bytes(plan, N, H, W, mode)), dtype=torch.uint8, device="cuda")

    x0, x_exact = to_device(c2["X"], dtype, a.layout)
    xs = [x0] + [x0.clone() for _ in range(max(1, a.rotate) - 1)]
    ys = [empty_act(N, M, H, W, dtype, a.layout) for _ in xs]
    stream = torch.cuda.current_stream()

    def step(i):
        k = i % len(xs)
        gd.gdws_forward(plan, xs[k], ys[k], N, H, W, workspace=ws, mode=mode, stream=stream)

    clock_ramp(step, a.ramp_ms)
    for i in range(a.warmup):
        step(i)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record(stream)
    for i in range(a.steps):
        step(i)
    ev1.record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    wall_ms = (t1 - t0) * 1e3 / a.steps
    dev_ms = ev0.elapsed_time(ev1) / a.steps

    # algorithmic traffic of one launch: read X once, write Y once, read the factors and the tables
    alg_bytes = b * (N * C * H * W + N * M * H * W) + b * G * (K * K + M) + 4 * (C + 1 + G)
    flops = 2.0 * N * H * W * G * (K * K + M)
    fused = gd.gdws_workspace_bytes(plan, N, H, W, mode) == 0
    achieved = alg_bytes / (dev_ms * 1e-3) / 1e9
    out = {
        "metric": "GDWS layer images/sec at batch 256",
        "value": N / (wall_ms * 1e-3),
        "unit": "images/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": wall_ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dtype, "data": "synthetic",
        "config": {"workload": f"{a.workload}: GDWS layer bf16 N=256 C=128 16x16 K=3 M=128 G={G}",
                   "layout": a.layout, "path": "fused" if fused else "unfused (gdw + pw through HBM)",
                   "rotating_buffers": len(xs), "clock_ramp_ms": a.ramp_ms},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": measured_traffic(a.workload, a.layout) if fused else None,
                     "kernel_ms": dev_ms, "tflops": flops / (dev_ms * 1e-3) / 1e12,
                     "algorithmic_bytes": alg_bytes},
    }

    if not a.no_cpu_baseline:
        import oracle
        dw, pw = gd.gdws_plan_factors(plan)
        threads = min(oracle.max_threads(), os.cpu_count() or 1, 16)
        t0 = time.perf_counter()
        ref = oracle.gdws_forward(x_exact, g, dw, pw, stride=1, pad=1, threads=threads)
        dt1 = time.perf_counter() - t0
        err = rel_l2(from_device(ys[0], dtype, a.layout), ref)
        reps = max(1, int(round(12.0 / dt1)))            # about 12 s of oracle work in all
        t0 = time.perf_counter()
        for _ in range(reps):
            oracle.gdws_forward(x_exact, g, dw, pw, stride=1, pad=1, threads=threads)
        dt = time.perf_counter() - t0
        n_o = reps * N
        out["cpu_baseline"] = {"value": n_o / dt, "unit": "images/s", "cores": threads, "kind": "oracle",
                               "sample": f"the full batch of {N} images, {reps} passes, fp64 direct loops with OpenMP, {dt:.2f} s",
                               "rel_l2_gpu_vs_oracle": err}
    if a.copy_calibration:
        src = torch.empty(a.copy_calibration << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
