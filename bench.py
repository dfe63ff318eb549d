#!/usr/bin/env python3
"""Throughput of the GDWS layer forward pass on one MI355X.

One step = one pass of the whole hot path (generalized depthwise + pointwise + epilogue)
over one batch of synthetic input already resident in HBM.  Default workload: the bf16
layer with C = M = 128 on 16 x 16 feature maps at batch 256, g from the greedy 25 % MAC
budget (G = 269).  Prints ONE JSON line with images/s, the dominant kernel's roofline
figures and the CPU oracle timed on the host cores.

Clocks: `value` and `ms_per_step` are host wall time around the timed steps (synchronised on
both sides); `roofline.kernel_ms` is device time between two events recorded on the launch
stream around the same steps.  The steps are issued through a launch graph recorded once
(one graph launch replays `--rotate` steps), unless --no-graph is given.
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
MFMA_PEAK_TFLOPS = 2500.0          # dense bf16 / fp16

NETWORKS = {"vgg16": ("f16", 256, 32), "resnet18": ("bf16", 512, 32), "resnet50": ("bf16", 128, 224),
            "wrn28_4": ("bf16", 256, 32)}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="timed steps (0 = the workload's default)")
    ap.add_argument("--warmup", type=int, default=-1, help="untimed steps before them (-1 = the workload's default)")
    ap.add_argument("--workload", default="config2",
                    choices=["config1", "config2", "config2_g9", "config2_g1", "config2_dense", "config2_backward"] + sorted(NETWORKS),
                    help="config2 (default, the headline layer), its two sub-runs, the standard convolution it "
                         "approximates (config2_dense: conv_dense_forward on the same shape), the layer's backward "
                         "pass (config2_backward: gdws_backward, all four gradients), the small fp32 layer at batch 1 "
                         "(config1: latency of one call), or a network-shaped "
                         "workload (VGG-16 fp16 batch 256, ResNet-18 bf16 batch 512, WRN-28-4 bf16 batch 256 at 32x32; "
                         "ResNet-50 bf16 batch 128 at 224x224)")
    ap.add_argument("--batch", type=int, default=0, help="network workloads: batch size (0 = the workload's own); "
                    "--batch 1 is the paper's frames-per-second protocol (5000 warm-up and 10000 timed forwards)")
    ap.add_argument("--layout", default="nhwc", choices=["nhwc", "nchw"])
    ap.add_argument("--mode", default="auto", choices=["auto", "fused", "unfused"])
    ap.add_argument("--no-graph", action="store_true", help="issue every step with its own launch calls")
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


class Stepper:
    """Issues steps 0, 1, 2, ... on `stream`: step i is fn(i % period).  With a graph, `period` consecutive steps are
    recorded once and replayed by one graph launch; what does not fill a whole period is issued eagerly."""

    def __init__(self, gd, fn, period, stream, use_graph):
        import torch
        self.gd, self.fn, self.period, self.stream = gd, fn, period, stream
        self.graph = None
        self.next = 0
        with torch.cuda.stream(stream):
            for k in range(period):          # every recorded call must have run once, eagerly
                fn(k)
            stream.synchronize()
            if use_graph:
                gd.gdws_capture_begin(stream)
                for k in range(period):
                    fn(k)
                self.graph = gd.gdws_capture_end(stream)

    def run(self, n):
        while n > 0:
            if self.graph is not None and self.next % self.period == 0 and n >= self.period:
                self.gd.gdws_graph_launch(self.graph, self.stream)
                n -= self.period
                self.next += self.period
            else:
                self.fn(self.next % self.period)
                n -= 1
                self.next += 1


def clock_ramp(stepper, ramp_ms):
    """Keep the GPU busy with steps for about ramp_ms so that its clocks are at their steady state."""
    t0 = time.perf_counter()
    while (time.perf_counter() - t0) * 1e3 < ramp_ms:
        stepper.run(4 * stepper.period)
        stepper.stream.synchronize()
    stepper.run((-stepper.next) % stepper.period)      # back to a period boundary


def timed(stepper, steps, warmup):
    """(wall ms per step, device ms per step) of `steps` steps after `warmup` untimed ones."""
    import torch
    stream = stepper.stream
    stepper.run(warmup)
    stepper.run((-stepper.next) % stepper.period)
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record(stream)
    stepper.run(steps)
    ev1.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    return wall_ms, ev0.elapsed_time(ev1) / steps


def copy_rate_gbs(stream):
    """Read + write rate of a plain 256 MiB device-to-device copy on this chip: the practical HBM ceiling."""
    import torch
    with torch.cuda.stream(stream):
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record(stream)
        for _ in range(10):
            dst.copy_(src)
        ev1.record(stream)
        stream.synchronize()
    return 2 * src.numel() * 10 / (ev0.elapsed_time(ev1) * 1e-3) / 1e9


def profile_traffic(workload, layout):
    """HBM bytes per launch from the committed counter summary of this workload (rocprofv3 --pmc FETCH_SIZE and
    WRITE_SIZE, separate runs), with the file it comes from; (None, None) if there is none."""
    name = f"fused_{workload}_{layout}_hbm_traffic.txt"
    try:
        for line in open(os.path.join(ROOT, "profiles", name)):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1]), "profiles/" + name
    except OSError:
        pass
    return None, None


def oracle_threads():
    import oracle
    return min(oracle.max_threads(), os.cpu_count() or 1, 16)


def run_network(a):
    """Whole-network forward of a VGG-16 / ResNet-18 / ResNet-50 / WRN-28-4 shaped stack (every 3x3 convolution a GDWS layer)."""
    import numpy as np
    import torch
    import paper_2110_14871_amd as gd
    import workloads
    from gpu_util import empty_act, from_device, rel_l2, to_device
    from net_util import build_network

    torch.cuda.set_device(0)
    dtype, batch, size = NETWORKS[a.workload]
    maker = {"vgg16": workloads.vgg16_shape, "resnet18": workloads.resnet18_shape, "resnet50": workloads.resnet50_shape,
             "wrn28_4": workloads.wrn28_4_shape}[a.workload]
    N = a.batch or batch
    protocol = "batch-1 frames per second (5000 warm-up, 10000 timed forwards)" if N == 1 else "batched throughput"
    steps = a.steps or (10000 if N == 1 else 20)
    warmup = a.warmup if a.warmup >= 0 else (5000 if N == 1 else 3)
    shapes = maker(size, size)
    net, params = build_network(shapes, dtype, a.layout)
    x, x_exact = to_device(workloads.rng.normal(900, (N, 3, size, size)), dtype, a.layout)
    last = shapes[-1]
    y = empty_act(N, last.M, last.Ho, last.Wo, dtype, a.layout)
    ws = torch.empty(max(1, gd.gdws_net_workspace_bytes(net, N, size, size)), dtype=torch.uint8, device="cuda")
    stream = torch.cuda.Stream()
    stepper = Stepper(gd, lambda k: gd.gdws_network_forward(net, x, y, N, size, size, workspace=ws, stream=stream), 1,
                      stream, not a.no_graph)
    clock_ramp(stepper, a.ramp_ms)
    wall_ms, dev_ms = timed(stepper, steps, warmup)
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
    out = {
        "metric": "GDWS network images/sec", "value": N / (wall_ms * 1e-3), "unit": "images/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": wall_ms, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": dtype, "data": "synthetic",
        "config": {"workload": f"{a.workload}-shaped network, batch {N}, {size}x{size} input, {len(shapes)} layers",
                   "layout": a.layout, "protocol": protocol, "launch": "eager" if a.no_graph else "launch graph",
                   "clock_ramp_ms": a.ramp_ms, "value_clock": "host wall time", "kernel_ms_clock": "device events"},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": None, "kernel_ms": dev_ms,
                     "tflops": flops / (dev_ms * 1e-3) / 1e12, "algorithmic_bytes": alg_bytes,
                     "measured_copy_rate_gbs": copy_rate_gbs(stream)}}
    if not a.no_cpu_baseline:
        import oracle
        pick = sorted({0, N - 1})
        threads = oracle_threads()
        t0 = time.perf_counter()
        ref = oracle.network_forward(shapes, params, x_exact[pick], store=dtype, round_intermediate=dtype, threads=threads)
        dt = time.perf_counter() - t0
        yh = from_device(y, dtype, a.layout)[pick]
        out["cpu_baseline"] = {"value": len(pick) / dt, "unit": "images/s", "cores": threads, "kind": "oracle",
                               "sample": f"images {pick} of the batch, one pass, fp64 direct loops with OpenMP, {dt:.2f} s",
                               "rel_l2_gpu_vs_oracle": rel_l2(yh, ref)}
    print(json.dumps(out))

FP32_VECTOR_PEAK_TFLOPS = 157.3


def run_backward(a):
    """gdws_backward on config 2 (dx, dD, dPw, dbias): general vector-ALU kernels, priced against the fp32 vector peak."""
    import numpy as np
    import torch
    import paper_2110_14871_amd as gd
    import workloads
    from gpu_util import empty_act, from_device, rel_l2, to_device

    torch.cuda.set_device(0)
    steps = a.steps or 200
    warmup = a.warmup if a.warmup >= 0 else 20
    c2 = workloads.config2(N=256)
    N, C, H, W, M, K = c2["N"], c2["C"], c2["H"], c2["W"], c2["M"], c2["K"]
    dtype = "bf16"
    s, r = gd.gdws_singular_values(c2["Wt"])
    g = gd.gdws_mego(s, r, gd.gdws_budget_gamma(c2["rho"], C, K, M), g_init=np.ones(C, np.int32), cap=9)
    G = int(g.sum())
    plan = gd.gdws_plan(gd.make_desc(C, M, K, 1, 1, dtype, a.layout), g, W=c2["Wt"])
    stream = torch.cuda.Stream()
    xd, x_exact = to_device(c2["X"], dtype, a.layout)
    dyd, dy_exact = to_device(workloads.rng.normal(13, (N, M, H, W)), dtype, a.layout)
    dx = empty_act(N, C, H, W, dtype, a.layout)
    d_dw = torch.empty(G, K, K, dtype=torch.float32, device="cuda")
    d_pw = torch.empty(M, G, dtype=torch.float32, device="cuda")
    d_b = torch.empty(M, dtype=torch.float32, device="cuda")
    ws = torch.empty(gd.gdws_backward_workspace_bytes(plan, N, H, W), dtype=torch.uint8, device="cuda")

    def step(k):
        gd.gdws_backward(plan, xd, dyd, N, H, W, dx=dx, d_dw=d_dw, d_pw=d_pw, d_bias=d_b, workspace=ws, stream=stream)

    stepper = Stepper(gd, step, 1, stream, not a.no_graph)
    clock_ramp(stepper, a.ramp_ms)
    wall_ms, dev_ms = timed(stepper, steps, warmup)
    # the intermediate and its gradient (K^2 + M products per element each), dPw (M), dD and dx (K^2 each)
    flops = 2.0 * N * H * W * G * (3 * K * K + 2 * M)
    tflops = flops / (dev_ms * 1e-3) / 1e12
    out = {
        "metric": "GDWS layer backward passes (images/sec) at batch 256", "value": N / (wall_ms * 1e-3), "unit": "images/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": wall_ms, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"config2_backward: gdws_backward (dx, dD, dPw, dbias) bf16 N=256 C=128 16x16 K=3 M=128 G={G}",
                   "layout": a.layout, "path": "general vector-ALU kernels, intermediate and its gradient in fp32 through HBM",
                   "launch": "eager" if a.no_graph else "launch graph of 1 step"},
        "roofline": {"bound": "alu", "achieved": tflops, "peak": FP32_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": tflops / FP32_VECTOR_PEAK_TFLOPS, "traffic": None, "kernel_ms": dev_ms, "flops": flops},
    }
    if not a.no_cpu_baseline:
        import oracle
        dwq, pwq = gd.gdws_plan_factors(plan)
        n1 = 4
        t0 = time.perf_counter()
        ref = oracle.gdws_backward(x_exact[:n1], g, dwq, pwq, dy_exact[:n1], 1, 1, threads=oracle_threads())
        dt = time.perf_counter() - t0
        # dx of an image depends on that image alone: checked on the sample
        err = rel_l2(from_device(dx, dtype, a.layout)[:n1], ref[0])
        out["cpu_baseline"] = {"value": n1 / dt, "unit": "images/s", "cores": 1, "kind": "oracle",
                               "sample": f"the first {n1} images, one pass of the numpy loops over filters and taps, {dt:.2f} s",
                               "rel_l2_dx_gpu_vs_oracle": err}
    print(json.dumps(out))

def run_config1(a):
    """Configuration 1 (fp32, N = 1, 16 -> 32 channels, 32 x 32, NCHW): the latency of one call, which at this size is a
    launch latency; priced against the fp32 vector peak only to give the line its roofline object."""
    import torch
    import paper_2110_14871_amd as gd
    import workloads
    from gpu_util import empty_act, from_device, rel_l2, to_device

    torch.cuda.set_device(0)
    steps = a.steps or 2000
    warmup = a.warmup if a.warmup >= 0 else 200
    c = workloads.config1()
    N, C, H, W, M, K = c["N"], c["C"], c["H"], c["W"], c["M"], c["K"]
    mode = {"auto": gd.MODE_AUTO, "fused": gd.MODE_FUSED, "unfused": gd.MODE_UNFUSED}[a.mode]
    plan = gd.gdws_plan(gd.make_desc(C, M, K, 1, 1, "f32", "nchw"), c["g"], W=c["Wt"])
    G = int(c["g"].sum())
    stream = torch.cuda.Stream()
    xd, x_exact = to_device(c["X"], "f32", "nchw")
    y = empty_act(N, M, H, W, "f32", "nchw")
    ws = torch.empty(max(1, gd.gdws_workspace_bytes(plan, N, H, W, mode)), dtype=torch.uint8, device="cuda")

    def step(k):
        gd.gdws_forward(plan, xd, y, N, H, W, workspace=ws, mode=mode, stream=stream)

    stepper = Stepper(gd, step, 1, stream, False)     # call by call: the figure is the latency of a call
    clock_ramp(stepper, a.ramp_ms)
    wall_ms, dev_ms = timed(stepper, steps, warmup)
    flops = 2.0 * N * H * W * G * (K * K + M)
    tflops = flops / (dev_ms * 1e-3) / 1e12
    fused = gd.gdws_workspace_bytes(plan, N, H, W, mode) == 0
    out = {
        "metric": "GDWS layer images/sec at batch 1 (configuration 1, latency)", "value": N / (wall_ms * 1e-3),
        "unit": "images/s", "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": wall_ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"config1: GDWS layer fp32 N=1 C=16 32x32 K=3 M=32 G={G}", "layout": "nchw",
                   "path": "fused (vector-ALU kernel)" if fused else "unfused (direct depthwise + fp32 MFMA pointwise)",
                   "launch": "eager, one call per step"},
        "roofline": {"bound": "alu", "achieved": tflops, "peak": FP32_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": tflops / FP32_VECTOR_PEAK_TFLOPS, "traffic": None, "kernel_ms": dev_ms, "flops": flops},
    }
    if not a.no_cpu_baseline:
        import oracle
        dw, pw = gd.gdws_plan_factors(plan)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        reps = 200
        for _ in range(reps):
            ref = oracle.gdws_forward(x_exact, c["g"], dw, pw, stride=1, pad=1, threads=1)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": reps / dt, "unit": "images/s", "cores": 1, "kind": "oracle",
                               "sample": f"the one image, {reps} passes of the fp64 loops on one thread, {dt:.2f} s",
                               "rel_l2_gpu_vs_oracle": rel_l2(from_device(y, "f32", "nchw"), ref)}
    print(json.dumps(out))


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path needs no collective; batch shards would "
              "each run this same kernel) -- use --gpus 1", file=sys.stderr)
        sys.exit(2)
    if a.workload in NETWORKS:
        return run_network(a)
    if a.workload == "config2_backward":
        return run_backward(a)
    if a.workload == "config1":
        return run_config1(a)

    import numpy as np
    import torch
    import paper_2110_14871_amd as gd
    import workloads
    from gpu_util import empty_act, from_device, quantise, rel_l2, to_device

    torch.cuda.set_device(0)
    steps = a.steps or 2000
    warmup = a.warmup if a.warmup >= 0 else 200
    c2 = workloads.config2(N=256)
    N, C, H, W, M, K = c2["N"], c2["C"], c2["H"], c2["W"], c2["M"], c2["K"]
    dtype, b = "bf16", 2
    dense = a.workload == "config2_dense"
    stream = torch.cuda.Stream()
    x0, x_exact = to_device(c2["X"], dtype, a.layout)
    xs = [x0] + [x0.clone() for _ in range(max(1, a.rotate) - 1)]
    ys = [empty_act(N, M, H, W, dtype, a.layout) for _ in xs]
    if dense:
        desc = gd.make_desc(C, M, K, 1, 1, dtype, a.layout)
        wd, w_exact = to_device(c2["Wt"], dtype, "nchw")
        ws = torch.empty(max(1, gd.conv_dense_workspace_bytes(desc)), dtype=torch.uint8, device="cuda")
        G, fused = C * K * K, True

        def step(k):
            gd.conv_dense_forward(desc, wd, xs[k], ys[k], N, H, W, workspace=ws, stream=stream)
        # eq. 2: the standard convolution's own work and traffic
        alg_bytes = b * (N * C * H * W + N * M * H * W) + b * M * C * K * K
        flops = 2.0 * N * H * W * M * C * K * K
    else:
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
        fused = gd.gdws_workspace_bytes(plan, N, H, W, mode) == 0

        def step(k):
            gd.gdws_forward(plan, xs[k], ys[k], N, H, W, workspace=ws, mode=mode, stream=stream)
        # algorithmic traffic of one launch: read X once, write Y once, read the factors and the tables
        alg_bytes = b * (N * C * H * W + N * M * H * W) + b * G * (K * K + M) + 4 * (C + 1 + G)
        flops = 2.0 * N * H * W * G * (K * K + M)

    stepper = Stepper(gd, step, len(xs), stream, not a.no_graph)
    clock_ramp(stepper, a.ramp_ms)
    wall_ms, dev_ms = timed(stepper, steps, warmup)

    # the same step on one buffer pair only (33 MB of input and output, inside the 256 MB last-level cache): reported
    # beside the figure of the rotating buffers, which is the one that counts
    # (issued call by call: the host issues a launch faster than the kernel runs, a graph of one step it does not)
    one = Stepper(gd, lambda k: step(0), 1, stream, False)
    _, cached_ms = timed(one, min(steps, 500), min(warmup, 50))

    achieved = alg_bytes / (dev_ms * 1e-3) / 1e9
    tflops = flops / (dev_ms * 1e-3) / 1e12
    # which roofline binds: the arithmetic intensity against the ridge of the two peaks (312 FLOP per byte)
    mfma_bound = flops / alg_bytes > MFMA_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9)
    traffic, traffic_src = profile_traffic(a.workload, a.layout) if fused and not dense else (None, None)
    roof = {"bound": "mfma", "achieved": tflops, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": tflops / MFMA_PEAK_TFLOPS} if mfma_bound else \
           {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS}
    roof.update({"traffic": traffic, "traffic_source": traffic_src, "kernel_ms": dev_ms, "tflops": tflops,
                 "gbs_algorithmic": achieved, "algorithmic_bytes": alg_bytes, "flops": flops,
                 "kernel_ms_one_buffer_pair": cached_ms, "measured_copy_rate_gbs": copy_rate_gbs(stream)})
    what = "standard convolution (conv_dense_forward)" if dense else "GDWS layer"
    out = {
        "metric": "GDWS layer images/sec at batch 256",
        "value": N / (wall_ms * 1e-3),
        "unit": "images/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": wall_ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dtype, "data": "synthetic",
        "config": {"workload": f"{a.workload}: {what} bf16 N=256 C=128 16x16 K=3 M=128 G={G}",
                   "layout": a.layout, "path": "fused" if fused else "unfused (gdw + pw through HBM)",
                   "rotating_buffers": len(xs), "launch": "eager" if a.no_graph else f"launch graph of {len(xs)} steps",
                   "clock_ramp_ms": a.ramp_ms, "value_clock": "host wall time", "kernel_ms_clock": "device events"},
        "roofline": roof,
    }

    if not a.no_cpu_baseline:
        import oracle
        threads = oracle_threads()
        if dense:
            run_oracle = lambda xe, th: oracle.conv_dense(xe, w_exact, stride=1, pad=1, threads=th)
        else:
            dw, pw = gd.gdws_plan_factors(plan)
            run_oracle = lambda xe, th: oracle.gdws_forward(xe, g, dw, pw, stride=1, pad=1, threads=th)
        t0 = time.perf_counter()
        ref = run_oracle(x_exact, threads)
        dt1 = time.perf_counter() - t0
        err = rel_l2(from_device(ys[0], dtype, a.layout), ref)
        reps = max(1, int(round(10.0 / dt1)))            # about 10 s of oracle work in all
        t0 = time.perf_counter()
        for _ in range(reps):
            run_oracle(x_exact, threads)
        dt = time.perf_counter() - t0
        n1 = max(1, min(N, int(round(N * 3.0 / (dt1 * threads)))))     # about 3 s on one thread
        t0 = time.perf_counter()
        run_oracle(x_exact[:n1], 1)
        d1 = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": reps * N / dt, "unit": "images/s", "cores": threads, "kind": "oracle",
                               "sample": f"the full batch of {N} images, {reps} passes, fp64 direct loops with OpenMP, {dt:.2f} s",
                               "single_thread": {"value": n1 / d1, "unit": "images/s", "cores": 1,
                                                 "sample": f"the first {n1} images, one pass, {d1:.2f} s"},
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
