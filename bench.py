#!/usr/bin/env python3
"""Benchmark of the conv + loss hot path on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input:
forward, data gradient and filter gradient of all 63 convolution layers of the
DeepLabv3+-style network at N=2, 1152x768x16 (fp16 storage, fp32 accumulate),
plus the weighted pixel cross-entropy on the full-resolution 3-class logits.
Inputs are resident in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu-baseline] [--table]
    python bench.py --config N        (N = 1..4: per-layer table of that configuration, oracle timed beside it)
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_PEAK_TFLOPS = 2500.0          # MI355X dense fp16/bf16 matrix peak
HBM_PEAK_GBS = 8000.0
# The dominant kernel: the 3x3 halo-tile implicit-GEMM kernel
# (igemm_halo3x3_kernel<F16, 4>), which the two full-resolution decoder 3x3
# layers (87 % of all FLOPs) run for their forward and data-gradient passes.
# Timed here on the three calls per step that consist of that kernel alone
# (plus a microsecond-scale filter re-layout): both forward passes and the
# 256->256 data gradient.  (The 304-channel data gradient adds a launch of the
# 64-channel variant for its last 48 columns.)
DOMINANT_CALLS = (("dec.3x3.304-256", "fwd"), ("dec.3x3.256-256", "fwd"), ("dec.3x3.256-256", "dgrad"))


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--dtype", default="f16", choices=("f16", "bf16"),
                    help="storage type of the tensors (the headline configuration is f16; accumulation is fp32 either way)")
    ap.add_argument("--activations", default="abs", choices=("abs", "relu"),
                    help="distribution of the layers' input activations: |N(0,1)| (dense, the headline recipe) or "
                         "max(N(0,1), 0) (half of them exactly zero, as behind a ReLU at initialisation); the chip is "
                         "power-limited, so the time depends on the operand values")
    ap.add_argument("--fused-logits", action="store_true",
                    help="run the logits layer and the loss as the one fused call (logits_ce_fused_fwd_bwd) instead of "
                         "forward + loss + data gradient + filter gradient; not the headline configuration")
    ap.add_argument("--table", action="store_true", help="per-layer timing table on stderr")
    ap.add_argument("--tiramisu-table", action="store_true",
                    help="per-layer times at the layer shapes of the paper's second network (modified Tiramisu); "
                         "not part of the headline step")
    ap.add_argument("--deconv-table", action="store_true",
                    help="instead of the step: time the decoder's transposed-convolution layers (forward, data "
                         "gradient, filter gradient each) and print a table; no JSON line")
    ap.add_argument("--streams", type=int, default=3, choices=(1, 2, 3, 4),
                    help="2-4: filter gradients of the small layers run on 1-3 more HIP streams beside the "
                         "data-gradient chain")
    ap.add_argument("--traffic-file", default=os.path.join(ROOT, "profiles", "igemm_halo3x3_config5_traffic.txt"))
    ap.add_argument("--config", type=int, default=5, choices=(1, 2, 3, 4, 5),
                    help="5 (default): the headline step.  1-4: instead of the step, time every layer and pass of that "
                         "configuration in its own dtype and the fp64 oracle on the same layer in full; prints a table "
                         "and one JSON line per configuration")
    ap.add_argument("--no-microbench", action="store_true",
                    help="skip the register-resident MFMA loop and the plain streaming kernels that are run beside the "
                         "step (the machine's ceilings on this box, printed as context in the same line)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 1 GiB device-to-device copy, as the known-size reference for HBM byte counters")
    return ap.parse_args()


def device_inputs(layer, dtype, seed, torch, activations="abs"):
    """Synthetic tensors of the layer's shapes, generated on the device:
    |N(0,1)| activations (post-ReLU-like), He-scaled filters, N(0,1) upstream
    gradients; the stem gets smooth normalised fields from the host generator."""
    from paper_1810_01993_amd import synth
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    xs = (layer.N, layer.H, layer.W, layer.C)
    if layer.name == "stem7x7":
        _, bits = synth.quantize(synth.smooth_fields(seed, *xs), "bf16" if dtype == torch.bfloat16 else "f16")
        x = torch.from_numpy(bits.view(np.int16)).view(dtype).cuda()
    else:
        x = torch.randn(xs, generator=g, device="cuda", dtype=torch.float32)
        x = (x.abs_() if activations == "abs" else x.clamp_(min=0)).to(dtype)
    sigma = float(np.sqrt(2.0 / (layer.R * layer.S * layer.C)))
    w = (torch.randn((layer.K, layer.R, layer.S, layer.C), generator=g, device="cuda") * sigma).to(dtype)
    dy = torch.randn((layer.N, layer.P, layer.Q, layer.K), generator=g, device="cuda", dtype=torch.float32).to(dtype)
    return x, w, dy


class LayerState:
    """Device buffers of one occurrence of one layer shape."""

    def __init__(self, api, layer, seed, torch, dtype_name="f16", activations="abs"):
        self.layer = layer
        self.desc = api.desc_from_layer(layer, dtype_name)
        self.x, self.w, self.dy = device_inputs(layer, torch.bfloat16 if dtype_name == "bf16" else torch.float16, seed, torch,
                                                 activations)
        self.y = torch.empty_like(self.dy)
        self.dx = torch.empty_like(self.x)
        self.dw = torch.empty_like(self.w)
        nb = max(api.dl_conv_workspace_bytes(self.desc, p) for p in (0, 1))
        self.ws = torch.empty(max(nb, 16), dtype=torch.uint8, device="cuda")
        # the filter gradient may run beside the data gradient: its own workspace
        self.ws_w = torch.empty(max(api.dl_conv_workspace_bytes(self.desc, 2), 16), dtype=torch.uint8, device="cuda")


def cpu_baseline():
    """The fp64 oracle, as it stands, on a bounded sample of the same workload:
    forward + data gradient + filter gradient of a 128-row slab of one image of
    the 3x3 256->256 full-resolution decoder layer."""
    import oracle
    rows = 128
    s = oracle.ConvShape(1, rows, 1152, 256, 256, 3, 3, 1, 1, 1)
    g = np.random.default_rng(0)
    x = np.abs(g.standard_normal((1, rows, 1152, 256)))
    w = g.standard_normal((256, 3, 3, 256)) * np.sqrt(2.0 / 2304)
    dy = g.standard_normal((1, rows, 1152, 256))
    t0 = time.perf_counter()
    oracle.conv_fwd(s, x, w)
    oracle.conv_bwd_data(s, dy, w)
    oracle.conv_bwd_filter(s, x, dy)
    dt = time.perf_counter() - t0
    flops = 3 * 2 * rows * 1152 * 256 * 256 * 9
    cores = len(os.sched_getaffinity(0))
    omp = os.environ.get("OMP_NUM_THREADS")
    if omp:
        cores = min(cores, int(omp))
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "sample": f"fwd+dgrad+wgrad of a {rows}x1152 slab (1 image) of dec.3x3.256-256, fp64, {dt:.1f} s"}


def loss_hbm_resident(api, torch, mult=64, probes=True):
    """The loss kernel on mult x the step's pixel count (1.47 GB of traffic at 64x): the step's own 23 MB
    fit the last-level caches and take two kernel launches, so bandwidth is judged on this size."""
    n = 2 * 768 * 1152 * mult
    logits = torch.randn((n, 3), device="cuda", dtype=torch.float16)
    labels = (torch.rand(n, device="cuda") < 0.02).to(torch.uint8)
    cw = torch.tensor([1.0, 7.67, 31.6], dtype=torch.float32, device="cuda")
    dl = torch.empty_like(logits)
    loss = torch.empty(1, dtype=torch.float32, device="cuda")
    ws = torch.empty(max(api.dl_ce_workspace_bytes(n), 16), dtype=torch.uint8, device="cuda")
    run = lambda: api.weighted_pixel_ce_fwd_bwd(logits, labels, cw, 1.0 / n, loss=loss, dlogits=dl, workspace=ws)
    run()
    torch.cuda.synchronize()
    ts = []
    for _ in range(5):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(10):
            run()
        b.record()
        torch.cuda.synchronize()
        ts.append(a.elapsed_time(b) / 10)
    ms = float(np.median(ts))
    gbs = 13 * n / (ms * 1e-3) / 1e9
    out = {"n_pixels": n, "ms": ms, "gbs": gbs, "frac_of_hbm_peak": gbs / HBM_PEAK_GBS}
    if probes:
        # the same buffers through kernels that only move the bytes (no LDS hand-over, no arithmetic)
        sink = torch.zeros(4, dtype=torch.int32, device="cuda")
        nbytes = 6 * n
        for mode, name, moved in ((0, "read", nbytes), (1, "copy", 2 * nbytes), (2, "write", nbytes),
                                  (3, "loss_traffic_mix", 13 * n)):
            runp = lambda: api.probe_stream(mode, logits, labels, dl, nbytes, sink)
            runp()
            torch.cuda.synchronize()
            ts = []
            for _ in range(3):
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                for _ in range(5):
                    runp()
                b.record()
                torch.cuda.synchronize()
                ts.append(a.elapsed_time(b) / 5)
            out[f"probe_{name}_gbs"] = moved / (float(np.median(ts)) * 1e-3) / 1e9
    return out


def mfma_microbench(api, torch, iters=100000):
    """Register-resident MFMA loops (no memory traffic) in this process, on this machine: what the matrix
    units sustain with constant operands and with operands distributed like the benchmark's (the chip
    is power-limited: the shader clock drops with the operands' switching activity).  Context for the
    roofline fractions, which keep the published 2.5 PFLOP/s."""
    sink = torch.empty(api.PROBE_SINK_FLOATS, dtype=torch.float32, device="cuda")
    clocks = torch.zeros(2, dtype=torch.int64, device="cuda")
    out = {}
    for shape, sname in ((1, "16x16x32_f16"), (0, "32x32x16_f16")):
        for operands, oname in ((0, "constant_operands"), (1, "bench_like_operands")):
            api.probe_mfma(shape, operands, iters // 10, sink, clocks)
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            flop = api.probe_mfma(shape, operands, iters, sink, clocks)
            b.record()
            torch.cuda.synchronize()
            ms = a.elapsed_time(b)
            wall, cyc = (int(v) for v in clocks.cpu())
            out[f"{sname}.{oname}"] = {"tflops": flop / (ms * 1e-3) / 1e12, "ms": ms,
                                       "shader_clock_mhz": cyc / (wall / 100.0) if wall else None}
    return out


KERNEL_SOURCES = ("igemm_halo3x3.hip", "device_common.h")       # what the dominant kernel is compiled from


def kernel_source_hash():
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_1810_01993_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def read_traffic(path):
    """HBM bytes per launch of the dominant kernel, from the committed rocprofv3 counter summary
    (its 'bytes_per_launch = <number>' line), and where that number comes from: the file, and whether
    the kernel source it was measured on ('kernel_source_sha = <hash>') is the one in the tree now.
    A stale figure is still printed, flagged."""
    traffic, sha = None, None
    try:
        with open(path) as f:
            for line in f:
                t = line.strip()
                if t.startswith("bytes_per_launch"):
                    traffic = float(t.split("=")[1].split()[0])
                elif t.startswith("kernel_source_sha"):
                    sha = t.split("=")[1].split()[0]
    except OSError:
        pass
    now = kernel_source_hash()
    src = {"file": os.path.relpath(path, ROOT), "measured_on_kernel_source_sha": sha, "current_kernel_source_sha": now,
           "current": sha == now}
    return traffic, src


def deconv_table(args):
    """Transposed-convolution layers of the decoder's up-sampling path (not part of the headline
    step): HIP-event time of each entry point, median over --steps calls after --warmup."""
    import torch
    from paper_1810_01993_amd import api, layers

    torch.cuda.set_device(0)
    print(f"{'layer (underlying convolution)':34s} {'entry point':28s} {'ms':>9s} {'TFLOP/s':>9s} {'%MFMA':>6s}")
    for li, layer in enumerate(layers.deconv_layers(2, 768, 1152)):
        desc = api.desc_from_layer(layer, "f16")
        g = torch.Generator(device="cuda")
        g.manual_seed(1000 + li)
        x = torch.randn((layer.N, layer.P, layer.Q, layer.K), generator=g, device="cuda").abs_().half()
        sigma = float(np.sqrt(2.0 / (layer.R * layer.S * layer.K)))
        w = (torch.randn((layer.K, layer.R, layer.S, layer.C), generator=g, device="cuda") * sigma).half()
        dy = torch.randn((layer.N, layer.H, layer.W, layer.C), generator=g, device="cuda").half()
        y, dx, dw = torch.empty_like(dy), torch.empty_like(x), torch.empty_like(w)
        ws = torch.empty(max(16, max(api.dl_conv_workspace_bytes(desc, p) for p in range(3))), dtype=torch.uint8,
                         device="cuda")
        calls = {"conv2d_transpose_fwd": lambda: api.conv2d_transpose_fwd(desc, x, w, y=y, workspace=ws),
                 "conv2d_transpose_bwd_data": lambda: api.conv2d_transpose_bwd_data(desc, dy, w, dx=dx, workspace=ws),
                 "conv2d_transpose_bwd_filter": lambda: api.conv2d_transpose_bwd_filter(desc, x, dy, dw=dw, workspace=ws)}
        for name, fn in calls.items():
            for _ in range(args.warmup):
                fn()
            ts = []
            for _ in range(args.steps):
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                fn()
                b.record()
                torch.cuda.synchronize()
                ts.append(a.elapsed_time(b))
            ms = float(np.median(ts))
            tf = layer.flops() / (ms * 1e-3) / 1e12
            print(f"{layer.name:34s} {name:28s} {ms:9.4f} {tf:9.1f} {100 * tf / MFMA_PEAK_TFLOPS:6.1f}", flush=True)


def tiramisu_table(args):
    """Every layer shape of the paper's second network (layers.tiramisu_layers: growth 32, 5x5), N=2, fp16:
    HIP-event time of each pass, median over --steps calls after --warmup; the three passes of all layers
    are summed at the end (one stream, no overlap: an upper bound of the convolution time of a step)."""
    import torch
    from paper_1810_01993_amd import api, layers

    torch.cuda.set_device(0)
    convs, deconvs = layers.tiramisu_layers(2, 768, 1152)
    print(f"{'layer':34s} {'pass':8s} {'ms':>9s} {'TFLOP/s':>9s} {'%MFMA':>6s} {'GB/s(min)':>10s} {'%HBM':>6s}")
    total_ms, total_flop = 0.0, 0.0
    for li, layer in enumerate(convs + deconvs):
        transposed = li >= len(convs)
        desc = api.desc_from_layer(layer, "f16")
        g = torch.Generator(device="cuda")
        g.manual_seed(2000 + li)
        sigma = float(np.sqrt(2.0 / (layer.R * layer.S * (layer.K if transposed else layer.C))))
        w = (torch.randn((layer.K, layer.R, layer.S, layer.C), generator=g, device="cuda") * sigma).half()
        big = torch.randn((layer.N, layer.H, layer.W, layer.C), generator=g, device="cuda")       # the conv's input side
        small = torch.randn((layer.N, layer.P, layer.Q, layer.K), generator=g, device="cuda")     # the conv's output side
        if transposed:
            x, dy = small.abs_().half(), big.half()                # layer input [N,P,Q,K], output gradient [N,H,W,C]
            y, dx = torch.empty_like(dy), torch.empty_like(x)
        else:
            x, dy = big.abs_().half(), small.half()
            y, dx = torch.empty_like(dy), torch.empty_like(x)
        del big, small
        dw = torch.empty_like(w)
        ws = torch.empty(max(16, max(api.dl_conv_workspace_bytes(desc, p) for p in range(3))), dtype=torch.uint8,
                         device="cuda")
        if transposed:
            calls = {"fwd": lambda: api.conv2d_transpose_fwd(desc, x, w, y=y, workspace=ws),
                     "dgrad": lambda: api.conv2d_transpose_bwd_data(desc, dy, w, dx=dx, workspace=ws),
                     "wgrad": lambda: api.conv2d_transpose_bwd_filter(desc, x, dy, dw=dw, workspace=ws)}
        else:
            calls = {"fwd": lambda: api.conv2d_fwd(desc, x, w, y=y, workspace=ws),
                     "dgrad": lambda: api.conv2d_bwd_data(desc, dy, w, dx=dx, workspace=ws),
                     "wgrad": lambda: api.conv2d_bwd_filter(desc, x, dy, dw=dw, workspace=ws)}
        min_bytes = 2.0 * (x.numel() + w.numel() + dy.numel())
        for name, fn in calls.items():
            for _ in range(args.warmup):
                fn()
            ts = []
            for _ in range(args.steps):
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                fn()
                b.record()
                torch.cuda.synchronize()
                ts.append(a.elapsed_time(b))
            ms = float(np.median(ts))
            tf = layer.flops() / (ms * 1e-3) / 1e12
            gbs = min_bytes / (ms * 1e-3) / 1e9
            total_ms += ms
            total_flop += layer.flops()
            print(f"{layer.name:34s} {name:8s} {ms:9.4f} {tf:9.1f} {100 * tf / MFMA_PEAK_TFLOPS:6.1f} {gbs:10.0f} "
                  f"{100 * gbs / HBM_PEAK_GBS:6.1f}", flush=True)
        del x, dy, y, dx, w, dw, ws
        torch.cuda.empty_cache()
    print(f"sum of the three passes of all {len(convs) + len(deconvs)} layers: {total_ms:.3f} ms, "
          f"{total_flop / 1e12:.2f} TFLOP, {total_flop / (total_ms * 1e-3) / 1e12:.1f} TFLOP/s "
          f"({2 / (total_ms * 1e-3):.1f} samples/s for the convolutions alone)")


def config_table(args):
    """Configurations 1-4 (the parity cases that are not the headline): every layer and pass in the
    configuration's own dtype, median HIP-event time per call over groups of back-to-back calls on
    rotating buffer sets (so that the 1x1 layers do not re-read cache-resident tensors), and beside it the fp64 oracle
    on the very same layer in full, on the host cores (a baseline, not a target)."""
    import torch
    import oracle
    from paper_1810_01993_amd import api, layers, synth

    torch.cuda.set_device(0)
    dtype, table = {1: layers.config1, 2: layers.config2, 3: layers.config3, 4: layers.config4}[args.config]()
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float16
    cores = len(os.sched_getaffinity(0))
    if os.environ.get("OMP_NUM_THREADS"):
        cores = min(cores, int(os.environ["OMP_NUM_THREADS"]))
    print(f"# config {args.config}, {dtype}, fp32 accumulate; oracle: fp64 on {cores} host cores", flush=True)
    print(f"{'layer':24s} {'pass':6s} {'ms':>9s} {'p16':>8s} {'p84':>8s} {'TFLOP/s':>9s} {'%MFMA':>6s} {'GB/s(min)':>10s} {'%HBM':>6s} "
          f"{'oracle s':>9s} {'oracle GFLOP/s':>14s}  kernels", flush=True)
    tot_ms, tot_flop, tot_orc = 0.0, 0.0, 0.0
    for li, layer in enumerate(table):
        seed = synth.seed_for(args.config, 10 * li)
        kind = "fields" if layer.R == 7 else "half_normal"
        xs = (layer.N, layer.H, layer.W, layer.C)
        x64 = synth.smooth_fields(seed, *xs) if kind == "fields" else synth.half_normal(seed, xs)
        w64 = synth.he_filter(seed + 1, layer.K, layer.R, layer.S, layer.C)
        dy64 = synth.normal(seed + 2, (layer.N, layer.P, layer.Q, layer.K))
        (x32, xb), (w32, wb), (dy32, dyb) = (synth.quantize(t, dtype) for t in (x64, w64, dy64))
        del x64, w64, dy64
        dev = lambda bits: torch.from_numpy(bits.view(np.int16)).view(tdt).cuda()
        nsets = max(2, min(8, int(6e8 // max(layer.bytes_fwd(), 1))))       # > 512 MB of rotating buffers for small layers
        sets = []
        desc = api.desc_from_layer(layer, dtype)
        for _ in range(nsets):
            x, w, dy = dev(xb), dev(wb), dev(dyb)
            sets.append((x, w, dy, torch.empty_like(dy), torch.empty_like(x), torch.empty_like(w),
                         torch.empty(max(16, max(api.dl_conv_workspace_bytes(desc, p) for p in range(3))),
                                     dtype=torch.uint8, device="cuda")))
        shp = oracle.ConvShape(layer.N, layer.H, layer.W, layer.C, layer.K, layer.R, layer.S, layer.stride, layer.pad, layer.dil)
        calls = {"fwd": (lambda b: api.conv2d_fwd(desc, b[0], b[1], y=b[3], workspace=b[6]), api.PASS_FWD,
                         lambda: oracle.conv_fwd(shp, x32, w32)),
                 "dgrad": (lambda b: api.conv2d_bwd_data(desc, b[2], b[1], dx=b[4], workspace=b[6]), api.PASS_BWD_DATA,
                           lambda: oracle.conv_bwd_data(shp, dy32, w32)),
                 "wgrad": (lambda b: api.conv2d_bwd_filter(desc, b[0], b[2], dw=b[5], workspace=b[6]), api.PASS_BWD_FILTER,
                           lambda: oracle.conv_bwd_filter(shp, x32, dy32))}
        for which, (fn, pid, orc) in calls.items():
            for i in range(max(args.warmup, nsets)):
                fn(sets[i % nsets])
            torch.cuda.synchronize()
            # groups of back-to-back calls between two events (launch latency is not what is measured),
            # each call on the next buffer set
            reps = 10 if layer.flops() < 1e11 else 3
            ts = []
            for g in range(max(args.steps, 10)):
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                for i in range(reps):
                    fn(sets[(g * reps + i) % nsets])
                b.record()
                torch.cuda.synchronize()
                ts.append(a.elapsed_time(b) / reps)
            ms = float(np.median(ts))
            t0 = time.perf_counter()
            orc()
            osec = time.perf_counter() - t0
            tf = layer.flops() / (ms * 1e-3) / 1e12
            gbs = layer.bytes_fwd() / (ms * 1e-3) / 1e9
            tot_ms += ms
            tot_flop += layer.flops()
            tot_orc += osec
            lo, hi = np.percentile(ts, [16, 84])
            print(f"{layer.name:24s} {which:6s} {ms:9.4f} {lo:8.4f} {hi:8.4f} {tf:9.1f} {100 * tf / MFMA_PEAK_TFLOPS:6.1f} {gbs:10.0f} "
                  f"{100 * gbs / HBM_PEAK_GBS:6.1f} {osec:9.2f} {layer.flops() / osec / 1e9:14.1f}  "
                  f"{api.dl_conv_describe(desc, pid)}", flush=True)
        del sets
        torch.cuda.empty_cache()
    line = {"metric": f"conv fwd+bwd TFLOP/s, config {args.config} (sum over its layers and passes, one stream)",
            "value": tot_flop / (tot_ms * 1e-3) / 1e12, "unit": "TFLOP/s", "n_gpus": 1, "dtype": dtype, "data": "synthetic",
            "config": {"workload": f"config{args.config}", "ms_sum_of_medians": tot_ms, "flop": tot_flop,
                       "frac_of_mfma_peak": tot_flop / (tot_ms * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS},
            "cpu_baseline": {"value": tot_flop / tot_orc / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
                             "sample": f"the same layers and passes in full, {tot_orc:.1f} s"}}
    print(json.dumps(line), flush=True)


def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py measures one GPU's share of the step; it runs with --gpus 1 only "
              "(no collectives are part of this build).", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_1810_01993_amd import api, layers, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.deconv_table:
        deconv_table(args)
        return
    if args.tiramisu_table:
        tiramisu_table(args)
        return
    if args.config != 5:
        config_table(args)
        return
    _, table = layers.config5()

    # one buffer set per occurrence, so repeated shapes do not re-use cache-resident tensors
    net = []
    for li, layer in enumerate(table):
        for occ in range(layer.count):
            net.append(LayerState(api, layer, synth.seed_for(5, 100 * li + occ), torch, args.dtype, args.activations))
    n_pix = 2 * 768 * 1152
    tdtype = torch.bfloat16 if args.dtype == "bf16" else torch.float16
    logits = torch.randn((n_pix, 3), device="cuda").to(tdtype)
    labels = torch.from_numpy(synth.ellipse_labels(synth.seed_for(5, 990), 2, 768, 1152).ravel()).cuda()
    cw = torch.tensor(synth.CLASS_WEIGHTS, dtype=torch.float32, device="cuda")
    dlogits = torch.empty_like(logits)
    loss = torch.empty(1, dtype=torch.float32, device="cuda")
    ce_ws = torch.empty(max(api.dl_ce_workspace_bytes(n_pix), 16), dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()

    # HIP events bracket the calls of the dominant kernel and the loss in every timed step;
    # with --table every call is bracketed (a few hundred more events per step).
    timed = {(i, which) for i, st in enumerate(net) for (name, which) in DOMINANT_CALLS if st.layer.name == name}
    timed.add(("loss", "loss"))

    side_streams = [torch.cuda.Stream() for _ in range(args.streams - 1)]   # default priority
    fused_i, fused_ws = None, None
    if args.fused_logits:
        fused_i = next(i for i, st in enumerate(net) if st.layer.name.startswith("logits"))
        fused_ws = torch.empty(api.logits_ce_workspace_bytes(n_pix, net[fused_i].layer.C), dtype=torch.uint8, device="cuda")

    def step(events=None):
        def rec(key):
            if events is not None and (args.table or (key[0], key[1]) in timed):
                e = torch.cuda.Event(enable_timing=True)
                e.record()
                events.append((key, e))
        for i, st in enumerate(net):
            if i == fused_i:
                continue
            rec((i, "fwd", 0))
            api.conv2d_fwd(st.desc, st.x, st.w, y=st.y, workspace=st.ws)
            rec((i, "fwd", 1))
        rec(("loss", "loss", 0))
        if fused_i is None:
            api.weighted_pixel_ce_fwd_bwd(logits, labels, cw, 1.0 / n_pix, loss=loss, dlogits=dlogits, workspace=ce_ws)
        else:       # forward, loss and both gradients of the logits layer: one pass over its input
            st = net[fused_i]
            api.logits_ce_fused_fwd_bwd(st.x.view(n_pix, -1), st.w, labels, cw, 1.0 / n_pix, dx=st.dx.view(n_pix, -1),
                                        workspace=fused_ws, logits=st.y.view(n_pix, 3), dlogits=dlogits, loss=loss, dw=st.dw)
        rec(("loss", "loss", 1))
        # Backward.  In the network, layer i's filter gradient and data gradient both consume
        # dy_i, which the layer above has produced before either starts.  With several streams the
        # data-gradient chain stays on the main stream and the filter gradients of the small
        # layers (tens of microseconds each, too short to fill the chip alone) follow on the
        # side streams in turn (they are independent of each other), each gated by an event recorded on the main stream at the point where
        # its dy exists; the large decoder layers and the bandwidth-bound full-resolution logits
        # layer, which fill the chip by themselves, keep both passes on the main stream.
        for i in range(len(net) - 1, -1, -1):
            if i == fused_i:
                continue
            st = net[i]
            side = bool(side_streams) and st.layer.flops() < 1e12 and st.layer.bytes_fwd() < 2e8
            if side:
                side_stream = side_streams[i % len(side_streams)]
                ready = torch.cuda.Event()
                ready.record()
                side_stream.wait_event(ready)
            rec((i, "dgrad", 0))
            api.conv2d_bwd_data(st.desc, st.dy, st.w, dx=st.dx, workspace=st.ws)
            rec((i, "dgrad", 1))
            if side:
                with torch.cuda.stream(side_stream):
                    rec((i, "wgrad", 0))
                    api.conv2d_bwd_filter(st.desc, st.x, st.dy, dw=st.dw, workspace=st.ws_w)
                    rec((i, "wgrad", 1))
            else:
                rec((i, "wgrad", 0))
                api.conv2d_bwd_filter(st.desc, st.x, st.dy, dw=st.dw, workspace=st.ws_w)
                rec((i, "wgrad", 1))
        for ss in side_streams:
            done = torch.cuda.Event()
            done.record(ss)
            torch.cuda.current_stream().wait_event(done)

    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")      # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    all_events = []
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]    # step boundaries on the main stream
    t0 = time.perf_counter()
    for k in range(args.steps):
        ev = []
        marks[k].record()
        step(ev)
        all_events.append(ev)
    marks[args.steps].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    # the paper's throughput statistic (Sec. "Performance Measurement"): median over the steps, with the
    # 0.16 and 0.84 percentiles as the error bar
    per_step = np.array([marks[k].elapsed_time(marks[k + 1]) for k in range(args.steps)])
    step_stat = {"median": float(np.median(per_step)), "p16": float(np.percentile(per_step, 16)),
                 "p84": float(np.percentile(per_step, 84))}

    # per-call device times from the HIP events recorded inside the timed region
    times = {}
    for ev in all_events:
        opened = {}
        for (key, e) in ev:
            who, which, end = key
            if end == 0:
                opened[(who, which)] = e
            else:
                times.setdefault((who, which), []).append(opened[(who, which)].elapsed_time(e))
    med = {k: float(np.median(v)) for k, v in times.items()}

    loss_big = loss_hbm_resident(api, torch, probes=not args.no_microbench)
    micro = None if args.no_microbench else mfma_microbench(api, torch)

    step_flops = layers.total_flops(table, passes=3)
    value = step_flops / (ms_per_step * 1e-3) / 1e12

    dom_ms, dom_flops, dom_n = 0.0, 0.0, 0
    for i, st in enumerate(net):
        for (name, which) in DOMINANT_CALLS:
            if st.layer.name == name:
                dom_ms += float(np.mean(times[(i, which)]))
                dom_flops += st.layer.flops()
                dom_n += 1
    achieved = (dom_flops / dom_n) / (dom_ms / dom_n * 1e-3) / 1e12
    conv_ms = sum(v for (who, which), v in med.items() if which != "loss") if args.table else None
    loss_ms = med[("loss", "loss")]

    if args.table:
        print(f"{'layer':28s} {'pass':6s} {'ms':>9s} {'p16':>8s} {'p84':>8s} {'TFLOP/s':>9s} {'%MFMA':>6s} {'GB/s(min)':>10s} {'%HBM':>6s}",
              file=sys.stderr)
        for i, st in enumerate(net):
            for which in ("fwd", "dgrad", "wgrad"):
                if (i, which) not in med:                 # --fused-logits: inside the "loss" line
                    continue
                ms = med[(i, which)]
                tf = st.layer.flops() / (ms * 1e-3) / 1e12
                gbs = st.layer.bytes_fwd() / (ms * 1e-3) / 1e9
                lo, hi = np.percentile(times[(i, which)], [16, 84])
                print(f"{st.layer.name:28s} {which:6s} {ms:9.4f} {lo:8.4f} {hi:8.4f} {tf:9.1f} {100 * tf / MFMA_PEAK_TFLOPS:6.1f} {gbs:10.0f} "
                      f"{100 * gbs / HBM_PEAK_GBS:6.1f}", file=sys.stderr)
        print(f"loss: {loss_ms:.4f} ms  ({13 * n_pix / (loss_ms * 1e-3) / 1e9:.0f} GB/s algorithmic)", file=sys.stderr)
        print(f"sum of per-call medians: conv {conv_ms:.3f} ms, loss {loss_ms:.4f} ms; wall {ms_per_step:.3f} ms/step",
              file=sys.stderr)

    # the dominant kernel's name comes from the dispatch these calls actually take
    pass_id = {"fwd": api.PASS_FWD, "dgrad": api.PASS_BWD_DATA, "wgrad": api.PASS_BWD_FILTER}
    plans = []
    for i, st in enumerate(net):
        for (name, which) in DOMINANT_CALLS:
            if st.layer.name == name:
                plans.append(f"{name} {which}: " + api.dl_conv_describe(st.desc, pass_id[which]))
    main_kernels = sorted({k.split("[")[0] for pl in plans for k in pl.split(": ", 1)[1].split("; ")
                           if not k.startswith("filter_block_kernel")})
    traffic, traffic_src = read_traffic(args.traffic_file)

    out = {
        "metric": "conv fwd+bwd TFLOP/s, DeepLabv3+ layers @1152x768x16 (63 conv layers x fwd/dgrad/wgrad + weighted pixel CE)",
        "value": value,
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": args.dtype,
        "data": "synthetic",
        "config": {"workload": f"config5: DeepLabv3+ conv stack + loss, N=2, 1152x768x16, {'bf16' if args.dtype == 'bf16' else 'fp16'} in / fp32 accumulate",
                   "streams": args.streams, "activations": args.activations, "fused_logits": bool(args.fused_logits),
                   "flop_per_step": step_flops, "frac_of_mfma_peak": value / MFMA_PEAK_TFLOPS,
                   "step_ms": step_stat,
                   "tflops_median_p16_p84": [step_flops / (step_stat[q] * 1e-3) / 1e12 for q in ("median", "p84", "p16")],
                   "conv_ms_sum_of_medians": conv_ms, "loss_ms": loss_ms,
                   "loss_gbs": 13 * n_pix / (loss_ms * 1e-3) / 1e9,
                   "loss_hbm_resident": loss_big, "mfma_microbench": micro},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / MFMA_PEAK_TFLOPS, "traffic": traffic, "traffic_source": traffic_src,
                     "kernel": " + ".join(main_kernels) + f" ({args.dtype})", "dispatch": plans,
                     "launches_per_step": dom_n,
                     "avg_launch_ms": dom_ms / dom_n, "flop_per_launch": dom_flops / dom_n},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
