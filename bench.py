#!/usr/bin/env python3
"""Benchmark of the DyBit hot path on one MI355X.

A step is one pass of the path over one batch of seeded synthetic input that is already
resident in HBM: per-tensor absmax scale of the fp32 activations -> quantize them to DyBit
codes -> DyBit x DyBit GEMM (decode, MFMA contraction, scale/bias epilogue) against weights
that were quantized once at set-up.  The default workload is the large configuration the
targets are quoted on: M = N = K = 8192, 4-bit signed weights (Laplace), 8-bit signed
activations (Gaussian with 1 % outliers at 10 sigma), followed by the standalone quantize
of a 2^28-element Laplace tensor at 4 and 8 bits, which is reported separately.

Prints ONE JSON line.  `value` is the effective throughput of the whole step,
2*M*N*K / step time, in TOPS.  `roofline` describes the GEMM kernel alone (HIP events
around its launches inside the timed region), `quantize` / `roofline_quantize` the HBM-bound
quantize pass, `cpu_baseline` the plain C oracle timed on the host cores over a bounded sample.
Two more objects come from extra kernels timed after the step: `roofline_4bit_w_a` (the same
8192^3 product with the activations quantized to 4 bits, which runs on the fp8 matrix path)
and `conv_4bit_w_a` (the 3x3 convolution of configuration 2).

`--workload cfg1|cfg2|cfg3|cfg4` time the other configurations; `--table` runs all of them.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

SETTLE_STEPS = 30          # untimed steps that always run before the timed region (clock settling)
PEAK_FP16_MFMA_TFLOPS = 2500.0   # MI355X dense fp16/bf16 matrix peak
PEAK_FP8_MFMA_TFLOPS = 5000.0    # MI355X dense fp8 matrix peak (pairs of 4-bit formats run on it)
PEAK_HBM_GBPS = 8000.0           # MI355X HBM3E peak

# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (units of 2 KiB and 1 KiB on
# this device, calibrated on a 1 GiB copy); the summaries are under profiles/.
MEASURED_TRAFFIC = {"cfg5": 262303 * 2048 + 262222 * 1024, "cfg2": 2119 * 2048 + 12544 * 1024, "cfg1": None}
MEASURED_TRAFFIC_GEMM_4BIT = 196756 * 2048 + 262305 * 1024
MEASURED_TRAFFIC_QUANTIZE4 = 524376 * 2048 + 131072 * 1024


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=30,
                    help="untimed steps; the device needs a few tens of milliseconds of load to settle its clocks")
    ap.add_argument("--workload", default="cfg5", choices=["cfg5", "cfg2", "cfg1", "cfg3", "cfg4", "modes", "search", "dwconv"],
                    help="cfg5 (default): 8192^3 GEMM + 2^28 quantize; cfg1 / cfg2: the small GEMM and the "
                         "convolution; cfg3 / cfg4: one forward pass of the ResNet-18 / ResNet-50 chains")
    ap.add_argument("--network", default="resnet18", choices=["resnet18", "resnet50"], help="network of --workload search")
    ap.add_argument("--table", action="store_true",
                    help="run every configuration in a child process each and print a markdown table")
    ap.add_argument("--size", type=int, default=8192, help="M=N=K of the cfg5 GEMM")
    ap.add_argument("--quantize-log2n", type=int, default=28)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-quantize", action="store_true", help="skip the standalone 2^28 quantize")
    return ap.parse_args()


def time_events(fn, steps, warmup, torch):
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for s, e in ev:
        s.record()
        fn()
        e.record()
    torch.cuda.synchronize()
    ts = sorted(s.elapsed_time(e) for s, e in ev)
    return float(np.mean(ts)), float(ts[len(ts) // 2])


def time_batches(fn, launches, batches, warmup, torch):
    """Average duration of a launch over back-to-back launches: one event pair around each batch (a
    kernel shorter than the gap between two host calls is otherwise timed with that gap included)."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    ts = []
    for _ in range(batches):
        s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s.record()
        for _ in range(launches):
            fn()
        e.record()
        torch.cuda.synchronize()
        ts.append(s.elapsed_time(e) / launches)
    return float(np.mean(ts))


def network_roofline(work, ms):
    """Network-level bound of the dynamic chain: per layer the larger of its matrix time at the peak
    of the MFMA type its operands run on (e4m3 for two 4-bit operands, else fp16) and its HBM time for
    the algorithmic bytes (packed operands once, fp32 output once, fp32 shortcut once), plus the HBM
    time of the quantize pass over the layer's input (4 + bits/8 bytes per activation); summed over
    the layers and divided by the measured time of a forward pass."""
    t_mfma = t_hbm = t_bound = 0.0
    for w in work:
        flops = 2.0 * w["M"] * w["N"] * w["K"]
        peak = PEAK_FP8_MFMA_TFLOPS if (w["bits_w"] == 4 and w["bits_a"] == 4) else PEAK_FP16_MFMA_TFLOPS
        byts = w["inputs"] * w["bits_a"] / 8 + w["N"] * w["K"] * w["bits_w"] / 8 + 4.0 * w["M"] * w["N"] * (2 if w["shortcut"] else 1)
        quant = w["inputs"] * (4 + w["bits_a"] / 8)
        tm, th = flops / (peak * 1e12), byts / (PEAK_HBM_GBPS * 1e9)
        t_mfma += tm
        t_hbm += th + quant / (PEAK_HBM_GBPS * 1e9)
        t_bound += max(tm, th) + quant / (PEAK_HBM_GBPS * 1e9)
    flops = sum(2.0 * w["M"] * w["N"] * w["K"] for w in work)
    return {"bound": "hbm+mfma", "rule": "per layer max(mfma time, hbm time) + hbm time of its quantize pass, summed",
            "achieved": round(flops / (ms * 1e-3) / 1e12, 3), "peak": round(flops / t_bound / 1e12, 3), "unit": "TOPS",
            "frac": round(t_bound * 1e3 / ms, 4), "bound_ms": round(t_bound * 1e3, 4),
            "mfma_ms_at_peak": round(t_mfma * 1e3, 4), "hbm_ms_at_peak": round(t_hbm * 1e3, 4), "traffic": None}


def bench_modes(args):
    """The (W, A) bitwidth mode matrix {8, 4, 2} x {8, 4, 2} the mixed-precision search chooses from
    (Sec. III-C), plus the 6-bit column and row: kernel time of the cfg5 GEMM shape for every pair, on the
    tensors of config 5 (weights signed, activations signed).  One JSON line with a TFLOP/s table."""
    import torch
    from paper_2302_12510_amd import binding as B
    from paper_2302_12510_amd import synth

    torch.cuda.set_device(0)
    B.lib()
    size = args.size
    cfg = synth.config5a(size=size)
    A = torch.from_numpy(cfg["A"]).cuda().reshape(-1)
    Wf = torch.from_numpy(cfg["W"]).cuda().reshape(-1)
    C = torch.empty((size, size), dtype=torch.float32, device="cuda")
    flops = 2.0 * size ** 3
    table = {}
    for bw in (8, 6, 4, 2):
        sw = B.dybit_absmax_scale(Wf, bw, True)
        qw = B.dybit_quantize(Wf, sw, bw, True)
        for ba in (8, 6, 4, 2):
            sa = B.dybit_absmax_scale(A, ba, True)
            qa = B.dybit_quantize(A, sa, ba, True)
            ms, _ = time_events(lambda: B.dybit_gemm(size, size, size, qa, (ba, True), sa, qw, (bw, True), sw, out=C),
                                args.steps, args.warmup, torch)
            table["W%d/A%d" % (bw, ba)] = {"kernel_ms": round(ms, 4), "TFLOPs": round(flops / (ms * 1e-3) / 1e12, 1)}
    assert B.dybit_get_last_async_error() == B.OK
    print(json.dumps({"metric": "DyBit GEMM kernel TFLOP/s per (W, A) bitwidth mode", "unit": "TFLOP/s", "n_gpus": 1,
                      "steps": args.steps, "warmup": args.warmup, "data": "synthetic",
                      "config": {"workload": "mode matrix: GEMM M=N=K=%d on the config 5 tensors, W and A signed" % size},
                      "modes": table}))


def bench_dwconv(args):
    """Depthwise 3 x 3 convolutions of the depthwise-separable network of Sec. IV (MobileNetV2 shapes, batch
    64): absmax-scaled 4-bit unsigned activations, 4-bit signed filters.  HBM-bound: bytes = codes read +
    fp32 results written.  One JSON line."""
    import torch
    from paper_2302_12510_amd import binding as B
    from paper_2302_12510_amd import synth

    torch.cuda.set_device(0)
    B.lib()
    rows = []
    for (hw, c, stride) in ((112, 96, 2), (56, 144, 1), (28, 192, 1), (14, 576, 1), (7, 960, 1)):
        x = torch.from_numpy(synth.half_normal((64, hw, hw, c), 1.0, seed=1)).cuda().reshape(-1)
        w = torch.from_numpy(synth.kaiming_normal((3, 3, c), 9, seed=2)).cuda().reshape(-1)
        sx = B.dybit_absmax_scale(x, 4, False)
        qx = B.dybit_quantize(x, sx, 4, False)
        sw = B.dybit_absmax_scale(w, 4, True)
        qw = B.dybit_quantize(w, sw, 4, True)
        ho = (hw + 2 - 3) // stride + 1
        y = torch.empty((64, ho, ho, c), dtype=torch.float32, device="cuda")
        ms, _ = time_events(lambda: B.dybit_dwconv2d(64, hw, hw, c, 3, 3, stride, 1, qx, (4, False), sx, qw, (4, True), sw,
                                                     None, True, None, out=y), args.steps, args.warmup, torch)
        byts = qx.numel() + qw.numel() + 4 * y.numel()
        rows.append({"shape": "64x%dx%dx%d stride %d" % (hw, hw, c, stride), "kernel_ms": round(ms, 4),
                     "GBps": round(byts / (ms * 1e-3) / 1e9, 1), "frac_of_8TBps": round(byts / (ms * 1e-3) / 1e9 / PEAK_HBM_GBPS, 4),
                     "GMACps": round(9.0 * y.numel() / (ms * 1e-3) / 1e9, 1)})
        del x, y, qx
    assert B.dybit_get_last_async_error() == B.OK
    best = max(rows, key=lambda r: r["GBps"])
    print(json.dumps({"metric": "DyBit depthwise convolution GB/s", "value": best["GBps"], "unit": "GB/s", "n_gpus": 1,
                      "steps": args.steps, "warmup": args.warmup, "higher_is_better": True, "dtype": "f32", "data": "synthetic",
                      "config": {"workload": "depthwise 3x3 convolutions, MobileNetV2 shapes, batch 64, W 4-bit signed, A 4-bit unsigned"},
                      "roofline": {"bound": "hbm", "kernel": "dybit dwconv_kernel", "achieved": best["GBps"], "peak": PEAK_HBM_GBPS,
                                   "unit": "GB/s", "frac": best["frac_of_8TBps"], "traffic": None, "shape": best["shape"]},
                      "layers": rows}))


def bench_search(args):
    """The layer-wise bitwidth search (Sec. III-C, Alg. 1) on measured latencies: every conv / linear layer
    of the network is timed on the device in the nine (W, A) modes of {8, 4, 2}^2, the tensor errors (Eq. 2)
    come from dybit_rmse, dybit_search picks the widths for a few constraints of both strategies, and the
    network is run with the widths found.  One JSON line."""
    import torch
    from paper_2302_12510_amd import binding as B
    from paper_2302_12510_amd import search, synth
    from paper_2302_12510_amd.network import DybitNetwork

    torch.cuda.set_device(0)
    B.lib()
    layers, batch = (synth.resnet18_layers(), 64) if args.network == "resnet18" else (synth.resnet50_layers(), 128)
    weights = synth.network_weights(layers, seed=0)
    x = torch.from_numpy(synth.network_input(batch, 224, seed=0)).cuda()
    t0 = time.perf_counter()
    tables = search.measure_tables(layers, weights, x, steps=max(3, args.steps // 5), warmup=3)
    t_tables = time.perf_counter() - t0

    def run(widths):
        net = DybitNetwork(layers, weights, widths)
        for _ in range(args.warmup):
            net.forward(x)
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(args.steps):
            net.forward(x)
        torch.cuda.synchronize()
        return (time.perf_counter() - t) * 1e3 / args.steps

    names = tables["names"]
    base_ms = run({n: (8, 8) for n in names})
    lat = tables["lat"]
    results = []
    for strategy, constraint in (("speedup", 1.05), ("speedup", 1.1), ("speedup", 1.15), ("rmse", 1.5), ("rmse", 2.0), ("rmse", 4.0)):
        t0 = time.perf_counter()
        widths, ratio, met = search.search_bitwidths(tables, strategy, constraint, 4)
        t_search = time.perf_counter() - t0
        idx = {8: 0, 4: 1, 2: 2}
        predicted = sum(lat[i, idx[widths[n][0]], idx[widths[n][1]]] for i, n in enumerate(names))
        error = sum(tables["rmse_w"][i, idx[widths[n][0]]] + tables["rmse_a"][i, idx[widths[n][1]]] for i, n in enumerate(names))
        ms = run(widths)
        results.append({"strategy": strategy, "constraint": constraint, "k": 4, "met": met, "ratio": round(ratio, 4),
                        "search_ms": round(t_search * 1e3, 3),
                        "sum_of_layer_latencies_ms": round(float(predicted), 4), "sum_of_layer_rmse": round(float(error), 4),
                        "forward_ms": round(ms, 4), "measured_speedup_over_8_8": round(base_ms / ms, 4),
                        "widths_W_A": {n: list(widths[n]) for n in names}})
    assert B.dybit_get_last_async_error() == B.OK
    print(json.dumps({
        "metric": "layer-wise bitwidth search on measured latencies", "unit": "ms", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "data": "synthetic (random weights: the error columns are those of these tensors, not of a trained model)",
        "config": {"workload": "search: %s, batch %d, 224x224, widths from {8,4,2}, k = 4" % (args.network, batch),
                   "layers": len(names)},
        "tables_seconds": round(t_tables, 1),
        "forward_ms_8_8": round(base_ms, 4),
        "sum_of_layer_latencies_ms_8_8": round(float(lat[:, 0, 0].sum()), 4),
        "sum_of_layer_latencies_ms_2_2": round(float(lat[:, 2, 2].sum()), 4),
        "sum_of_layer_rmse_8_8": round(float(tables["rmse_w"][:, 0].sum() + tables["rmse_a"][:, 0].sum()), 4),
        "layer_latency_ms": {n: [[round(float(v), 4) for v in row] for row in lat[i]] for i, n in enumerate(names)},
        "results": results}))


def bench_network(args):
    """Configs 3 and 4: a step is one forward pass of the chained network (per conv / linear layer
    scale -> quantize -> dybit_conv2d_ex with bias, shortcut and ReLU fused; pooling in torch)."""
    import torch
    from paper_2302_12510_amd import binding as B
    from paper_2302_12510_amd import synth
    from paper_2302_12510_amd.network import DybitNetwork

    torch.cuda.set_device(0)
    B.lib()
    if args.workload == "cfg3":
        layers, batch = synth.resnet18_layers(), 64
        bits = synth.bitwidths_fixed(layers)
        name = "cfg3 ResNet-18 forward, batch 64, 224x224; first conv and fc 8-bit, other layers 4-bit W/A"
    else:
        layers, batch = synth.resnet50_layers(), 128
        bits = synth.bitwidths_mixed(layers, 0)
        name = "cfg4 ResNet-50 forward, batch 128, 224x224; per-layer (W, A) bits drawn from {4,6,8}, seed 0"
    net = DybitNetwork(layers, synth.network_weights(layers, seed=0), bits)
    x = torch.from_numpy(synth.network_input(batch, 224, seed=0)).cuda()

    def timed(fn):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / args.steps

    # a step = one forward pass; the same pass is also recorded into a HIP graph (every launch of the
    # pass, no host work per launch) and replayed: the faster of the two is the reported step
    ms_eager = timed(lambda: net.forward(x))
    graph, _ = net.capture(x)
    ms_graph = timed(graph.replay)
    ms = min(ms_eager, ms_graph)
    assert B.dybit_get_last_async_error() == B.OK
    shapes = net.gemm_shapes(batch, 224)
    flops = sum(2.0 * m * n * k for _, m, n, k in shapes)
    # the same network with calibrated (static) scales and the write-back fused into the epilogues
    net.calibrate(x)
    ms_static_eager = timed(lambda: net.forward(x, static=True))
    graph_static, _ = net.capture(x, static=True)
    ms_static_graph = timed(graph_static.replay)
    ms_static = min(ms_static_eager, ms_static_graph)
    assert B.dybit_get_last_async_error() == B.OK
    # ... and with the shortcuts and the max-pool on codes as well (no fp32 tensor between the stem and the average pool
    # wherever the readers of a tensor agree on a format)
    del graph, graph_static
    net_c = DybitNetwork(layers, synth.network_weights(layers, seed=0), bits, code_shortcuts=True)
    net_c.calibrate(x)
    ms_codes_eager = timed(lambda: net_c.forward(x, static=True))
    graph_codes, _ = net_c.capture(x, static=True)
    ms_codes_graph = timed(graph_codes.replay)
    ms_codes = min(ms_codes_eager, ms_codes_graph)
    assert B.dybit_get_last_async_error() == B.OK
    out = {
        "metric": "DyBit GEMM effective TOPS at 4-bit W/A (+ quantize GB/s), % of roofline",
        "value": round(flops / (ms * 1e-3) / 1e12, 3), "unit": "TOPS", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16 or e4m3 MFMA inputs by layer (exact), f32 accumulate", "data": "synthetic",
        "config": {"workload": name, "gemms": len(shapes), "GMAC": round(flops / 2e9, 1),
                   "step": "per layer scale + quantize + conv (bias, shortcut, ReLU and max|result| in the epilogue); pooling in torch; "
                           + ("launched from a HIP graph of the pass" if ms_graph <= ms_eager else "launched call by call")},
        "launch": {"eager_ms_per_step": round(ms_eager, 4), "hip_graph_replay_ms_per_step": round(ms_graph, 4)},
        "roofline": network_roofline(net.layer_work(batch, 224), ms),
        "fused_write_back": {"ms_per_step": round(ms_static, 4), "TOPS": round(flops / (ms_static * 1e-3) / 1e12, 3),
                             "eager_ms_per_step": round(ms_static_eager, 4), "hip_graph_replay_ms_per_step": round(ms_static_graph, 4),
                             "step": "scales fixed by a calibration pass; every convolution whose consumers agree on a "
                                     "format writes DyBit codes from its epilogue (dybit_conv2d_wb), fp32 only where a "
                                     "shortcut, a pooling or the output needs it",
                             "layers_writing_codes": sum(1 for p in net.plan.values() if p["fmt"]),
                             "layers_writing_codes_only": sum(1 for p in net.plan.values() if not p["fp32"])},
        "codes_only_chain": {"ms_per_step": round(ms_codes, 4), "TOPS": round(flops / (ms_codes * 1e-3) / 1e12, 3),
                             "eager_ms_per_step": round(ms_codes_eager, 4), "hip_graph_replay_ms_per_step": round(ms_codes_graph, 4),
                             "step": "the fused chain with the shortcut of a residual block read as the DyBit codes its tensor is "
                                     "stored as (dybit_conv2d_wb_rc) and the max-pool on codes (dybit_maxpool2d_codes)",
                             "shortcuts_read_as_codes": sum(1 for p in net_c.plan.values() if p["shortcut_codes"]),
                             "maxpools_on_codes": sum(1 for f in net_c.pool_fmt.values() if f),
                             "layers_writing_codes_only": sum(1 for p in net_c.plan.values() if not p["fp32"])},
    }
    if not args.no_cpu_baseline:
        # the oracle's convolution on a few images of one mid-network layer; the forward pass
        # has the same kind of work throughout, so its rate is what a full oracle pass would run at
        from oracle import c_ref
        rng = np.random.default_rng(0)
        xq = rng.integers(0, 16, (2, 28, 28, 128)).astype(np.uint8)
        wq = rng.integers(0, 16, (128, 3, 3, 128)).astype(np.uint8)
        t0 = time.perf_counter()
        c_ref.conv2d(xq, (4, False), 1.0, wq, (4, True), 1.0, 1, 1, want_den=False)
        dt = time.perf_counter() - t0
        rate = 2.0 * 2 * 28 * 28 * 128 * 9 * 128 / dt
        out["cpu_baseline"] = {"value": round(rate / 1e12, 5), "unit": "TOPS", "cores": c_ref.num_threads(),
                               "kind": "oracle", "seconds": round(dt, 2),
                               "sample": "3x3 conv 128->128 on 28x28, 2 images (one layer shape of the network); "
                                         "a full oracle pass at this rate would take %.0f s" % (flops / rate)}
    print(json.dumps(out))


def table(args):
    """Every configuration, each in a child process, as one markdown table."""
    import subprocess
    rows = []
    for wl in ("cfg1", "cfg2", "cfg3", "cfg4", "cfg5"):
        cmd = [sys.executable, os.path.abspath(__file__), "--workload", wl, "--steps", str(args.steps),
               "--warmup", str(args.warmup)] + (["--no-cpu-baseline"] if args.no_cpu_baseline else [])
        p = subprocess.run(cmd, capture_output=True, text=True)
        if p.returncode:
            sys.stderr.write(p.stderr)
            sys.exit(p.returncode)
        rows.append((wl, json.loads([l for l in p.stdout.splitlines() if l.startswith("{")][-1])))
    print("| Config | GPU time per step | Effective TOPS / GB/s | Dominant kernel alone | % of roofline | Oracle (cores) |")
    print("|---|---|---|---|---|---|")
    for wl, r in rows:
        rf, cb = r.get("roofline"), r.get("cpu_baseline")
        if rf and "kernel" in rf:
            kern = "%s: %.4f ms, %.1f TFLOP/s" % (rf["kernel"], rf["kernel_ms"], rf["achieved"])
            frac = "%.1f %% of %.0f TFLOP/s" % (100 * rf["frac"], rf["peak"])
        elif rf:                                                    # chained networks: per-layer bound, summed
            kern = "-"
            frac = "%.1f %% of the per-layer max(MFMA, HBM) bound (%.3f ms: MFMA %.3f ms, HBM %.3f ms at peak)" % (
                100 * rf["frac"], rf["bound_ms"], rf["mfma_ms_at_peak"], rf["hbm_ms_at_peak"])
        else:
            kern = frac = "-"
        orc = "%.4f TOPS (%d), %s" % (cb["value"], cb["cores"], cb["sample"]) if cb else "-"
        print("| %s | %.4f ms | %.3f TOPS | %s | %s | %s |" % (r["config"]["workload"], r["ms_per_step"], r["value"], kern, frac, orc))
        if "fused_write_back" in r:
            f = r["fused_write_back"]
            print("| the same network, calibrated scales, write-back fused into the epilogues (%d of %d layers write codes, %d of them codes only) | %.4f ms | %.3f TOPS | - | - | - |"
                  % (f["layers_writing_codes"], r["config"]["gemms"], f["layers_writing_codes_only"], f["ms_per_step"], f["TOPS"]))
        if "codes_only_chain" in r:
            f = r["codes_only_chain"]
            print("| the same fused chain with shortcuts and max-pool on codes (%d shortcuts, %d max-pools; %d layers codes only) | %.4f ms | %.3f TOPS | - | - | - |"
                  % (f["shortcuts_read_as_codes"], f["maxpools_on_codes"], f["layers_writing_codes_only"], f["ms_per_step"], f["TOPS"]))
        if "roofline_4bit_w_a" in r:
            f = r["roofline_4bit_w_a"]
            print("| 8192^3 GEMM at 4-bit W / 4-bit A (same tensors, activations quantized to 4-bit signed) | %.4f ms (kernel) | %.1f TOPS | %s | %.1f %% of %.0f TFLOP/s | - |"
                  % (f["kernel_ms"], f["achieved"], f["kernel"], 100 * f["frac"], f["peak"]))
        if "quantize" in r:
            q = r["quantize"]
            print("| cfg5b quantize 2^28 fp32, 4-bit / 8-bit | %.4f / %.4f ms | %.0f / %.0f GB/s | quantize_kernel | %.1f %% / %.1f %% of 8000 GB/s (copy: %.0f GB/s) | - |"
                  % (q["4bit"]["ms"], q["8bit"]["ms"], q["4bit"]["GBps"], q["8bit"]["GBps"],
                     100 * q["4bit"]["frac_of_8TBps"], 100 * q["8bit"]["frac_of_8TBps"], q["torch_copy_reference"]["GBps"]))
    print(json.dumps({wl: r for wl, r in rows}))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (--gpus must be 1)", file=sys.stderr)
        sys.exit(2)
    if args.table:
        return table(args)
    if args.workload in ("cfg3", "cfg4"):
        return bench_network(args)
    if args.workload == "modes":
        return bench_modes(args)
    if args.workload == "search":
        return bench_search(args)
    if args.workload == "dwconv":
        return bench_dwconv(args)
    import torch
    from paper_2302_12510_amd import binding as B
    from paper_2302_12510_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    B.lib()

    # ---------------- set-up (untimed): inputs to HBM, weights quantized once -----------
    if args.workload == "cfg5":
        size = args.size
        cfg = synth.config5a(size=size)
        a_fmt, w_fmt = (8, True), (4, True)
        M = N = K = size
        A = torch.from_numpy(cfg["A"]).cuda().reshape(-1)
        Wf = torch.from_numpy(cfg["W"]).cuda().reshape(-1)
        conv = None
        name = f"cfg5a GEMM M=N=K={size}, W 4-bit signed Laplace(0,0.02), A 8-bit signed N(0,1)+1% outliers at 10 sigma"
    elif args.workload == "cfg1":
        cfg = synth.config1()
        a_fmt, w_fmt = (4, False), (4, True)
        M, K = cfg["A"].shape
        N = cfg["W"].shape[0]
        A = torch.from_numpy(cfg["A"]).cuda().reshape(-1)
        Wf = torch.from_numpy(cfg["W"]).cuda().reshape(-1)
        conv = None
        name = "cfg1 GEMM 64x64x256, W 4-bit signed, A 4-bit unsigned"
    else:
        cfg = synth.config2()
        a_fmt, w_fmt = (4, False), (4, True)
        Bn, H, Wd, Cin = cfg["X"].shape
        Cout, kh, kw, _ = cfg["Wt"].shape
        M, N, K = Bn * H * Wd, Cout, kh * kw * Cin
        A = torch.from_numpy(cfg["X"]).cuda().reshape(-1)
        Wf = torch.from_numpy(cfg["Wt"]).cuda().reshape(-1)
        conv = (Bn, H, Wd, Cin, Cout, kh, kw, cfg["stride"], cfg["pad"])
        name = "cfg2 conv 3x3 256->256 on 14x14, batch 64 (M=12544,N=256,K=2304), W 4-bit signed, A 4-bit unsigned"

    sw = B.dybit_absmax_scale(Wf, *w_fmt)
    qw = B.dybit_quantize(Wf, sw, *w_fmt)
    del Wf
    sa = torch.empty(1, dtype=torch.float32, device="cuda")
    qa = torch.empty(B.dybit_packed_bytes(*a_fmt, A.numel()), dtype=torch.uint8, device="cuda")
    C = torch.empty((M, N), dtype=torch.float32, device="cuda")
    g0 = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    g1 = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]

    def step(i=None):
        B.dybit_absmax_scale(A, *a_fmt, out=sa)
        B.dybit_quantize(A, sa, *a_fmt, out=qa)
        if i is not None:
            g0[i].record()
        if conv is None:
            B.dybit_gemm(M, N, K, qa, a_fmt, sa, qw, w_fmt, sw, out=C)
        else:
            B.dybit_conv2d(*conv, qa, a_fmt, sa, qw, w_fmt, sw, out=C)
        if i is not None:
            g1[i].record()

    # The device settles its clocks only after some tens of milliseconds of this load (the first 10 to
    # 15 steps of a process run 10 to 25 % slower).  SETTLE_STEPS untimed steps therefore always run,
    # whatever --warmup asks for beyond them; the line reports them as "settle_steps".
    for _ in range(max(args.warmup, SETTLE_STEPS)):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    assert B.dybit_get_last_async_error() == B.OK
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    gemm_ms = float(np.mean([a.elapsed_time(b) for a, b in zip(g0, g1)]))
    flops = 2.0 * M * N * K
    value = flops / (ms_per_step * 1e-3) / 1e12
    gemm_tflops = flops / (gemm_ms * 1e-3) / 1e12

    use_f8 = a_fmt[0] == 4 and w_fmt[0] == 4       # pairs of 4-bit formats run on the fp8 matrix path
    peak = PEAK_FP8_MFMA_TFLOPS if use_f8 else PEAK_FP16_MFMA_TFLOPS
    out = {
        "metric": "DyBit GEMM effective TOPS at 4-bit W/A (+ quantize GB/s), % of roofline",
        "value": round(value, 3), "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "settle_steps": max(args.warmup, SETTLE_STEPS),
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": ("e4m3" if use_f8 else "f16") + " MFMA inputs (exact), f32 accumulate", "data": "synthetic",
        "config": {"workload": name, "M": M, "N": N, "K": K, "a_fmt": list(a_fmt), "w_fmt": list(w_fmt),
                   "step": "absmax + quantize activations + gemm; weights pre-quantized"},
        "roofline": {"bound": "mfma", "kernel": {"cfg5": "dybit::fast::gemm_fast_kernel (256x256 tiles, fp16 MFMA)", "cfg2": "dybit::f8::gemm_f8_kernel (128x128 tiles, two k-groups, e4m3 MFMA)", "cfg1": "dybit::f8::gemm_f8_kernel (128x128 tiles, e4m3 MFMA)"}[args.workload], "achieved": round(gemm_tflops, 2),
                     "peak": peak, "unit": "TFLOP/s",
                     "frac": round(gemm_tflops / peak, 4),
                     "kernel_ms": round(gemm_ms, 4), "traffic": MEASURED_TRAFFIC[args.workload]},
    }

    # ---------------- the matrix cores alone, on decoded values of this workload ------------
    # (the sustained clock of an MFMA-bound kernel depends on the operand values: the A operand of
    # the instruction gets activation values, the B operands weight values, as in the product)
    def sample(q, fmt, s, need):
        n = min(need, q.numel() * 8 // fmt[0])
        v = B.dybit_dequantize(q[: n * fmt[0] // 8], n, s, *fmt) / s
        if not use_f8 and fmt[0] in (6, 8):
            v = v * 2.0 ** -14                     # the fp16 kernels decode 6- and 8-bit operands on this scale
        return v.repeat((need + n - 1) // n)[:need]
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    per_lane = 32 if use_f8 else 8                 # operand elements per lane of one instruction
    ops = torch.cat([sample(qa, a_fmt, sa, 512 * per_lane), sample(qw, w_fmt, sw, 8 * 512 * per_lane)])
    if use_f8:
        ops = ops.to(torch.float8_e4m3fn).view(torch.uint8).contiguous()
        diag, iters = B.dybit_diag_mfma_f8, 1000
    else:
        ops = ops.to(torch.float16).contiguous()
        diag, iters = B.dybit_diag_mfma_f16, 2000
    wgs = 256 * 2
    fl = diag(ops, wgs, iters, sink)
    mf_ms, _ = time_events(lambda: diag(ops, wgs, iters, sink), 5, 2, torch)
    out["roofline"]["mfma_only_measured_TFLOPs"] = round(fl / (mf_ms * 1e-3) / 1e12, 1)
    out["roofline"]["frac_of_mfma_only_measured"] = round(gemm_tflops / (fl / (mf_ms * 1e-3) / 1e12), 4)

    # ---------------- activation-side passes of the step, timed alone --------------------
    nA = A.numel()
    absmax_ms, _ = time_events(lambda: B.dybit_absmax_scale(A, *a_fmt, out=sa), 10, 2, torch)
    qa_ms, _ = time_events(lambda: B.dybit_quantize(A, sa, *a_fmt, out=qa), 10, 2, torch)
    out["step_breakdown_ms"] = {"absmax": round(absmax_ms, 4), "quantize_activations": round(qa_ms, 4),
                                "gemm": round(gemm_ms, 4)}

    # ---------------- standalone quantize (config 5b) and a copy for reference -----------
    if args.workload == "cfg5" and not args.no_quantize:
        del C
        n = 1 << args.quantize_log2n
        x = torch.from_numpy(synth.config5b(n=n)).cuda()
        q = {}
        for bits in (4, 8):
            fmt = (bits, True)
            s = B.dybit_absmax_scale(x, *fmt)
            codes = torch.empty(B.dybit_packed_bytes(*fmt, n), dtype=torch.uint8, device="cuda")
            ms, med = time_events(lambda: B.dybit_quantize(x, s, *fmt, out=codes), 20, 3, torch)
            gbps = (4 + bits / 8) * n / (ms * 1e-3) / 1e9
            q[f"{bits}bit"] = {"ms": round(ms, 4), "GBps": round(gbps, 1), "frac_of_8TBps": round(gbps / PEAK_HBM_GBPS, 4)}
            if bits == 8:
                y = torch.empty(n, dtype=torch.float32, device="cuda")
                dms, _ = time_events(lambda: B.dybit_dequantize(codes, n, s, *fmt, out=y), 10, 2, torch)
                q["dequantize_8bit"] = {"ms": round(dms, 4), "GBps": round(5.0 * n / (dms * 1e-3) / 1e9, 1)}
                del y
            del codes
        ams, _ = time_events(lambda: B.dybit_absmax_scale(x, 8, True, out=sa), 10, 2, torch)
        q["absmax"] = {"ms": round(ams, 4), "GBps": round(4.0 * n / (ams * 1e-3) / 1e9, 1)}
        y = torch.empty(n, dtype=torch.float32, device="cuda")
        fms, _ = time_events(lambda: B.dybit_fake_quant(x, s, 8, True, out=y), 10, 2, torch)
        q["fake_quant_8bit"] = {"ms": round(fms, 4), "GBps": round(8.0 * n / (fms * 1e-3) / 1e9, 1)}
        del y
        err = torch.empty(4, dtype=torch.float64, device="cuda")
        rms, _ = time_events(lambda: B.dybit_rmse(x, s, 8, True, out=err), 10, 2, torch)
        q["rmse_8bit"] = {"ms": round(rms, 4), "GBps": round(4.0 * n / (rms * 1e-3) / 1e9, 1), "value": round(err[0].item(), 6)}
        y = torch.empty_like(x)
        cms, _ = time_events(lambda: y.copy_(x), 10, 2, torch)
        q["torch_copy_reference"] = {"ms": round(cms, 4), "GBps": round(8.0 * n / (cms * 1e-3) / 1e9, 1)}
        q["n"] = n
        out["quantize"] = q
        out["roofline_quantize"] = {"bound": "hbm", "kernel": "dybit quantize_kernel<4,signed>",
                                    "achieved": q["4bit"]["GBps"], "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                                    "frac": q["4bit"]["frac_of_8TBps"], "traffic": MEASURED_TRAFFIC_QUANTIZE4,
                                    "frac_of_measured_copy": round(q["4bit"]["GBps"] / q["torch_copy_reference"]["GBps"], 4)}
        del x, y

    # ---------------- the same product with 4-bit activations (4-bit W / 4-bit A) -----------
    # Two 4-bit operands are exact in e4m3 and run on the fp8 matrix path: its peak is the roofline.
    if args.workload == "cfg5" and not args.no_quantize:
        f4 = (4, True)
        sa4 = B.dybit_absmax_scale(A, *f4)
        qa4 = B.dybit_quantize(A, sa4, *f4)
        C4 = torch.empty((M, N), dtype=torch.float32, device="cuda")
        g4_ms, _ = time_events(lambda: B.dybit_gemm(M, N, K, qa4, f4, sa4, qw, w_fmt, sw, out=C4), args.steps, args.warmup, torch)
        tf4 = flops / (g4_ms * 1e-3) / 1e12
        # the fp8 matrix cores alone on e4m3 bytes of these values (torch has the dtype; the library only times it)
        def sample8(q, s, need):
            v = B.dybit_dequantize(q[: need // 2], need, s, *f4) / s
            return v.to(torch.float8_e4m3fn).view(torch.uint8)
        ops8 = torch.cat([sample8(qa4, sa4, 512 * 32), sample8(qw, sw, 8 * 512 * 32)]).contiguous()
        fl8 = B.dybit_diag_mfma_f8(ops8, 512, 1000, sink)
        m8_ms, _ = time_events(lambda: B.dybit_diag_mfma_f8(ops8, 512, 1000, sink), 5, 2, torch)
        out["roofline_4bit_w_a"] = {"bound": "mfma", "kernel": "dybit::f8::gemm_f8_kernel (256x256 tiles, e4m3 MFMA)",
                                    "workload": "the same 8192^3 product with the activations quantized to 4-bit signed",
                                    "achieved": round(tf4, 2), "peak": PEAK_FP8_MFMA_TFLOPS, "unit": "TFLOP/s",
                                    "frac": round(tf4 / PEAK_FP8_MFMA_TFLOPS, 4), "kernel_ms": round(g4_ms, 4), "traffic": MEASURED_TRAFFIC_GEMM_4BIT,
                                    "mfma_only_measured_TFLOPs": round(fl8 / (m8_ms * 1e-3) / 1e12, 1),
                                    "frac_of_mfma_only_measured": round(tf4 / (fl8 / (m8_ms * 1e-3) / 1e12), 4)}
        out["value_4bit_w_a"] = {"value": round(tf4, 2), "unit": "TOPS", "what": "the same product at 4-bit W / 4-bit A, kernel alone"}
        del C4, qa4

    # ---------------- the 4-bit W / 4-bit A convolution (config 2), kernel alone ------------
    if args.workload == "cfg5" and not args.no_quantize:
        c2 = synth.config2()
        f_x, f_w = (4, False), (4, True)
        Bn, H, Wd, Cin = c2["X"].shape
        Cout, kh, kw, _ = c2["Wt"].shape
        X2 = torch.from_numpy(c2["X"]).cuda().reshape(-1)
        W2 = torch.from_numpy(c2["Wt"]).cuda().reshape(-1)
        sx2, sw2 = B.dybit_absmax_scale(X2, *f_x), B.dybit_absmax_scale(W2, *f_w)
        qx2, qw2 = B.dybit_quantize(X2, sx2, *f_x), B.dybit_quantize(W2, sw2, *f_w)
        Y2 = torch.empty((Bn, H, Wd, Cout), dtype=torch.float32, device="cuda")
        conv2 = (Bn, H, Wd, Cin, Cout, kh, kw, c2["stride"], c2["pad"])
        c2_ms = time_batches(lambda: B.dybit_conv2d(*conv2, qx2, f_x, sx2, qw2, f_w, sw2, out=Y2), 25, 4, 5, torch)
        fl2 = 2.0 * Bn * H * Wd * Cout * kh * kw * Cin
        out["conv_4bit_w_a"] = {"workload": "cfg2 conv 3x3 256->256 on 14x14, batch 64, W 4-bit signed, A 4-bit unsigned",
                                "kernel": "dybit::f8::gemm_f8_kernel (128x128 tiles, two k-groups, e4m3 MFMA)",
                                "kernel_ms": round(c2_ms, 4), "timing": "HIP events around batches of 25 back-to-back launches",
                                "TFLOPs": round(fl2 / (c2_ms * 1e-3) / 1e12, 1),
                                "frac_of_fp8_mfma_peak": round(fl2 / (c2_ms * 1e-3) / 1e12 / PEAK_FP8_MFMA_TFLOPS, 4)}
        del X2, W2, Y2

    # ---------------- CPU baseline: the plain C oracle on a bounded sample -----------------
    if not args.no_cpu_baseline:
        from oracle import c_ref, dybit_ref as R
        qa_h = qa.cpu().numpy()
        qw_h = qw.cpu().numpy()
        if conv is None:
            rows = min(M, max(1, int(4.5e11 // (N * K))))       # ~450 GMAC of scalar C: 10-15 s on 16 cores
            a_codes = R.unpack(qa_h[: rows * K * a_fmt[0] // 8], rows * K, a_fmt[0]).reshape(rows, K)
            w_codes = R.unpack(qw_h, N * K, w_fmt[0]).reshape(N, K)
            t0 = time.perf_counter()
            c_ref.gemm(a_codes, a_fmt, sa.item(), w_codes, w_fmt, sw.item(), want_den=False)
            dt = time.perf_counter() - t0
            sample = f"first {rows} of {M} rows of the same GEMM (all N, all K)"
            sflops = 2.0 * rows * N * K
        else:
            Bn, H, Wd, Cin, Cout, kh, kw, stride, pad = conv
            nb = Bn
            x_codes = R.unpack(qa_h[: nb * H * Wd * Cin * a_fmt[0] // 8], nb * H * Wd * Cin, a_fmt[0]).reshape(nb, H, Wd, Cin)
            w_codes = R.unpack(qw_h, Cout * kh * kw * Cin, w_fmt[0]).reshape(Cout, kh, kw, Cin)
            t0 = time.perf_counter()
            c_ref.conv2d(x_codes, a_fmt, sa.item(), w_codes, w_fmt, sw.item(), stride, pad, want_den=False)
            dt = time.perf_counter() - t0
            sample = f"first {nb} of {Bn} images of the same convolution"
            sflops = 2.0 * (M // Bn * nb) * N * K
        out["cpu_baseline"] = {"value": round(sflops / dt / 1e12, 5), "unit": "TOPS", "cores": c_ref.num_threads(),
                               "kind": "oracle", "sample": sample, "seconds": round(dt, 2)}

    print(json.dumps(out))


if __name__ == "__main__":
    main()
