"""Hardware-aware layer-wise bitwidth search on the device (Sec. III-C, Eq. 2 - Eq. 4, Alg. 1).

The paper's framework asks a cycle-accurate simulator of its accelerator for the latency of every
layer in every (W, A) mode.  Here the device itself is asked: each convolution / linear layer of a
network is timed in all nine modes {8, 4, 2} x {8, 4, 2} with the library's kernels on the layer's
real input tensor, the quantization error of every weight and activation tensor at each width comes
from dybit_rmse, and dybit_search runs the search flow over those tables.  Weights are whatever the
caller supplies (random in the benchmark: accuracy is out of reach without trained models, the
latency side is not).
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B
from .network import DybitNetwork

LEVELS = (8, 4, 2)


def _time(fn, steps: int, warmup: int) -> float:
    """Mean milliseconds per call, from device events on the current stream."""
    for _ in range(warmup):
        fn()
    t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0.record()
    for _ in range(steps):
        fn()
    t1.record()
    t1.synchronize()
    return t0.elapsed_time(t1) / steps


def measure_tables(layers, weights, x: torch.Tensor, steps: int = 10, warmup: int = 3):
    """Latency and error tables of a network for the input batch x (NHWC float32 on the device).

    A layer's latency in mode (W, A) is one step of the chain as DybitNetwork runs it: encode the
    layer's fp32 input at A bits from its known maximum (dybit_quantize_absmax), then the
    convolution against the W-bit weights with bias, shortcut, ReLU and the running maximum in
    the epilogue (dybit_conv2d_ex).  The input tensors are those of the (8, 8) network.
    Returns {"names", "lat" [L][3][3] ms, "rmse_w" [L][3], "rmse_a" [L][3]}."""
    names = [l["name"] for l in layers if l["op"] in ("conv", "fc")]
    index = {n: i for i, n in enumerate(names)}
    lat = np.zeros((len(names), 3, 3))
    rmse_w = np.zeros((len(names), 3))
    rmse_a = np.zeros((len(names), 3))
    err = torch.empty(4, dtype=torch.float64, device=x.device)

    # inputs of every layer, from a pass of the all-8-bit network
    inputs = {}
    reference = DybitNetwork(layers, weights, {n: (8, 8) for n in names}, device=x.device)
    reference.forward(x, record=lambda name, rec: inputs.__setitem__(name, (rec["x"][..., :rec["cin"]].contiguous(),
                                                                            rec["a_fmt"][1], rec["shortcut"])))
    for name in names:
        src, a_signed, _ = inputs[name]
        flat = src.reshape(-1)
        for ai, ba in enumerate(LEVELS):
            s = B.dybit_absmax_scale(flat, ba, a_signed)
            rmse_a[index[name], ai] = B.dybit_rmse(flat, s, ba, a_signed, out=err)[0].item()
        wd = torch.from_numpy(np.ascontiguousarray(weights[name][0])).to(x.device).reshape(-1)
        for wi, bw in enumerate(LEVELS):
            s = B.dybit_absmax_scale(wd, bw, True)
            rmse_w[index[name], wi] = B.dybit_rmse(wd, s, bw, True, out=err)[0].item()

    word = torch.zeros(1, dtype=torch.float32, device=x.device)
    for wi, bw in enumerate(LEVELS):
        for ai, ba in enumerate(LEVELS):
            net = DybitNetwork(layers, weights, {n: (bw, ba) for n in names}, device=x.device)
            for l in layers:
                if l["op"] not in ("conv", "fc"):
                    continue
                src, a_signed, shortcut = inputs[l["name"]]
                Bn, H, W, C = src.shape
                p = net._layer_params(l, H, W) if l["op"] == "conv" else net.params[l["name"]]
                if p["cpad"] != C:
                    src = torch.nn.functional.pad(src, (0, p["cpad"] - C))
                flat = src.reshape(-1)
                a_fmt = (ba, a_signed)
                amax = flat.abs().max().reshape(1)
                stride, pad = (l["stride"], l["pad"]) if l["op"] == "conv" else (1, 0)
                relu = bool(l.get("relu"))
                codes = torch.empty(B.dybit_packed_bytes(ba, a_signed, flat.numel()), dtype=torch.uint8, device=x.device)
                scale = torch.empty(1, dtype=torch.float32, device=x.device)
                Ho = (H + 2 * pad - p["k"]) // stride + 1
                Wo = (W + 2 * pad - p["kw"]) // stride + 1
                y = torch.empty((Bn, Ho, Wo, p["cout"]), dtype=torch.float32, device=x.device)

                def step():
                    B.dybit_quantize_absmax(flat, amax, *a_fmt, out=codes, scale_out=scale)
                    B.dybit_conv2d_ex(Bn, H, W, p["cpad"], p["cout"], p["k"], p["kw"], stride, pad, codes, a_fmt, scale,
                                      p["w_codes"], p["w_fmt"], p["w_scale"], p["bias"], shortcut, relu, word, out=y)

                lat[index[l["name"]], wi, ai] = _time(step, steps, warmup)
            del net
    if B.dybit_get_last_async_error() != B.OK:
        raise RuntimeError("a kernel reported an unusable scale while the tables were measured")
    return {"names": names, "lat": lat, "rmse_w": rmse_w, "rmse_a": rmse_a}


def search_bitwidths(tables, strategy: str, constraint: float, k: int):
    """Runs dybit_search over measured tables.  Returns ({layer: (bits_W, bits_A)}, ratio, met)."""
    code = {"speedup": B.SEARCH_SPEEDUP, "rmse": B.SEARCH_RMSE}[strategy]
    w, a, ratio, met = B.dybit_search(tables["lat"], tables["rmse_w"], tables["rmse_a"], code, constraint, k)
    return {n: (w[i], a[i]) for i, n in enumerate(tables["names"])}, ratio, met
