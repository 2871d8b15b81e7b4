"""Seeded synthetic inputs for the DyBit workloads.

This module only draws random tensors and lists layer shapes; it contains none
of the method's arithmetic (no codebook, no quantizer, no GEMM), so both the
HIP tests/benchmark and the CPU oracle may take their inputs from it.

All tensors are float32 numpy arrays drawn from numpy's PCG64 generator.  They
stand in for the ImageNet activations and the pretrained weights of the paper's
evaluation (Sec. IV-A): same shapes (ResNet-18/50 layers at 224x224) and the
value distributions usually assumed for them (Laplace / Kaiming-normal weights,
half-normal post-ReLU activations, Gaussian inputs with rare outliers).
"""
from __future__ import annotations

import numpy as np

_CHUNK = 1 << 24


def _rng(seed: int, stream: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([seed, stream]))


def _chunked(n: int, draw) -> np.ndarray:
    out = np.empty(n, dtype=np.float32)
    for lo in range(0, n, _CHUNK):
        hi = min(n, lo + _CHUNK)
        out[lo:hi] = draw(hi - lo)
    return out


def laplace(shape, b: float = 0.02, seed: int = 0, stream: int = 0) -> np.ndarray:
    """Laplace(0, b) weights."""
    g = _rng(seed, stream)
    n = int(np.prod(shape))
    return _chunked(n, lambda k: g.laplace(0.0, b, k)).reshape(shape)


def normal(shape, sigma: float = 1.0, seed: int = 0, stream: int = 0) -> np.ndarray:
    g = _rng(seed, stream)
    n = int(np.prod(shape))
    return _chunked(n, lambda k: g.normal(0.0, sigma, k)).reshape(shape)


def half_normal(shape, sigma: float = 1.0, seed: int = 0, stream: int = 0) -> np.ndarray:
    """|N(0, sigma)|: the shape of a post-ReLU activation."""
    return np.abs(normal(shape, sigma, seed, stream))


def kaiming_normal(shape, fan_in: int, seed: int = 0, stream: int = 0) -> np.ndarray:
    """N(0, sqrt(2 / fan_in)) convolution / linear weights."""
    return normal(shape, float(np.sqrt(2.0 / fan_in)), seed, stream)


def normal_with_outliers(shape, frac: float = 0.01, magnitude: float = 10.0,
                         seed: int = 0, stream: int = 0) -> np.ndarray:
    """N(0,1) with a Bernoulli(frac) subset replaced by +-magnitude (random sign)."""
    g = _rng(seed, stream)
    n = int(np.prod(shape))

    def draw(k):
        v = g.normal(0.0, 1.0, k)
        mask = g.random(k) < frac
        sign = np.where(g.random(k) < 0.5, -1.0, 1.0)
        return np.where(mask, sign * magnitude, v)

    return _chunked(n, draw).reshape(shape)


# --------------------------------------------------------------------------
# The five benchmark configurations
# --------------------------------------------------------------------------
def config1(seed: int = 0):
    """Small GEMM M=N=64, K=256: Laplace weights [N][K], half-normal activations [M][K]."""
    return {"W": laplace((64, 256), 0.02, seed, 1), "A": half_normal((64, 256), 1.0, seed, 2)}


def config2(seed: int = 0, batch: int = 64):
    """3x3 conv 256->256 on 14x14 (NHWC), stride 1, pad 1."""
    return {"X": half_normal((batch, 14, 14, 256), 1.0, seed, 1),
            "Wt": kaiming_normal((256, 3, 3, 256), 256 * 9, seed, 2),
            "stride": 1, "pad": 1}


def config5a(seed: int = 0, size: int = 8192):
    """Large GEMM: Laplace weights [N][K], Gaussian activations with 1% outliers at 10 sigma."""
    return {"W": laplace((size, size), 0.02, seed, 1),
            "A": normal_with_outliers((size, size), 0.01, 10.0, seed, 2)}


def config5b(seed: int = 0, n: int = 1 << 28):
    """Flat Laplace tensor for the standalone quantize pass."""
    return laplace((n,), 0.02, seed, 3)


# --------------------------------------------------------------------------
# Layer lists of the two chained networks (shapes only)
# --------------------------------------------------------------------------
def _conv(name, cin, cout, k, stride, pad, src, relu=True, add=None):
    return {"name": name, "op": "conv", "cin": cin, "cout": cout, "k": k, "stride": stride,
            "pad": pad, "src": src, "relu": relu, "add": add}


def resnet18_layers():
    """Layer list of the ResNet-18 topology (7x7/2 stem, 3x3/2 max-pool, four stages
    of two basic blocks, global average pool, 1000-way linear layer).

    Every entry names its input tensor (`src`), and, for the second conv of a
    block, the tensor added before the final ReLU (`add`)."""
    L = [_conv("conv1", 3, 64, 7, 2, 3, "input"),
         {"name": "pool1", "op": "maxpool", "k": 3, "stride": 2, "pad": 1, "src": "conv1"}]
    prev = "pool1"
    cin = 64
    for stage, cout in enumerate([64, 128, 256, 512], start=1):
        for blk in range(2):
            stride = 2 if (stage > 1 and blk == 0) else 1
            base = f"l{stage}b{blk}"
            skip = prev
            if stride != 1 or cin != cout:
                L.append(_conv(base + "ds", cin, cout, 1, stride, 0, prev, relu=False))
                skip = base + "ds"
            L.append(_conv(base + "c1", cin, cout, 3, stride, 1, prev))
            L.append(_conv(base + "c2", cout, cout, 3, 1, 1, base + "c1", relu=True, add=skip))
            prev = base + "c2"
            cin = cout
    L.append({"name": "avgpool", "op": "avgpool", "src": prev})
    L.append({"name": "fc", "op": "fc", "cin": 512, "cout": 1000, "src": "avgpool", "relu": False})
    return L


def resnet50_layers():
    """Bottleneck ResNet-50 topology with the stride on the 3x3 convolution."""
    L = [_conv("conv1", 3, 64, 7, 2, 3, "input"),
         {"name": "pool1", "op": "maxpool", "k": 3, "stride": 2, "pad": 1, "src": "conv1"}]
    prev = "pool1"
    cin = 64
    for stage, (width, nblk) in enumerate([(64, 3), (128, 4), (256, 6), (512, 3)], start=1):
        cout = width * 4
        for blk in range(nblk):
            stride = 2 if (stage > 1 and blk == 0) else 1
            base = f"l{stage}b{blk}"
            skip = prev
            if blk == 0:
                L.append(_conv(base + "ds", cin, cout, 1, stride, 0, prev, relu=False))
                skip = base + "ds"
            L.append(_conv(base + "c1", cin, width, 1, 1, 0, prev))
            L.append(_conv(base + "c2", width, width, 3, stride, 1, base + "c1"))
            L.append(_conv(base + "c3", width, cout, 1, 1, 0, base + "c2", relu=True, add=skip))
            prev = base + "c3"
            cin = cout
    L.append({"name": "avgpool", "op": "avgpool", "src": prev})
    L.append({"name": "fc", "op": "fc", "cin": 2048, "cout": 1000, "src": "avgpool", "relu": False})
    return L


def network_weights(layers, seed: int = 0):
    """Kaiming-normal weights [Cout][kh][kw][Cin] and small N(0, 0.01) biases (the
    folded batch-norm shift) for every conv / fc layer, keyed by layer name."""
    out = {}
    for idx, l in enumerate(layers):
        if l["op"] == "conv":
            k = l["k"]
            w = kaiming_normal((l["cout"], k, k, l["cin"]), l["cin"] * k * k, seed, 100 + idx)
        elif l["op"] == "fc":
            w = kaiming_normal((l["cout"], 1, 1, l["cin"]), l["cin"], seed, 100 + idx)
        else:
            continue
        b = normal((l["cout"],), 0.01, seed, 1000 + idx)
        out[l["name"]] = (w, b)
    return out


def network_input(batch: int, hw: int = 224, seed: int = 0) -> np.ndarray:
    """N(0,1) image batch, NHWC."""
    return normal((batch, hw, hw, 3), 1.0, seed, 7)


def bitwidths_fixed(layers):
    """Config 3: first conv and the linear layer 8-bit, everything else 4-bit (W, A)."""
    out = {}
    for l in layers:
        if l["op"] in ("conv", "fc"):
            b = 8 if l["name"] in ("conv1", "fc") else 4
            out[l["name"]] = (b, b)
    return out


def bitwidths_mixed(layers, seed: int = 0):
    """Config 4: (bitsW, bitsA) drawn uniformly from {4, 6, 8} per layer, in layer order."""
    g = _rng(seed, 11)
    out = {}
    for l in layers:
        if l["op"] in ("conv", "fc"):
            bw, ba = g.choice([4, 6, 8], size=2)
            out[l["name"]] = (int(bw), int(ba))
    return out
