"""GPU parity of dybit_rmse (Sec. III-C, Eq. 2) against the oracle, and of the search driver's tables.

Tolerance.  The kernel forms each difference x - x_hat with one float rounding (relative 2^-24);
squares and sums are in double.  An element within float rounding (2^-23) of a decision point may land
on the other neighbour: its error then changes by up to 2^-15 of itself, but only about one element in
2^16 is that close, so the sum moves by 2^-31.  The ratio under the root is within 2^-23 of the
oracle's and the root halves that: 1e-6 relative leaves more than a factor of ten."""
import numpy as np
import pytest
import torch

from oracle import dybit_ref as R
from paper_2302_12510_amd import binding as B
from paper_2302_12510_amd import synth
from gpu_util import dev, scalar

pytestmark = pytest.mark.gpu

FMTS = [(b, s) for b in (2, 4, 6, 8) for s in (False, True)]
REL = 1e-6


def tensor(kind: str, n: int, seed: int) -> np.ndarray:
    """The value distributions of the workloads: weights (Laplace), network input / pre-activation
    (normal with outliers), post-ReLU activations (half-normal with exact zeros), shifted mean."""
    if kind == "laplace":
        return synth.laplace((n,), 0.02, seed=seed)
    if kind == "outliers":
        return synth.normal_with_outliers((n,), seed=seed)
    if kind == "relu":
        return np.maximum(synth.normal((n,), 1.0, seed=seed), 0.0).astype(np.float32)
    if kind == "shifted":
        return (synth.normal((n,), 1.0, seed=seed) + np.float32(40.0)).astype(np.float32)
    raise ValueError(kind)


def check(x: np.ndarray, s, fmt):
    out = B.dybit_rmse(dev(x), scalar(s), *fmt)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    x64 = x.astype(np.float64)
    want = R.quantization_rmse(x, s, *fmt)
    assert got[0] == pytest.approx(want, rel=REL), (fmt, x.size)
    assert got[1] == pytest.approx(want ** 2 * x64.var() * x.size, rel=4 * REL)
    assert got[2] == pytest.approx(x64.sum(), rel=1e-12, abs=1e-9 * np.abs(x64).sum())
    assert got[3] == pytest.approx((x64 * x64).sum(), rel=1e-12)


@pytest.mark.parametrize("fmt", FMTS)
@pytest.mark.parametrize("kind", ["laplace", "outliers", "relu", "shifted"])
def test_rmse_matches_oracle(fmt, kind):
    n = (1 << 18) + 4 * 256 * 3 + 7                      # several grid strides, a ragged block and a tail
    x = tensor(kind, n, seed=7)
    check(x, R.absmax_scale(x, *fmt), fmt)
    check(x, np.float32(0.37) * R.absmax_scale(x, *fmt), fmt)        # the largest values saturate


@pytest.mark.parametrize("n", [2, 3, 4, 5, 7, 255, 1024, 1025, 4099, (1 << 21) + 1])
def test_rmse_sizes(n):
    x = tensor("outliers", n, seed=n)
    for fmt in ((4, True), (8, False)):
        check(x, R.absmax_scale(x, *fmt), fmt)


def test_rmse_small_and_large_scales():
    x = tensor("outliers", 5000, seed=3)
    for e in (-90, -30, 30, 90):
        f = np.float32(2.0 ** e)
        check((x * f).astype(np.float32), R.absmax_scale(x, 8, True) * f, (8, True))


def test_rmse_zero_on_representable_values():
    for fmt in FMTS:
        cb = R.codebook(*fmt).astype(np.float32)
        x = np.tile(np.float32(0.75) * cb, 33)
        out = B.dybit_rmse(dev(x), scalar(0.75), *fmt)
        assert out[0].item() == 0.0 and out[1].item() == 0.0


def test_rmse_degenerate_inputs():
    one = B.dybit_rmse(dev(np.array([0.3], dtype=np.float32)), scalar(1.0), 4, True)     # sigma = 0
    assert not np.isfinite(one[0].item())
    x = tensor("outliers", 1000, seed=1)
    x[17] = np.nan
    assert np.isnan(B.dybit_rmse(dev(x), scalar(1.0), 8, True)[0].item())
    assert B.dybit_get_last_async_error() == B.OK


@pytest.mark.parametrize("bad", [0.0, -1.0, float("inf"), float("nan"), 1e-38, 2.0 ** -101, 2.0 ** 101])
def test_rmse_unusable_scale(bad):
    x = tensor("outliers", 3000, seed=2)
    assert B.dybit_get_last_async_error() == B.OK
    out = B.dybit_rmse(dev(x), scalar(bad), 4, True)
    assert B.dybit_get_last_async_error() == B.ERR_BAD_SCALE
    assert np.isnan(out[0].item())
    assert B.dybit_get_last_async_error() == B.OK


def test_rmse_full_size_in_the_benchmark_configuration():
    """2^28 elements (the size the benchmark times): 256 copies of one block of 2^20 have the block's
    mean, variance and mean squared error, so the oracle's value for the block is the expected result."""
    block = tensor("outliers", 1 << 20, seed=11)
    xd = dev(block).repeat(256)
    assert xd.numel() == 1 << 28
    for fmt in ((4, True), (8, True), (2, False)):
        s = R.absmax_scale(block, *fmt)
        out = B.dybit_rmse(xd, scalar(s), *fmt)
        torch.cuda.synchronize()
        assert out[0].item() == pytest.approx(R.quantization_rmse(block, s, *fmt), rel=REL)
        assert out[2].item() == pytest.approx(256 * block.astype(np.float64).sum(), rel=1e-10, abs=1e-6)


def test_search_driver_on_a_small_network():
    """measure_tables on a three-layer network: its error tables equal the oracle's Eq. 2 on the same
    tensors, its latencies are positive, and the widths it finds are those the search oracle finds on
    the measured tables; the network with those widths runs."""
    from oracle import search_ref as S
    from paper_2302_12510_amd import search as drv
    from paper_2302_12510_amd.network import DybitNetwork

    layers = [
        {"name": "c1", "op": "conv", "src": "input", "cin": 3, "cout": 64, "k": 3, "stride": 1, "pad": 1, "relu": True},
        {"name": "c2", "op": "conv", "src": "c1", "cin": 64, "cout": 64, "k": 3, "stride": 2, "pad": 1, "relu": True},
        {"name": "c3", "op": "conv", "src": "c2", "cin": 64, "cout": 128, "k": 1, "stride": 1, "pad": 0, "relu": False},
    ]
    weights = synth.network_weights(layers, seed=3)
    x = dev(synth.network_input(4, 32, seed=3))
    tables = drv.measure_tables(layers, weights, x, steps=2, warmup=1)
    assert tables["names"] == ["c1", "c2", "c3"]
    assert (tables["lat"] > 0).all()
    for i, name in enumerate(tables["names"]):
        w = weights[name][0].reshape(-1)
        for j, bits in enumerate((8, 4, 2)):
            assert tables["rmse_w"][i, j] == pytest.approx(R.quantization_rmse(w, R.absmax_scale(w, bits, True), bits, True), rel=REL)
    x0 = x.cpu().numpy().reshape(-1)
    for j, bits in enumerate((8, 4, 2)):
        assert tables["rmse_a"][0, j] == pytest.approx(R.quantization_rmse(x0, R.absmax_scale(x0, bits, True), bits, True), rel=REL)
    assert (np.diff(tables["rmse_w"], axis=1) > 0).all() and (np.diff(tables["rmse_a"], axis=1) > 0).all()
    for strategy, constraint in (("speedup", 1.05), ("rmse", 3.0)):
        widths, ratio, met = drv.search_bitwidths(tables, strategy, constraint, 2)
        w, a, r, m = S.search(tables["lat"].tolist(), tables["rmse_w"].tolist(), tables["rmse_a"].tolist(), strategy, constraint, 2)
        assert [widths[n] for n in tables["names"]] == list(zip(w, a)) and ratio == r and met == m
        out = DybitNetwork(layers, weights, widths).forward(x)
        assert torch.isfinite(out).all()
