"""GPU parity of the per-output-channel weight scales: dybit_quantize_rows against the oracle's row-wise
quantizer (scales and codes bit-exact) and dybit_gemm_pc / dybit_conv2d_pc against the oracle's products
with a vector of weight scales (GEMM tolerance; written-back codes bit-exact on the kernel's own fp32)."""
import numpy as np
import pytest
import torch

from oracle import dybit_ref as R
from paper_2302_12510_amd import binding as B
from paper_2302_12510_amd import synth
from gpu_util import dev, scalar, pack_rows_dev, assert_within
from test_gpu_gemm import force_kernel, random_codes  # noqa: F401  (fixture)
from test_gpu_writeback import check_codes

pytestmark = pytest.mark.gpu

FORMATS = [(b, s) for b in (2, 4, 6, 8) for s in (True, False)]


@pytest.mark.parametrize("fmt", FORMATS)
@pytest.mark.parametrize("shape", [(1, 8), (5, 64), (70, 576), (3, 1000), (256, 4608)])
def test_quantize_rows(fmt, shape):
    rows, cols = shape
    w = synth.laplace(shape, 0.02, seed=rows + fmt[0]) * np.logspace(-2, 2, rows, dtype=np.float32)[:, None]
    if rows > 2:
        w[2] = 0.0                                              # an all-zero row: scale 1, codes 0
    w = w.astype(np.float32)
    s, q = B.dybit_quantize_rows(dev(w), *fmt)
    torch.cuda.synchronize()
    want_s, want_q = R.quantize_rows(w, *fmt)
    assert np.array_equal(s.cpu().numpy(), want_s)
    assert np.array_equal(q.cpu().numpy(), R.pack_rows(want_q, fmt[0]))
    assert B.dybit_get_last_async_error() == B.OK


def test_quantize_rows_edge_cases():
    s, q = B.dybit_quantize_rows(torch.empty((0, 16), device="cuda"), 4, True)
    assert s.numel() == 0 and q.numel() == 0
    w = np.ones((2, 8), dtype=np.float32)
    w[1, 3] = np.inf                                            # an infinite maximum: flag, no codes for that row
    q0 = B.dybit_quantize_rows(dev(w), 8, True)[1]
    assert B.dybit_get_last_async_error() == B.ERR_BAD_SCALE
    assert np.array_equal(q0[0].cpu().numpy(), np.full(8, 127, dtype=np.uint8))


@pytest.mark.parametrize("force_kernel", ["large", "mid1", "mid2", "mid64", "ws", "general"], indirect=True)
@pytest.mark.parametrize("a_fmt", [(8, True), (4, False)])
@pytest.mark.parametrize("with_codes", [False, True])
def test_gemm_per_channel(force_kernel, a_fmt, with_codes):
    rng = np.random.default_rng(61 + a_fmt[0])
    w_fmt = (4, True)
    M, N, K = (290, 480, 128) if force_kernel != "ws" else (777, 96, 128)
    qa = random_codes(rng, (M, K), a_fmt)
    qw = random_codes(rng, (N, K), w_fmt)
    sw = np.logspace(-2, 1, N).astype(np.float32)
    rng.shuffle(sw)
    bias = rng.normal(0, 3, N).astype(np.float32)
    res = rng.normal(0, 30, (M, N)).astype(np.float32)
    want, den = R.gemm(qa, a_fmt, 0.37, qw, w_fmt, sw, bias, True, res)
    mx = torch.zeros(1, dtype=torch.float32, device="cuda")
    c_fmt = (8, False) if with_codes else None
    c_scale = np.float32(np.abs(want).max() / R.vmax(8, False))
    c, codes = B.dybit_gemm_pc(M, N, K, pack_rows_dev(qa, a_fmt[0]), a_fmt, scalar(0.37), pack_rows_dev(qw, 4), w_fmt, dev(sw),
                               dev(bias), dev(res), True, mx, c_fmt, scalar(c_scale) if with_codes else None)
    torch.cuda.synchronize()
    c32 = c.cpu().numpy()
    assert_within(c32, want, den, shortcut=True)
    assert mx.item() == np.abs(c32).max()
    if with_codes:
        check_codes(codes, c32, c_scale, c_fmt)
    else:
        assert codes is None


@pytest.mark.parametrize("force_kernel", ["mid1", "mid64", "ws", "general"], indirect=True)
def test_conv2d_per_channel(force_kernel):
    rng = np.random.default_rng(67)
    x_fmt, w_fmt = (4, False), (4, True)
    Cout = 96
    qx = random_codes(rng, (2, 9, 10, 64), x_fmt)
    qw = random_codes(rng, (Cout, 3, 3, 64), w_fmt)
    sw = rng.uniform(0.001, 0.5, Cout).astype(np.float32)
    bias = rng.normal(0, 1, Cout).astype(np.float32)
    want, den = R.conv2d(qx, x_fmt, 0.3, qw, w_fmt, sw, 1, 1, bias, True)
    y, _ = B.dybit_conv2d_pc(2, 9, 10, 64, Cout, 3, 3, 1, 1, pack_rows_dev(qx.reshape(-1, 64), 4), x_fmt, scalar(0.3),
                             pack_rows_dev(qw.reshape(-1, 64), 4), w_fmt, dev(sw), dev(bias), None, True)
    torch.cuda.synchronize()
    assert_within(y.cpu().numpy(), want, den)


def test_per_channel_scales_lower_the_weight_error():
    """Rows whose ranges span a factor of 30: one scale for the tensor leaves the small rows with few
    codes; a scale per row does not (Eq. 2 of the decoded weights against the originals, via the oracle:
    0.14 against 0.22 -- the format's own exponent already absorbs part of the spread)."""
    w = (synth.laplace((64, 256), 0.02, seed=5) * np.logspace(-1.5, 0, 64, dtype=np.float32)[:, None]).astype(np.float32)
    wd = dev(w)
    s, q = B.dybit_quantize_rows(wd, 4, True)
    w_rows = np.stack([R.dequantize(R.unpack(q[i].cpu().numpy(), 256, 4), s[i].item(), 4, True) for i in range(64)])
    st = B.dybit_absmax_scale(wd.reshape(-1), 4, True)
    w_tensor = R.dequantize(R.unpack(B.dybit_quantize(wd.reshape(-1), st, 4, True).cpu().numpy(), w.size, 4), st.item(), 4, True)
    assert R.rmse(w, w_rows) < 0.75 * R.rmse(w, w_tensor.reshape(w.shape))


def test_network_with_per_channel_weight_scales():
    """A small residual network with one weight scale per output channel: every layer's weight scales and
    codes equal the oracle's row-wise quantizer on the padded filter matrix, every layer's output is within
    tolerance of the oracle's convolution with that vector of scales on the GPU's own input codes, and the
    fused write-back chain reproduces the dynamic chain's logits on the calibration input."""
    from paper_2302_12510_amd.network import DybitNetwork
    layers = [
        {"name": "c1", "op": "conv", "src": "input", "cin": 3, "cout": 64, "k": 3, "stride": 1, "pad": 1, "relu": True},
        {"name": "c2", "op": "conv", "src": "c1", "cin": 64, "cout": 64, "k": 3, "stride": 1, "pad": 1, "relu": True},
        {"name": "c3", "op": "conv", "src": "c2", "cin": 64, "cout": 64, "k": 3, "stride": 1, "pad": 1, "relu": True, "add": "c1"},
        {"name": "c4", "op": "conv", "src": "c3", "cin": 64, "cout": 128, "k": 1, "stride": 2, "pad": 0, "relu": False},
    ]
    weights = synth.network_weights(layers, seed=4)
    for name, (w, b) in weights.items():                          # channels of different range
        w *= np.logspace(-1, 0.5, w.shape[0], dtype=np.float32)[:, None, None, None]
    bits = {"c1": (8, 8), "c2": (4, 4), "c3": (4, 8), "c4": (8, 4)}
    net = DybitNetwork(layers, weights, bits, per_channel=True)
    x = dev(synth.network_input(2, 24, seed=4))
    recs = {}
    out = net.forward(x, record=lambda n, r: recs.__setitem__(n, r))
    torch.cuda.synchronize()
    for l in layers:
        name, rec = l["name"], recs[l["name"]]
        w, bias = weights[name]
        cout, k, kw, cin = w.shape
        C = rec["x"].shape[-1]
        wp = np.zeros((cout, rec["k"], rec["kw"], C), dtype=np.float32)
        wp[:, :k, :kw, :cin] = w
        sw, qw = R.quantize_rows(wp.reshape(cout, -1), *rec["w_fmt"])
        assert np.array_equal(rec["w_scale"].cpu().numpy(), sw), name
        assert np.array_equal(rec["w_codes"].cpu().numpy(), R.pack_rows(qw, rec["w_fmt"][0])), name
        xs = rec["x"].cpu().numpy()
        qx = R.unpack(rec["a_codes"].cpu().numpy(), xs.size, rec["a_fmt"][0]).reshape(xs.shape)
        shortcut = None if rec["shortcut"] is None else rec["shortcut"].cpu().numpy()
        want, den = R.conv2d(qx, rec["a_fmt"], rec["a_scale"].item(), qw.reshape(wp.shape), rec["w_fmt"], sw,
                             rec["stride"], rec["pad"], bias, rec["relu"], shortcut)
        assert_within(rec["y"].cpu().numpy(), want, den, shortcut=shortcut is not None)
    net.calibrate(x)
    fused = net.forward(x, static=True)
    assert torch.equal(fused, out)
    assert B.dybit_get_last_async_error() == B.OK
