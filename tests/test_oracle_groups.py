"""Pins for the oracle's grouped convolution, per-column (depthwise filter) scales and the
straight-through gradient of the quantize-then-decode operator.  CPU only."""
import numpy as np
import pytest
import torch

from oracle import dybit_ref as R


def _codes(rng, shape, fmt):
    return rng.integers(0, 1 << fmt[0], shape).astype(np.uint8)


@pytest.mark.parametrize("x_fmt,w_fmt", [((4, False), (4, True)), ((8, True), (6, True)), ((2, True), (8, True))])
@pytest.mark.parametrize("groups,cin,cout", [(1, 6, 4), (2, 6, 4), (3, 6, 9), (4, 8, 4), (6, 6, 6)])
@pytest.mark.parametrize("geom", [(3, 1, 1), (1, 2, 0), (3, 2, 1)])
def test_group_conv_vs_torch_float64(x_fmt, w_fmt, groups, cin, cout, geom):
    """Library routine: torch's grouped convolution in float64 on the decoded values.  A wrong channel
    slice, a wrong group of an output channel or a transposed filter changes the result."""
    k, stride, pad = geom
    rng = np.random.default_rng(groups * 100 + cin + k)
    x = _codes(rng, (2, 7, 6, cin), x_fmt)
    w = _codes(rng, (cout, k, k, cin // groups), w_fmt)
    bias = rng.normal(0, 1, cout).astype(np.float32)
    sx = np.float32(0.25)
    sw = np.float32(2.0) ** rng.integers(-3, 2, cout).astype(np.float32)          # exact scaling, one per output channel
    y, d = R.group_conv2d(x, x_fmt, sx, w, w_fmt, sw, stride, pad, groups, bias, relu=True)
    vx = torch.from_numpy(R.codebook(*x_fmt)[x] * float(sx)).permute(0, 3, 1, 2)
    vw = torch.from_numpy(R.codebook(*w_fmt)[w] * sw.astype(np.float64)[:, None, None, None]).permute(0, 3, 1, 2)
    want = torch.nn.functional.conv2d(vx, vw, torch.from_numpy(bias.astype(np.float64)), stride=stride, padding=pad,
                                      groups=groups).clamp_min(0).permute(0, 2, 3, 1).numpy()
    assert y.shape == want.shape
    assert np.allclose(y, want, rtol=1e-13, atol=1e-13)
    assert np.all(d >= np.abs(y) - 1e-12)


def test_group_conv_special_cases():
    """groups = 1 is the dense convolution; groups = C with one filter per channel is the depthwise
    convolution on the transposed filter layout; the shortcut is added per output channel."""
    rng = np.random.default_rng(5)
    x_fmt, w_fmt = (4, False), (4, True)
    x = _codes(rng, (2, 6, 5, 8), x_fmt)
    w = _codes(rng, (12, 3, 3, 8), w_fmt)
    bias = rng.normal(0, 1, 12).astype(np.float32)
    res = rng.normal(0, 1, (2, 6, 5, 12)).astype(np.float32)
    y1, d1 = R.group_conv2d(x, x_fmt, 0.3, w, w_fmt, 0.02, 1, 1, 1, bias, True, res)
    y0, d0 = R.conv2d(x, x_fmt, 0.3, w, w_fmt, 0.02, 1, 1, bias, True, res)
    assert np.array_equal(y1, y0) and np.array_equal(d1, d0)
    wd = _codes(rng, (8, 3, 3, 1), w_fmt)                                   # [C][kh][kw][1]
    yg, dg = R.group_conv2d(x, x_fmt, 0.3, wd, w_fmt, 0.02, 2, 1, 8, bias[:8], False)
    yd, dd = R.dwconv2d(x, x_fmt, 0.3, np.ascontiguousarray(wd[..., 0].transpose(1, 2, 0)), w_fmt, 0.02, 2, 1, bias[:8], False)
    assert np.array_equal(yg, yd) and np.array_equal(dg, dd)
    with pytest.raises(ValueError):
        R.group_conv2d(x, x_fmt, 0.3, w, w_fmt, 0.02, 1, 1, 3)


def test_dwconv_per_channel_scale_is_the_scalar_case_channel_by_channel():
    rng = np.random.default_rng(6)
    x_fmt, w_fmt = (8, False), (4, True)
    x = _codes(rng, (2, 7, 7, 5), x_fmt)
    w = _codes(rng, (3, 3, 5), w_fmt)
    sw = np.array([0.5, 0.01, 3.0, 0.125, 1.0], np.float32)
    bias = rng.normal(0, 1, 5).astype(np.float32)
    y, d = R.dwconv2d(x, x_fmt, 0.7, w, w_fmt, sw, 1, 1, bias, True)
    for c in range(5):
        yc, dc = R.dwconv2d(x[..., c:c + 1], x_fmt, 0.7, w[..., c:c + 1], w_fmt, sw[c], 1, 1, bias[c:c + 1], True)
        assert np.array_equal(y[..., c:c + 1], yc) and np.array_equal(d[..., c:c + 1], dc)


@pytest.mark.parametrize("fmt", [(4, True), (8, True), (6, False), (2, True)])
def test_quantize_cols_is_quantize_per_column(fmt):
    rng = np.random.default_rng(7)
    x = (rng.laplace(0, 1, (9, 6)) * np.logspace(-2, 1, 6)).astype(np.float32)
    x[:, 3] = 0.0                                                             # an all-zero channel: scale 1
    scales, codes = R.quantize_cols(x, *fmt)
    assert scales.dtype == np.float32 and codes.shape == x.shape
    for c in range(6):
        s = R.absmax_scale(x[:, c], *fmt)
        assert scales[c] == s
        assert np.array_equal(codes[:, c], R.quantize(x[:, c], s, *fmt))
    assert scales[3] == 1.0 and not codes[:, 3].any()


@pytest.mark.parametrize("fmt", [(4, True), (4, False), (8, True), (6, False)])
def test_fake_quant_grad_is_the_derivative_of_the_clamp(fmt):
    """The straight-through estimator differentiates x -> clamp(x, lo, hi).  Pins: torch's autograd
    of clamp (library routine), a central finite difference away from the two bounds, and the
    bounds themselves (included in the pass-through range)."""
    rng = np.random.default_rng(8)
    s = np.float32(0.37)
    hi = float(s) * R.vmax(*fmt)
    lo = -hi if fmt[1] else 0.0
    x = rng.normal(0, hi, 4000).astype(np.float32)
    x[:6] = [hi, np.nextafter(np.float32(hi), np.float32(np.inf)), lo, np.nextafter(np.float32(lo), np.float32(-np.inf)), 0.0, np.nan]
    g = rng.normal(0, 1, x.size).astype(np.float32)
    got = R.fake_quant_grad(x, g, s, *fmt)
    xt = torch.tensor(x[6:].astype(np.float64), requires_grad=True)
    torch.clamp(xt, lo, hi).backward(torch.from_numpy(g[6:].astype(np.float64)))
    assert np.array_equal(got[6:], xt.grad.numpy().astype(np.float32))
    h = 1e-3 * hi
    far = (np.abs(x[6:] - hi) > 2 * h) & (np.abs(x[6:] - lo) > 2 * h)
    xd = x[6:].astype(np.float64)
    fd = (np.clip(xd + h, lo, hi) - np.clip(xd - h, lo, hi)) / (2 * h)
    assert np.allclose(got[6:][far], (fd * g[6:])[far], rtol=0, atol=1e-6)
    assert got[0] == g[0] and got[1] == 0.0 and got[2] == g[2] and got[3] == 0.0 and got[4] == g[4] and got[5] == 0.0
    # the quantize-then-decode operator itself is flat beyond the range and follows x inside it
    inside = x[6:][(x[6:] > lo) & (x[6:] < hi)]
    fq = R.dequantize(R.quantize(inside, s, *fmt), s, *fmt)
    step = float(s) * np.max(np.diff(np.sort(np.unique(np.abs(R.codebook(*fmt))))))
    assert np.all(np.abs(fq - inside) <= step / 2 + 1e-6)
