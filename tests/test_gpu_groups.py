"""GPU parity of the rest of the survey's "next" row 4 against the oracle: grouped convolution, per-channel
scales of depthwise filters (dybit_quantize_cols, dybit_dwconv2d_wb), codes out of the depthwise epilogue,
and the straight-through gradient of the quantize-then-decode operator."""
import numpy as np
import pytest
import torch

from oracle import dybit_ref as R
from paper_2302_12510_amd import binding as B
from gpu_util import dev, scalar, pack_rows_dev, assert_within
from test_gpu_gemm import random_codes

pytestmark = pytest.mark.gpu
FORMATS = [(b, s) for b in (2, 4, 6, 8) for s in (True, False)]


# ---- grouped convolution ------------------------------------------------------------------------------
@pytest.mark.parametrize("x_fmt,w_fmt", [((4, False), (4, True)), ((8, True), (4, True)), ((8, False), (8, True)),
                                          ((6, False), (6, True)), ((2, True), (8, True))])
@pytest.mark.parametrize("groups,cin,cout", [(2, 128, 128), (4, 256, 64), (2, 96, 40), (3, 24, 9), (8, 64, 64), (1, 64, 70)])
@pytest.mark.parametrize("geom", [(3, 1, 1), (1, 1, 0), (3, 2, 1)])
def test_group_conv_matches_oracle(x_fmt, w_fmt, groups, cin, cout, geom):
    """Groups of 64 / 128 channels (the tiled kernels on a channel slice of every pixel), of 48 (sixteen-code
    vectors), of 8 (code by code); bias, shortcut, ReLU and the running maximum across the groups."""
    k, stride, pad = geom
    cg = cin // groups
    if (cg * x_fmt[0]) % 8 or (cg * w_fmt[0]) % 8:
        pytest.skip("a group must start on a byte")
    rng = np.random.default_rng(groups * 1000 + cin + k)
    Bn, H, W = 2, 9, 11
    qx = random_codes(rng, (Bn, H, W, cin), x_fmt)
    qw = random_codes(rng, (cout, k, k, cg), w_fmt)
    bias = rng.normal(0, 1, cout).astype(np.float32)
    Ho, Wo = (H + 2 * pad - k) // stride + 1, (W + 2 * pad - k) // stride + 1
    res = rng.normal(0, 5, (Bn, Ho, Wo, cout)).astype(np.float32)
    want, den = R.group_conv2d(qx, x_fmt, 0.21, qw, w_fmt, 0.05, stride, pad, groups, bias, True, res)
    mx = torch.zeros(1, dtype=torch.float32, device="cuda")
    y = B.dybit_group_conv2d(Bn, H, W, cin, cout, k, k, stride, pad, groups, pack_rows_dev(qx.reshape(-1, cin), x_fmt[0]), x_fmt,
                             scalar(0.21), pack_rows_dev(qw.reshape(-1, cg), w_fmt[0]), w_fmt, scalar(0.05), dev(bias), dev(res),
                             True, mx)
    torch.cuda.synchronize()
    got = y.cpu().numpy()
    assert got.shape == want.shape
    assert_within(got, want, den, shortcut=True)
    assert mx.item() == np.abs(got).max()


def test_group_conv_per_channel_scales_and_depthwise_case():
    """One weight scale per output channel; groups = C is the depthwise convolution on [C][kh][kw][1] filters."""
    rng = np.random.default_rng(77)
    x_fmt, w_fmt = (8, False), (8, True)
    Bn, H, W, C = 2, 7, 9, 16
    qx = random_codes(rng, (Bn, H, W, C), x_fmt)
    qw = random_codes(rng, (C, 3, 3, 1), w_fmt)
    sw = np.logspace(-2, 0, C).astype(np.float32)
    want, den = R.group_conv2d(qx, x_fmt, 0.4, qw, w_fmt, sw, 1, 1, C)
    wd, dd = R.dwconv2d(qx, x_fmt, 0.4, np.ascontiguousarray(qw[..., 0].transpose(1, 2, 0)), w_fmt, sw, 1, 1)
    assert np.array_equal(want, wd)
    y = B.dybit_group_conv2d(Bn, H, W, C, C, 3, 3, 1, 1, C, pack_rows_dev(qx.reshape(-1, C), 8), x_fmt, scalar(0.4),
                             pack_rows_dev(qw.reshape(-1, 1), 8), w_fmt, dev(sw), per_channel=True)
    torch.cuda.synchronize()
    assert_within(y.cpu().numpy(), want, den)


def test_group_conv_refused_arguments():
    x = torch.zeros(64, dtype=torch.uint8, device="cuda")
    s = scalar(1.0)
    def call(cin, cout, groups, x_fmt=(4, False), w_fmt=(4, True)):
        return B.lib().dybit_group_conv2d(1, 2, 2, cin, cout, 1, 1, 1, 0, groups, x.data_ptr(), B.fmt(*x_fmt), s.data_ptr(),
                                          x.data_ptr(), B.fmt(*w_fmt), s.data_ptr(), 0, None, None, 0, x.data_ptr(), None, None)
    assert call(8, 8, 3) == B.ERR_INVALID_ARG             # groups does not divide the channels
    assert call(8, 6, 4) == B.ERR_INVALID_ARG
    assert call(8, 8, 0) == B.ERR_INVALID_ARG
    assert call(4, 4, 4) == B.ERR_ALIGNMENT               # one 4-bit channel per group: half a byte
    assert call(8, 8, 2, x_fmt=(3, True)) == B.ERR_UNSUPPORTED_BITS


# ---- per-channel scales of a depthwise filter, codes out of the depthwise epilogue ---------------------
@pytest.mark.parametrize("fmt", FORMATS)
@pytest.mark.parametrize("shape", [(9, 32), (1, 8), (25, 100), (49, 960)])
def test_quantize_cols(fmt, shape):
    rows, cols = shape
    rng = np.random.default_rng(rows + cols + fmt[0])
    x = (rng.laplace(0, 1, shape) * np.logspace(-3, 1, cols)).astype(np.float32)
    x[:, cols // 2] = 0.0
    scales, codes = B.dybit_quantize_cols(dev(x), *fmt)
    torch.cuda.synchronize()
    ws, wq = R.quantize_cols(x, *fmt)
    assert np.array_equal(scales.cpu().numpy(), ws)
    assert np.array_equal(codes.cpu().numpy(), R.pack_rows(wq, fmt[0]))
    assert B.dybit_get_last_async_error() == B.OK


def test_quantize_cols_infinite_column_sets_the_flag():
    x = np.ones((4, 8), np.float32)
    x[2, 5] = np.inf
    scales, codes = B.dybit_quantize_cols(dev(x), 8, True)
    assert B.dybit_get_last_async_error() == B.ERR_BAD_SCALE
    q = codes.cpu().numpy()
    assert not q[:, 5].any() and np.all(q[:, 0] == 127)


@pytest.mark.parametrize("x_fmt,w_fmt", [((4, False), (4, True)), ((8, False), (8, True)), ((8, True), (4, True)), ((2, False), (8, True))])
@pytest.mark.parametrize("y_fmt", [(4, False), (4, True), (8, False), (8, True)])
@pytest.mark.parametrize("geom", [(3, 3, 1, 1), (3, 3, 2, 1), (5, 3, 1, 2)])
def test_dwconv_wb_per_channel_and_codes(x_fmt, w_fmt, y_fmt, geom):
    """Per-channel filter scales from dybit_quantize_cols; the fp32 output within the product tolerance; the
    codes written by the epilogue bit-exact the oracle's quantization of that fp32 output (saturating scale);
    codes only equal to the codes of the two-output call."""
    kh, kw, stride, pad = geom
    rng = np.random.default_rng(kh * 10 + stride + y_fmt[0])
    Bn, H, W, C = 2, 19, 23, 48
    qx = random_codes(rng, (Bn, H, W, C), x_fmt)
    wf = (rng.normal(0, 1, (kh * kw, C)) * np.logspace(-2, 1, C)).astype(np.float32)
    sw_d, qw_d = B.dybit_quantize_cols(dev(wf), *w_fmt)
    sw, qw = R.quantize_cols(wf, *w_fmt)
    assert np.array_equal(sw_d.cpu().numpy(), sw)
    bias = rng.normal(0, 1, C).astype(np.float32)
    relu = not y_fmt[1]
    want, den = R.dwconv2d(qx, x_fmt, 0.3, qw.reshape(kh, kw, C), w_fmt, sw, stride, pad, bias, relu)
    y_scale = np.float32(0.6 * np.abs(want).max() / R.vmax(*y_fmt))
    mx = torch.zeros(1, dtype=torch.float32, device="cuda")
    args = (Bn, H, W, C, kh, kw, stride, pad, pack_rows_dev(qx.reshape(-1, C), x_fmt[0]), x_fmt, scalar(0.3), qw_d, w_fmt, sw_d,
            dev(bias), relu)
    y, codes = B.dybit_dwconv2d_wb(*args, mx, y_fmt, scalar(y_scale), per_channel=True)
    torch.cuda.synchronize()
    y32 = y.cpu().numpy()
    assert_within(y32, want, den)
    assert mx.item() == np.abs(y32).max()
    wantq = R.pack_rows(R.quantize(y32.reshape(-1, C), y_scale, *y_fmt), y_fmt[0])
    assert np.array_equal(codes.cpu().numpy().reshape(wantq.shape), wantq)
    none, codes_only = B.dybit_dwconv2d_wb(*args, None, y_fmt, scalar(y_scale), per_channel=True, fp32=False)
    torch.cuda.synchronize()
    assert none is None and torch.equal(codes_only, codes)
    assert B.dybit_get_last_async_error() == B.OK


def test_dwconv_wb_bad_scale_and_refusals():
    x_fmt = w_fmt = (4, True)
    qx = torch.zeros(2 * 8 * 8 * 32 // 2, dtype=torch.uint8, device="cuda")
    qw = torch.zeros(9 * 32 // 2, dtype=torch.uint8, device="cuda")
    args = (2, 8, 8, 32, 3, 3, 1, 1, qx, x_fmt, scalar(1.0), qw, w_fmt, scalar(1.0), None, False, None)
    y, codes = B.dybit_dwconv2d_wb(*args, (8, True), scalar(0.0))
    assert B.dybit_get_last_async_error() == B.ERR_BAD_SCALE
    with pytest.raises(B.DybitError) as e:
        B.dybit_dwconv2d_wb(*args, (6, True), scalar(1.0))
    assert e.value.status == B.ERR_UNSUPPORTED_BITS


# ---- straight-through gradient -----------------------------------------------------------------------
@pytest.mark.parametrize("fmt", FORMATS)
@pytest.mark.parametrize("n", [1, 3, 4, 1023, 4099, (1 << 20) + 5])
def test_fake_quant_bwd(fmt, n):
    rng = np.random.default_rng(n + fmt[0])
    s = np.float32(0.0123)
    hi = np.float32(s * np.float32(R.vmax(*fmt)))
    x = rng.normal(0, float(hi), n).astype(np.float32)
    special = np.array([hi, np.nextafter(hi, np.float32(np.inf)), -hi, np.nextafter(-hi, np.float32(-np.inf)), 0.0, -0.0,
                        np.nan, np.inf, -np.inf], dtype=np.float32)
    x[: min(n, special.size)] = special[: min(n, special.size)]
    g = rng.normal(0, 1, n).astype(np.float32)
    want = R.fake_quant_grad(x, g, s, *fmt)
    got = B.dybit_fake_quant_bwd(dev(x), dev(g), scalar(s), *fmt)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy().view(np.uint32), want.view(np.uint32))


def test_fake_quant_bwd_in_place_huge_scale_and_bad_scale():
    x = dev(np.array([1.0, 3e38, np.inf, -3e38, -np.inf, np.nan, 0.0, 5.0], np.float32))
    g = dev(np.arange(1, 9, dtype=np.float32))
    s = np.float32(2.0 ** 125)                                  # s * vmax overflows a float: every finite x is inside
    want = R.fake_quant_grad(x.cpu().numpy(), g.cpu().numpy(), s, 8, True)
    B.dybit_fake_quant_bwd(x, g, scalar(s), 8, True, out=g)
    assert np.array_equal(g.cpu().numpy(), want)
    assert B.dybit_get_last_async_error() == B.OK
    y = torch.full((8,), 7.0, device="cuda")
    B.dybit_fake_quant_bwd(x, g, scalar(-1.0), 8, True, out=y)
    assert B.dybit_get_last_async_error() == B.ERR_BAD_SCALE
    assert bool((y == 7.0).all())
