"""GPU parity of the fused write-back (dybit_gemm_wb / dybit_conv2d_wb): the matrix-product epilogue
encodes its results as DyBit codes (Sec. III-B: intermediate results are quantized before they are
written back).

The decision "which code" is taken on the kernel's own fp32 result, so the check has two halves, both
against the oracle: the fp32 output is within the GEMM tolerance of the exact result, and the codes are
bit-exact the oracle's quantization of that fp32 output under the given scale."""
import numpy as np
import pytest
import torch

from oracle import dybit_ref as R
from paper_2302_12510_amd import binding as B
from gpu_util import dev, scalar, pack_rows_dev, assert_within
from test_gpu_gemm import force_kernel, random_codes  # noqa: F401  (fixture)

pytestmark = pytest.mark.gpu

OUT_FMTS = [(4, False), (4, True), (6, False), (6, True), (8, False), (8, True)]


def check_codes(codes_dev, c32: np.ndarray, c_scale, c_fmt):
    want = R.pack_rows(R.quantize(c32, np.float32(c_scale), *c_fmt).reshape(c32.shape), c_fmt[0])
    got = codes_dev.cpu().numpy().reshape(want.shape)
    bad = got != want
    assert not bad.any(), f"{bad.sum()} of {bad.size} packed bytes differ; first at {np.argwhere(bad)[0]}"


@pytest.mark.parametrize("force_kernel", ["large", "mid1", "mid2", "mid64", "general"], indirect=True)
@pytest.mark.parametrize("c_fmt", OUT_FMTS)
@pytest.mark.parametrize("a_fmt", [(8, True), (4, False), (2, False)])
def test_gemm_wb(force_kernel, c_fmt, a_fmt):
    """Ragged M, several column tiles, bias + shortcut, values from far below the smallest step up to
    saturation; both outputs, then codes only."""
    rng = np.random.default_rng(31 + c_fmt[0])
    w_fmt = (4, True)
    M, N, K = 290, 480, 128
    qa = random_codes(rng, (M, K), a_fmt)
    qw = random_codes(rng, (N, K), w_fmt)
    bias = rng.normal(0, 3, N).astype(np.float32)
    res = rng.normal(0, 30, (M, N)).astype(np.float32)
    relu = not c_fmt[1]
    want, den = R.gemm(qa, a_fmt, 0.37, qw, w_fmt, 0.011, bias, relu, res)
    c_scale = np.float32(0.6 * np.abs(want).max() / R.vmax(*c_fmt))          # the largest results saturate
    args = (M, N, K, pack_rows_dev(qa, a_fmt[0]), a_fmt, scalar(0.37), pack_rows_dev(qw, 4), w_fmt, scalar(0.011),
            c_fmt, scalar(c_scale))
    mx = torch.zeros(1, dtype=torch.float32, device="cuda")
    c, codes = B.dybit_gemm_wb(*args, dev(bias), dev(res), relu, mx)
    torch.cuda.synchronize()
    c32 = c.cpu().numpy()
    assert_within(c32, want, den, shortcut=True)
    check_codes(codes, c32, c_scale, c_fmt)
    assert mx.item() == np.abs(c32).max()
    none, codes_only = B.dybit_gemm_wb(*args, dev(bias), dev(res), relu, None, fp32=False)
    torch.cuda.synchronize()
    assert none is None and torch.equal(codes_only, codes)


@pytest.mark.parametrize("force_kernel", ["mid1", "general"], indirect=True)
@pytest.mark.parametrize("c_fmt", OUT_FMTS)
def test_gemm_wb_exact_ties_and_every_value(force_kernel, c_fmt):
    """One non-zero product per output, every 8-bit unsigned code times every 8-bit signed code, unit
    scales: the fp32 results are exact, thousands of them sit exactly on a decision point of the output
    format (ties go to the even code) and many lie beyond its range."""
    a_fmt, w_fmt = (8, False), (8, True)
    K = 64
    qa = np.zeros((256, K), dtype=np.uint8)
    qw = np.zeros((256, K), dtype=np.uint8)
    qa[:, 5] = np.arange(256)
    qw[:, 5] = np.arange(256)
    for c_scale in (1.0, 0.5, 0.046875):
        c, codes = B.dybit_gemm_wb(256, 256, K, pack_rows_dev(qa, 8), a_fmt, scalar(1.0), pack_rows_dev(qw, 8), w_fmt,
                                   scalar(1.0), c_fmt, scalar(c_scale))
        torch.cuda.synchronize()
        c32 = c.cpu().numpy()
        assert np.array_equal(c32, np.outer(R.codebook(*a_fmt), R.codebook(*w_fmt)).astype(np.float32))
        mids = R.midpoints(R.magnitude_bits(*c_fmt)) * c_scale
        assert np.isin(np.abs(c32), mids).sum() > 100            # the case is really there
        check_codes(codes, c32, c_scale, c_fmt)


@pytest.mark.parametrize("force_kernel", ["large", "large-f16", "mid1", "mid2", "mid64", "mid1-f16", "general"], indirect=True)
@pytest.mark.parametrize("y_fmt", [(4, False), (6, False), (8, True)])
def test_conv2d_wb(force_kernel, y_fmt):
    rng = np.random.default_rng(37)
    x_fmt, w_fmt = (4, False), (4, True)
    Cout = 96
    qx = random_codes(rng, (2, 9, 10, 64), x_fmt)
    qw = random_codes(rng, (Cout, 3, 3, 64), w_fmt)
    bias = rng.normal(0, 1, Cout).astype(np.float32)
    res = rng.normal(0, 20, (2, 9, 10, Cout)).astype(np.float32)
    relu = not y_fmt[1]
    want, den = R.conv2d(qx, x_fmt, 0.3, qw, w_fmt, 0.02, 1, 1, bias, relu, res)
    y_scale = np.float32(np.abs(want).max() / R.vmax(*y_fmt))
    y, codes = B.dybit_conv2d_wb(2, 9, 10, 64, Cout, 3, 3, 1, 1, pack_rows_dev(qx.reshape(-1, 64), 4), x_fmt, scalar(0.3),
                                 pack_rows_dev(qw.reshape(-1, 64), 4), w_fmt, scalar(0.02), y_fmt, scalar(y_scale),
                                 dev(bias), dev(res), relu)
    torch.cuda.synchronize()
    y32 = y.cpu().numpy()
    assert_within(y32, want, den, shortcut=True)
    check_codes(codes, y32.reshape(-1, Cout), y_scale, y_fmt)


@pytest.mark.parametrize("force_kernel", ["ws"], indirect=True)
@pytest.mark.parametrize("c_fmt", OUT_FMTS)
@pytest.mark.parametrize("N", [96, 320])
def test_gemm_wb_weight_stationary(force_kernel, c_fmt, N):
    """N = 320: five column groups of 64, each in a workgroup of its own."""
    rng = np.random.default_rng(47 + c_fmt[0])
    a_fmt, w_fmt = (8, False), (4, True)
    M, K = 777, 128
    qa = random_codes(rng, (M, K), a_fmt)
    qw = random_codes(rng, (N, K), w_fmt)
    bias = rng.normal(0, 3, N).astype(np.float32)
    res = rng.normal(0, 30, (M, N)).astype(np.float32)
    relu = not c_fmt[1]
    want, den = R.gemm(qa, a_fmt, 0.37, qw, w_fmt, 0.011, bias, relu, res)
    c_scale = np.float32(0.8 * np.abs(want).max() / R.vmax(*c_fmt))
    mx = torch.zeros(1, dtype=torch.float32, device="cuda")
    c, codes = B.dybit_gemm_wb(M, N, K, pack_rows_dev(qa, 8), a_fmt, scalar(0.37), pack_rows_dev(qw, 4), w_fmt, scalar(0.011),
                               c_fmt, scalar(c_scale), dev(bias), dev(res), relu, mx)
    torch.cuda.synchronize()
    c32 = c.cpu().numpy()
    assert_within(c32, want, den, shortcut=True)
    check_codes(codes, c32, c_scale, c_fmt)
    assert mx.item() == np.abs(c32).max()


def test_wb_codes_feed_the_next_product():
    """The packed codes are laid out as the activation operand of a following dybit_gemm."""
    rng = np.random.default_rng(41)
    a_fmt, w_fmt, c_fmt = (8, True), (4, True), (4, False)
    M, N, K, N2 = 130, 128, 64, 40
    qa = random_codes(rng, (M, K), a_fmt)
    qw = random_codes(rng, (N, K), w_fmt)
    qw2 = random_codes(rng, (N2, N), w_fmt)
    want1, _ = R.gemm(qa, a_fmt, 0.5, qw, w_fmt, 0.25, None, True)
    s1 = np.float32(np.abs(want1).max() / R.vmax(*c_fmt))
    c, codes = B.dybit_gemm_wb(M, N, K, pack_rows_dev(qa, 8), a_fmt, scalar(0.5), pack_rows_dev(qw, 4), w_fmt, scalar(0.25),
                               c_fmt, scalar(s1), None, None, True)
    out2 = B.dybit_gemm(M, N2, N, codes, c_fmt, scalar(s1), pack_rows_dev(qw2, 4), w_fmt, scalar(0.125))
    torch.cuda.synchronize()
    q1 = R.quantize(c.cpu().numpy(), s1, *c_fmt)
    want2, den2 = R.gemm(q1, c_fmt, s1, qw2, w_fmt, 0.125)
    assert_within(out2.cpu().numpy(), want2, den2)


@pytest.mark.parametrize("bad", [0.0, -1.0, float("inf"), float("nan"), 1e-38, 2.0 ** -101, 2.0 ** 101])
def test_wb_unusable_scale_writes_no_codes_and_sets_the_flag(bad):
    rng = np.random.default_rng(43)
    a_fmt, w_fmt, c_fmt = (4, False), (4, True), (8, False)
    M, N, K = 64, 64, 64
    qa = random_codes(rng, (M, K), a_fmt)
    qw = random_codes(rng, (N, K), w_fmt)
    assert B.dybit_get_last_async_error() == B.OK
    codes = torch.full((M, N), 0xA5, dtype=torch.uint8, device="cuda")
    c, _ = B.dybit_gemm_wb(M, N, K, pack_rows_dev(qa, 4), a_fmt, scalar(1.0), pack_rows_dev(qw, 4), w_fmt, scalar(1.0),
                           c_fmt, scalar(bad), codes_out=codes)
    assert B.dybit_get_last_async_error() == B.ERR_BAD_SCALE
    assert B.dybit_get_last_async_error() == B.OK
    assert bool((codes == 0xA5).all())
    want, den = R.gemm(qa, a_fmt, 1.0, qw, w_fmt, 1.0)
    assert_within(c.cpu().numpy(), want, den)


R_FMTS = [(4, False), (4, True), (6, False), (6, True), (8, False), (8, True)]


@pytest.mark.parametrize("force_kernel", ["large", "mid1", "mid2", "mid64", "general"], indirect=True)
@pytest.mark.parametrize("r_fmt", R_FMTS)
@pytest.mark.parametrize("a_fmt", [(8, True), (4, False)])
def test_gemm_wb_shortcut_as_codes(force_kernel, r_fmt, a_fmt):
    """The shortcut tensor given as DyBit codes (dybit_gemm_wb_rc): against the oracle with the decoded
    shortcut, and bit for bit the call that gets the same shortcut as the fp32 tensor dybit_dequantize
    writes.  Ragged M and N tiles, every code of the shortcut's format present."""
    rng = np.random.default_rng(53 + r_fmt[0])
    w_fmt, c_fmt = (4, True), (8, True)
    M, N, K = 290, 480, 128
    qa = random_codes(rng, (M, K), a_fmt)
    qw = random_codes(rng, (N, K), w_fmt)
    qr = rng.integers(0, 1 << r_fmt[0], (M, N)).astype(np.uint8)
    r_scale = np.float32(0.73)
    res = R.dequantize(qr, r_scale, *r_fmt)
    bias = rng.normal(0, 3, N).astype(np.float32)
    want, den = R.gemm(qa, a_fmt, 0.37, qw, w_fmt, 0.011, bias, True, res)
    c_scale = np.float32(0.6 * np.abs(want).max() / R.vmax(*c_fmt))
    args = (M, N, K, pack_rows_dev(qa, a_fmt[0]), a_fmt, scalar(0.37), pack_rows_dev(qw, 4), w_fmt, scalar(0.011),
            c_fmt, scalar(c_scale))
    mx = torch.zeros(1, dtype=torch.float32, device="cuda")
    c, codes = B.dybit_gemm_wb_rc(*args, pack_rows_dev(qr, r_fmt[0]), r_fmt, scalar(r_scale), dev(bias), True, mx)
    torch.cuda.synchronize()
    c32 = c.cpu().numpy()
    assert_within(c32, want, den, shortcut=True)
    check_codes(codes, c32, c_scale, c_fmt)
    assert mx.item() == np.abs(c32).max()
    c_ref, codes_ref = B.dybit_gemm_wb(*args, dev(bias), dev(res), True)
    none, codes_only = B.dybit_gemm_wb_rc(*args, pack_rows_dev(qr, r_fmt[0]), r_fmt, scalar(r_scale), dev(bias), True,
                                          None, fp32=False)
    torch.cuda.synchronize()
    assert torch.equal(c, c_ref) and torch.equal(codes, codes_ref)
    assert none is None and torch.equal(codes_only, codes)


@pytest.mark.parametrize("force_kernel", ["ws"], indirect=True)
@pytest.mark.parametrize("r_fmt", R_FMTS)
@pytest.mark.parametrize("N", [96, 320])
def test_gemm_wb_shortcut_as_codes_weight_stationary(force_kernel, r_fmt, N):
    rng = np.random.default_rng(59 + r_fmt[0])
    a_fmt, w_fmt, c_fmt = (8, False), (4, True), (4, False)
    M, K = 777, 128
    qa = random_codes(rng, (M, K), a_fmt)
    qw = random_codes(rng, (N, K), w_fmt)
    qr = rng.integers(0, 1 << r_fmt[0], (M, N)).astype(np.uint8)
    res = R.dequantize(qr, np.float32(1.9), *r_fmt)
    want, den = R.gemm(qa, a_fmt, 0.37, qw, w_fmt, 0.011, None, True, res)
    c_scale = np.float32(0.8 * np.abs(want).max() / R.vmax(*c_fmt))
    c, codes = B.dybit_gemm_wb_rc(M, N, K, pack_rows_dev(qa, 8), a_fmt, scalar(0.37), pack_rows_dev(qw, 4), w_fmt, scalar(0.011),
                                  c_fmt, scalar(c_scale), pack_rows_dev(qr, r_fmt[0]), r_fmt, scalar(1.9), None, True)
    torch.cuda.synchronize()
    c32 = c.cpu().numpy()
    assert_within(c32, want, den, shortcut=True)
    check_codes(codes, c32, c_scale, c_fmt)


@pytest.mark.parametrize("force_kernel", ["large", "mid1", "mid2", "mid64", "mid1-f16", "general"], indirect=True)
@pytest.mark.parametrize("r_fmt", [(4, False), (6, True), (8, False)])
def test_conv2d_wb_shortcut_as_codes(force_kernel, r_fmt):
    rng = np.random.default_rng(61)
    x_fmt, w_fmt, y_fmt = (4, False), (4, True), (4, False)
    Cout = 96
    qx = random_codes(rng, (2, 9, 10, 64), x_fmt)
    qw = random_codes(rng, (Cout, 3, 3, 64), w_fmt)
    qr = rng.integers(0, 1 << r_fmt[0], (2, 9, 10, Cout)).astype(np.uint8)
    res = R.dequantize(qr, np.float32(2.5), *r_fmt)
    bias = rng.normal(0, 1, Cout).astype(np.float32)
    want, den = R.conv2d(qx, x_fmt, 0.3, qw, w_fmt, 0.02, 1, 1, bias, True, res)
    y_scale = np.float32(np.abs(want).max() / R.vmax(*y_fmt))
    y, codes = B.dybit_conv2d_wb_rc(2, 9, 10, 64, Cout, 3, 3, 1, 1, pack_rows_dev(qx.reshape(-1, 64), 4), x_fmt, scalar(0.3),
                                    pack_rows_dev(qw.reshape(-1, 64), 4), w_fmt, scalar(0.02), y_fmt, scalar(y_scale),
                                    pack_rows_dev(qr.reshape(-1, Cout), r_fmt[0]), r_fmt, scalar(2.5), dev(bias), True)
    torch.cuda.synchronize()
    y32 = y.cpu().numpy()
    assert_within(y32, want, den, shortcut=True)
    check_codes(codes, y32.reshape(-1, Cout), y_scale, y_fmt)


def test_wb_rc_argument_errors():
    a = torch.zeros(64 * 64, dtype=torch.uint8, device="cuda")
    one = scalar(1.0)
    args = (64, 64, 64, a, (8, False), one, a, (8, True), one, (8, False), one)
    with pytest.raises(B.DybitError) as e:
        B.dybit_gemm_wb_rc(*args, a, (2, False), one)
    assert e.value.status == B.ERR_UNSUPPORTED_BITS
    with pytest.raises(B.DybitError) as e:
        B.dybit_gemm_wb_rc(*args, None, (4, False), one)
    assert e.value.status == B.ERR_NULL
    with pytest.raises(B.DybitError) as e:
        B.dybit_gemm_wb_rc(*args, a, (4, False), None)
    assert e.value.status == B.ERR_NULL
