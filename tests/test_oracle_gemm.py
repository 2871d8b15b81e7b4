"""Pins for the oracle's GEMM and convolution.  CPU only."""
import numpy as np
import pytest
import torch

from oracle import c_ref, dybit_ref as R

PAIRS = [((4, False), (4, True)), ((8, True), (4, True)), ((6, False), (6, True)),
         ((8, False), (8, True)), ((4, True), (8, False)), ((2, True), (4, False))]


def _codes(rng, shape, fmt):
    return rng.integers(0, 1 << fmt[0], shape).astype(np.uint8)


@pytest.mark.parametrize("a_fmt,w_fmt", PAIRS)
def test_gemm_vs_exact_loops(a_fmt, w_fmt):
    rng = np.random.default_rng(1)
    a = _codes(rng, (5, 12), a_fmt)
    w = _codes(rng, (4, 12), w_fmt)
    bias = rng.normal(0, 1, 4).astype(np.float32)
    sa, sw = np.float32(0.37), np.float32(0.011)
    for b, relu in ((None, False), (bias, False), (bias, True)):
        c, d = R.gemm(a, a_fmt, sa, w, w_fmt, sw, b, relu)
        want = R.gemm_loops(a, a_fmt, sa, w, w_fmt, sw, b, relu)
        assert np.all(np.abs(c - want) <= 4e-16 * d)       # a few float64 roundings of the scaling
        cc, dc = c_ref.gemm(a, a_fmt, sa, w, w_fmt, sw, b, relu)
        assert np.array_equal(cc, c) and np.array_equal(dc, d)
        assert np.all(d >= np.abs(c) - 1e-12)


@pytest.mark.parametrize("a_fmt,w_fmt", PAIRS)
def test_gemm_vs_float64_matmul_of_dequantized(a_fmt, w_fmt):
    """Library routine: numpy float64 matmul over the decoded values."""
    rng = np.random.default_rng(2)
    a = _codes(rng, (33, 70), a_fmt)
    w = _codes(rng, (21, 70), w_fmt)
    sa, sw = np.float32(0.5), np.float32(0.125)            # exact scaling
    va = R.codebook(*a_fmt)[a] * float(sa)
    vw = R.codebook(*w_fmt)[w] * float(sw)
    c, d = R.gemm(a, a_fmt, sa, w, w_fmt, sw)
    assert np.array_equal(c, va @ vw.T)                    # all partial sums exact in float64
    assert np.array_equal(d, np.abs(va) @ np.abs(vw).T)


def test_gemm_identity_and_popcount():
    rng = np.random.default_rng(3)
    a_fmt, w_fmt = (8, True), (4, True)
    K = 16
    a = _codes(rng, (9, K), a_fmt)
    one_w = int(np.where(R.codebook(*w_fmt) == 1.0)[0][0])
    w = np.zeros((K, K), np.uint8)
    w[np.arange(K), np.arange(K)] = one_w                  # identity in code space
    sa, sw = np.float32(0.3), np.float32(2.0)
    c, _ = R.gemm(a, a_fmt, sa, w, w_fmt, sw)
    assert np.allclose(c, 2.0 * np.float64(sa) * R.codebook(*a_fmt)[a], rtol=1e-15)
    # codes restricted to {0, 1.0}: the sum is the popcount of the AND
    one_a = int(np.where(R.codebook(*a_fmt) == 1.0)[0][0])
    ba = rng.integers(0, 2, (7, 40)).astype(bool)
    bw = rng.integers(0, 2, (6, 40)).astype(bool)
    c, d = R.gemm(np.where(ba, one_a, 0), a_fmt, 1.0, np.where(bw, one_w, 0), w_fmt, 1.0)
    pop = (ba[:, None, :] & bw[None, :, :]).sum(-1)
    assert np.array_equal(c, pop) and np.array_equal(d, pop)


def test_gemm_k_split_additivity_and_transpose_guard():
    rng = np.random.default_rng(4)
    a_fmt, w_fmt = (6, False), (8, True)
    a = _codes(rng, (8, 48), a_fmt)
    w = _codes(rng, (5, 48), w_fmt)
    c, _ = R.gemm(a, a_fmt, 1.0, w, w_fmt, 1.0)
    c1, _ = R.gemm(a[:, :20], a_fmt, 1.0, w[:, :20], w_fmt, 1.0)
    c2, _ = R.gemm(a[:, 20:], a_fmt, 1.0, w[:, 20:], w_fmt, 1.0)
    assert np.array_equal(c, c1 + c2)
    assert c.shape == (8, 5)                               # [M][N], W given as [N][K]
    # a single non-zero product lands where it must
    a0 = np.zeros((3, 4), np.uint8); w0 = np.zeros((2, 4), np.uint8)
    a0[2, 1] = 1; w0[1, 1] = 1
    c0, _ = R.gemm(a0, (8, False), 1.0, w0, (8, False), 1.0)
    assert c0[2, 1] == (1 / 128) ** 2 and np.count_nonzero(c0) == 1


@pytest.mark.parametrize("stride,pad,k", [(1, 1, 3), (2, 3, 7), (2, 0, 1), (1, 0, 3)])
def test_conv2d_vs_torch_float64(stride, pad, k):
    """Library routine: torch conv2d in float64 over the decoded tensors."""
    rng = np.random.default_rng(5)
    x_fmt, w_fmt = (4, False), (4, True)
    B, H, W, Cin, Cout = 2, 9, 8, 6, 5
    x = _codes(rng, (B, H, W, Cin), x_fmt)
    w = _codes(rng, (Cout, k, k, Cin), w_fmt)
    bias = rng.normal(0, 1, Cout).astype(np.float32)
    sx, sw = np.float32(0.25), np.float32(0.5)
    y, d = R.conv2d(x, x_fmt, sx, w, w_fmt, sw, stride, pad, bias, relu=True)
    vx = torch.from_numpy(R.codebook(*x_fmt)[x] * float(sx)).permute(0, 3, 1, 2)
    vw = torch.from_numpy(R.codebook(*w_fmt)[w] * float(sw)).permute(0, 3, 1, 2)
    want = torch.nn.functional.conv2d(vx, vw, torch.from_numpy(bias.astype(np.float64)),
                                      stride=stride, padding=pad).clamp_min(0).permute(0, 2, 3, 1).numpy()
    assert y.shape == want.shape
    assert np.allclose(y, want, rtol=1e-13, atol=1e-13)
    yc, dc = c_ref.conv2d(x, x_fmt, sx, w, w_fmt, sw, stride, pad, bias, relu=True)
    assert np.array_equal(yc, y) and np.array_equal(dc, d)
    # identity shortcut (the ResNet workloads): added before the ReLU; a sign error, an addition
    # after the ReLU or a transposed layout all change the result
    res = rng.normal(0, 1, want.shape).astype(np.float32)
    yr, dr = R.conv2d(x, x_fmt, sx, w, w_fmt, sw, stride, pad, bias, relu=True, residual=res)
    lin = torch.nn.functional.conv2d(vx, vw, torch.from_numpy(bias.astype(np.float64)),
                                     stride=stride, padding=pad).permute(0, 2, 3, 1).numpy()
    want_r = np.maximum(lin + res.astype(np.float64), 0.0)
    assert np.allclose(yr, want_r, rtol=1e-13, atol=1e-13)
    assert not np.allclose(yr, np.maximum(lin, 0.0) + res, atol=1e-6)       # not "ReLU, then add"
    y0, d0 = R.conv2d(x, x_fmt, sx, w, w_fmt, sw, stride, pad, bias, relu=False)
    assert np.array_equal(dr, d0)                                           # the shortcut stays out of the tolerance denominator
    yz, _ = R.conv2d(x, x_fmt, sx, w, w_fmt, sw, stride, pad, bias, relu=True, residual=np.zeros_like(res))
    assert np.array_equal(yz, y)


def test_c_gemm_matches_numpy_on_config1_shape():
    from paper_2302_12510_amd import synth
    cfg = synth.config1()
    a_fmt, w_fmt = (4, False), (4, True)
    sa = R.absmax_scale(cfg["A"], *a_fmt)
    sw = R.absmax_scale(cfg["W"], *w_fmt)
    qa = R.quantize(cfg["A"], sa, *a_fmt)
    qw = R.quantize(cfg["W"], sw, *w_fmt)
    c, d = R.gemm(qa, a_fmt, sa, qw, w_fmt, sw)
    cc, dc = c_ref.gemm(qa, a_fmt, sa, qw, w_fmt, sw)
    assert np.array_equal(c, cc) and np.array_equal(d, dc)
    # the quantized product tracks the float product (sanity of the whole chain)
    ref = cfg["A"].astype(np.float64) @ cfg["W"].astype(np.float64).T
    assert np.corrcoef(ref.ravel(), c.ravel())[0, 1] > 0.95


def test_per_channel_weight_scales_are_the_scalar_case_column_by_column():
    """A vector w_scale: column n of the result is the (pinned) scalar-scale product with sW[n]."""
    rng = np.random.default_rng(21)
    a_fmt, w_fmt = (8, True), (4, True)
    qa = rng.integers(0, 256, (7, 24)).astype(np.uint8)
    qw = rng.integers(0, 16, (5, 24)).astype(np.uint8)
    sw = rng.uniform(0.01, 2.0, 5).astype(np.float32)
    bias = rng.normal(0, 1, 5).astype(np.float32)
    res = rng.normal(0, 1, (7, 5)).astype(np.float32)
    c, d = R.gemm(qa, a_fmt, 0.3, qw, w_fmt, sw, bias, True, res)
    for n in range(5):
        cn, dn = R.gemm(qa, a_fmt, 0.3, qw[n:n + 1], w_fmt, sw[n], bias[n:n + 1], True, res[:, n:n + 1])
        assert np.array_equal(c[:, n:n + 1], cn) and np.array_equal(d[:, n:n + 1], dn)
    with pytest.raises(ValueError):
        R.gemm(qa, a_fmt, 0.3, qw, w_fmt, sw[:3])
    # convolution: the same through im2col
    qx = rng.integers(0, 16, (1, 5, 6, 4)).astype(np.uint8)
    qf = rng.integers(0, 16, (3, 3, 3, 4)).astype(np.uint8)
    y, _ = R.conv2d(qx, (4, False), 0.5, qf, (4, True), sw[:3], 1, 1)
    for n in range(3):
        yn, _ = R.conv2d(qx, (4, False), 0.5, qf[n:n + 1], (4, True), sw[n], 1, 1)
        assert np.array_equal(y[..., n:n + 1], yn)


def test_quantize_rows_is_row_by_row():
    rng = np.random.default_rng(22)
    w = rng.laplace(0, 0.02, (6, 40)).astype(np.float32) * rng.uniform(0.1, 10, (6, 1)).astype(np.float32)
    w[3] = 0.0
    s, q = R.quantize_rows(w, 4, True)
    assert s.dtype == np.float32 and s.shape == (6,) and q.shape == (6, 40)
    for i in range(6):
        assert s[i] == R.absmax_scale(w[i], 4, True)
        assert np.array_equal(q[i], R.quantize(w[i], s[i], 4, True))
    assert s[3] == 1.0 and not q[3].any()
    # every row uses the whole code range: its largest magnitude is the all-ones code
    assert all((q[i] & 7).max() == 7 for i in (0, 1, 2, 4, 5))


@pytest.mark.parametrize("stride,pad,kh,kw", [(1, 1, 3, 3), (2, 1, 3, 3), (1, 0, 1, 1), (2, 2, 5, 3), (1, 2, 3, 5)])
def test_dwconv2d_pins(stride, pad, kh, kw):
    """Depthwise convolution against (a) torch's grouped conv2d in float64 over the decoded tensors and
    (b) the dense oracle convolution with a filter that is zero wherever the two channels differ."""
    rng = np.random.default_rng(31 + kh)
    x_fmt, w_fmt = (4, False), (8, True)
    B, H, W, C = 2, 9, 7, 6
    x = _codes(rng, (B, H, W, C), x_fmt)
    w = _codes(rng, (kh, kw, C), w_fmt)
    bias = rng.normal(0, 1, C).astype(np.float32)
    sx, sw = np.float32(0.25), np.float32(0.5)
    y, d = R.dwconv2d(x, x_fmt, sx, w, w_fmt, sw, stride, pad, bias, relu=True)
    vx = torch.from_numpy(R.codebook(*x_fmt)[x] * float(sx)).permute(0, 3, 1, 2)
    vw = torch.from_numpy(R.codebook(*w_fmt)[w] * float(sw)).permute(2, 0, 1).unsqueeze(1)      # [C][1][kh][kw]
    want = torch.nn.functional.conv2d(vx, vw, torch.from_numpy(bias.astype(np.float64)), stride=stride,
                                      padding=pad, groups=C).clamp_min(0).permute(0, 2, 3, 1).numpy()
    assert y.shape == want.shape
    assert np.allclose(y, want, rtol=1e-13, atol=1e-13)
    dense = np.zeros((C, kh, kw, C), dtype=np.uint8)
    for c in range(C):
        dense[c, :, :, c] = w[:, :, c]
    y2, d2 = R.conv2d(x, x_fmt, sx, dense, w_fmt, sw, stride, pad, bias, relu=True)
    assert np.array_equal(y, y2) and np.array_equal(d, d2)
    # one non-zero input and one non-zero tap: the product lands at the pixel the geometry says, in its own channel
    x1 = np.zeros((1, 6, 6, 3), np.uint8); w1 = np.zeros((3, 3, 3), np.uint8)
    x1[0, 2, 3, 1] = 8; w1[0, 2, 1] = 8                           # value 1 in both 4-bit unsigned formats
    y1, _ = R.dwconv2d(x1, (4, False), 1.0, w1, (4, False), 1.0, 1, 1)
    assert np.count_nonzero(y1) == 1 and y1[0, 3, 2, 1] == 1.0    # ho = hi + pad - r = 2 + 1 - 0, wo = 3 + 1 - 2
