"""GPU parity: dybit_gemm and dybit_conv2d against the CPU oracle.

Tolerance (the stated bar): |C_gpu - C_ref| <= 1e-5 * (sA sW sum_k|a w| + |bias|) per output,
with C_ref accumulated exactly.  Both sides consume the same codes, produced by the oracle."""
import numpy as np
import pytest
import torch

from oracle import dybit_ref as R
from paper_2302_12510_amd import binding as B
from paper_2302_12510_amd import synth
from gpu_util import dev, scalar, oracle_codes, pack_rows_dev, assert_within

pytestmark = pytest.mark.gpu

PAIRS = [((4, False), (4, True)), ((8, True), (4, True)), ((8, False), (8, True)), ((6, False), (6, True)),
         ((4, True), (8, False)), ((6, True), (4, True)), ((2, True), (4, False)), ((8, True), (2, True)),
         ((4, False), (6, True)), ((2, False), (2, True))]


def run_gemm(qa, a_fmt, sa, qw, w_fmt, sw, bias=None, relu=False, ldc=None):
    M, K = qa.shape
    N = qw.shape[0]
    out = None
    if ldc is not None:
        out = torch.full((M, ldc), -777.0, dtype=torch.float32, device="cuda")
    c = B.dybit_gemm(M, N, K, pack_rows_dev(qa, a_fmt[0]), a_fmt, scalar(sa),
                     pack_rows_dev(qw, w_fmt[0]), w_fmt, scalar(sw),
                     None if bias is None else dev(bias), relu, out=out, ldc=ldc)
    assert_forced_kernel_ran()
    torch.cuda.synchronize()
    return c.cpu().numpy()


def random_codes(rng, shape, fmt):
    return rng.integers(0, 1 << fmt[0], shape).astype(np.uint8)


def test_config1_small_gemm():
    cfg = synth.config1()
    a_fmt, w_fmt = (4, False), (4, True)
    sa, qa = oracle_codes(cfg["A"], a_fmt)
    sw, qw = oracle_codes(cfg["W"], w_fmt)
    got = run_gemm(qa, a_fmt, sa, qw, w_fmt, sw)
    want, den = R.gemm(qa, a_fmt, sa, qw, w_fmt, sw)
    assert_within(got, want, den)


@pytest.mark.parametrize("a_fmt,w_fmt", PAIRS)
@pytest.mark.parametrize("shape", [(130, 70, 80), (257, 129, 208), (64, 64, 256), (1, 1, 16), (5, 3, 48)])
def test_format_pairs_ragged_shapes(a_fmt, w_fmt, shape):
    M, N, K = shape
    rng = np.random.default_rng(M * 1000 + N)
    qa = random_codes(rng, (M, K), a_fmt)
    qw = random_codes(rng, (N, K), w_fmt)
    bias = rng.normal(0, 3, N).astype(np.float32)
    sa, sw = np.float32(0.37), np.float32(0.011)
    for b, relu in ((None, False), (bias, True)):
        got = run_gemm(qa, a_fmt, sa, qw, w_fmt, sw, b, relu)
        want, den = R.gemm(qa, a_fmt, sa, qw, w_fmt, sw, b, relu)
        assert_within(got, want, den)


@pytest.mark.parametrize("a_fmt,w_fmt,K", [((8, True), (8, False), 147), ((8, True), (4, True), 26),
                                            ((4, False), (4, True), 18), ((6, True), (6, False), 20),
                                            ((2, True), (8, True), 12), ((4, True), (6, True), 4)])
def test_k_not_a_multiple_of_16(a_fmt, w_fmt, K):
    rng = np.random.default_rng(K)
    M, N = 77, 45
    qa = random_codes(rng, (M, K), a_fmt)
    qw = random_codes(rng, (N, K), w_fmt)
    got = run_gemm(qa, a_fmt, 1.5, qw, w_fmt, 0.25)
    want, den = R.gemm(qa, a_fmt, 1.5, qw, w_fmt, 0.25)
    assert_within(got, want, den)


def test_single_product_lands_in_the_right_cell():
    """Catches a transposed operand or a permuted accumulator layout."""
    a_fmt, w_fmt = (8, False), (8, False)
    M, N, K = 96, 80, 32
    one = int(np.where(R.codebook(*a_fmt) == 1.0)[0][0])
    two = int(np.where(R.codebook(*a_fmt) == 2.0)[0][0])
    for (i, j, k) in [(0, 0, 0), (37, 5, 9), (95, 79, 31), (33, 64, 17), (70, 31, 8)]:
        qa = np.zeros((M, K), np.uint8); qw = np.zeros((N, K), np.uint8)
        qa[i, k] = one; qw[j, k] = two
        got = run_gemm(qa, a_fmt, 1.0, qw, w_fmt, 1.0)
        want = np.zeros((M, N)); want[i, j] = 2.0
        assert np.array_equal(got, want), (i, j, k)


def test_ldc_and_untouched_padding():
    a_fmt, w_fmt = (4, False), (4, True)
    rng = np.random.default_rng(9)
    qa = random_codes(rng, (50, 32), a_fmt); qw = random_codes(rng, (20, 32), w_fmt)
    got = run_gemm(qa, a_fmt, 1.0, qw, w_fmt, 1.0, ldc=24)
    want, den = R.gemm(qa, a_fmt, 1.0, qw, w_fmt, 1.0)
    assert_within(got[:, :20], want, den)
    assert np.all(got[:, 20:] == -777.0)


@pytest.mark.parametrize("a_fmt", [(4, False), (8, True)])
def test_ldc_and_untouched_padding_tiled_kernels(a_fmt):
    """The tiled kernels' epilogue (buffer stores) with a leading dimension larger than N and
    ragged last rows / columns: nothing outside the M x N block is written."""
    w_fmt = (4, True)
    rng = np.random.default_rng(10)
    M, N, K, ldc = 300, 70, 128, 96
    qa = random_codes(rng, (M, K), a_fmt); qw = random_codes(rng, (N, K), w_fmt)
    out = torch.full((M + 40, ldc), -777.0, dtype=torch.float32, device="cuda")
    B.dybit_gemm(M, N, K, pack_rows_dev(qa, a_fmt[0]), a_fmt, scalar(1.0), pack_rows_dev(qw, 4), w_fmt, scalar(1.0),
                 out=out, ldc=ldc)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    want, den = R.gemm(qa, a_fmt, 1.0, qw, w_fmt, 1.0)
    assert_within(got[:M, :N], want, den)
    assert np.all(got[:M, N:] == -777.0) and np.all(got[M:] == -777.0)


def test_k_zero_writes_bias():
    bias = np.arange(7, dtype=np.float32) - 3
    c = B.dybit_gemm(5, 7, 0, None, (4, True), scalar(1.0), None, (4, True), scalar(1.0), dev(bias), True)
    assert np.array_equal(c.cpu().numpy(), np.tile(np.maximum(bias, 0), (5, 1)))


def test_exact_accumulation_when_sums_are_small():
    """With short K every partial sum is a small multiple of the product unit, so the fp32
    accumulator holds the exact integer and the result equals the oracle's to the last bit
    of the final scaling."""
    a_fmt, w_fmt = (8, True), (4, True)
    rng = np.random.default_rng(21)
    qa = random_codes(rng, (200, 64), a_fmt); qw = random_codes(rng, (136, 64), w_fmt)
    got = run_gemm(qa, a_fmt, 1.0, qw, w_fmt, 1.0)
    want, _ = R.gemm(qa, a_fmt, 1.0, qw, w_fmt, 1.0)
    assert np.array_equal(got.astype(np.float64), want)


# ---- convolution ------------------------------------------------------------
def run_conv(qx, x_fmt, sx, qw, w_fmt, sw, stride, pad, bias=None, relu=False):
    Bn, H, W, Cin = qx.shape
    Cout, kh, kw, _ = qw.shape
    y = B.dybit_conv2d(Bn, H, W, Cin, Cout, kh, kw, stride, pad,
                       pack_rows_dev(qx.reshape(-1, Cin), x_fmt[0]), x_fmt, scalar(sx),
                       pack_rows_dev(qw.reshape(-1, Cin), w_fmt[0]), w_fmt, scalar(sw),
                       None if bias is None else dev(bias), relu)
    assert_forced_kernel_ran()
    torch.cuda.synchronize()
    return y.cpu().numpy()


@pytest.mark.parametrize("x_fmt,w_fmt,Cin", [((4, False), (4, True), 32), ((4, False), (4, True), 6),
                                              ((8, True), (8, True), 3), ((6, False), (6, True), 16),
                                              ((8, False), (4, True), 48), ((6, True), (8, True), 4),
                                              ((2, True), (4, True), 64)])
@pytest.mark.parametrize("geom", [(3, 1, 1), (7, 2, 3), (1, 2, 0), (3, 2, 1), (1, 1, 0)])
def test_conv_small(x_fmt, w_fmt, Cin, geom):
    k, stride, pad = geom
    rng = np.random.default_rng(Cin * 10 + k)
    Bn, H, W, Cout = 3, 13, 11, 37
    qx = random_codes(rng, (Bn, H, W, Cin), x_fmt)
    qw = random_codes(rng, (Cout, k, k, Cin), w_fmt)
    bias = rng.normal(0, 1, Cout).astype(np.float32)
    got = run_conv(qx, x_fmt, 0.21, qw, w_fmt, 0.05, stride, pad, bias, True)
    want, den = R.conv2d(qx, x_fmt, 0.21, qw, w_fmt, 0.05, stride, pad, bias, True)
    assert got.shape == want.shape
    assert_within(got, want, den)


@pytest.mark.parametrize("x_fmt,w_fmt,Cin,kw", [((8, True), (8, True), 4, 8), ((6, True), (4, True), 4, 8),
                                                 ((4, False), (4, True), 4, 4), ((2, True), (8, True), 4, 8),
                                                 ((8, False), (6, True), 8, 2), ((4, True), (2, True), 8, 6),
                                                 ((8, True), (4, True), 2, 8), ((4, False), (8, True), 2, 16),
                                                 ((8, False), (8, True), 1, 16), ((6, False), (6, True), 8, 4)])
@pytest.mark.parametrize("kh,stride,pad,shape", [(7, 2, 3, (3, 23, 21)), (3, 1, 1, (2, 9, 17)), (1, 1, 0, (1, 5, 19)),
                                                 (2, 3, 4, (2, 12, 16)), (5, 2, 8, (1, 7, 16)),
                                                 (8, 2, 3, (3, 23, 21)), (4, 1, 2, (2, 9, 27)), (6, 2, 5, (1, 30, 17))])
def test_conv_few_channels(x_fmt, w_fmt, Cin, kw, kh, stride, pad, shape):
    """Few input channels with kw * Cin a multiple of 16 (the first layer of an image network with its
    filter rows padded by zero taps): the general kernel fetches runs of neighbouring taps, and where a
    filter row is exactly 32 codes and the filter has an even number of rows the 128 x 128 kernel fetches
    whole filter rows.  Rectangular
    filters, taps left / right / above / below the image, runs that start at any byte (6-bit: three bytes
    per pixel), tensors whose size is not a multiple of four bytes, padding wider than the filter."""
    Bn, H, W = shape
    if W + 2 * pad < kw or H + 2 * pad < kh:
        pytest.skip("filter larger than the padded image")
    rng = np.random.default_rng(Cin * 100 + kw * 10 + kh)
    Cout = 19 if kh % 2 else 150                                  # two column tiles for the tiled kernel
    qx = random_codes(rng, (Bn, H, W, Cin), x_fmt)
    qw = random_codes(rng, (Cout, kh, kw, Cin), w_fmt)
    bias = rng.normal(0, 1, Cout).astype(np.float32)
    got = run_conv(qx, x_fmt, 0.21, qw, w_fmt, 0.05, stride, pad, bias, False)
    # which kernel took it: whole filter rows (aligned words: tensors of whole words only), else the general one
    by_rows = kw * Cin == 32 and kh % 2 == 0 and (Bn * H * W * Cin * x_fmt[0] // 8) % 4 == 0
    assert B.dybit_last_gemm_kernel() == ("f16_128_rows" if by_rows else "general")
    want, den = R.conv2d(qx, x_fmt, 0.21, qw, w_fmt, 0.05, stride, pad, bias, False)
    assert got.shape == want.shape
    assert_within(got, want, den)


def test_config2_conv_full_size():
    cfg = synth.config2()
    x_fmt, w_fmt = (4, False), (4, True)
    sx, qx = oracle_codes(cfg["X"], x_fmt)
    sw, qw = oracle_codes(cfg["Wt"], w_fmt)
    got = run_conv(qx, x_fmt, sx, qw, w_fmt, sw, 1, 1)
    want, den = R.conv2d(qx, x_fmt, sx, qw, w_fmt, sw, 1, 1)
    assert_within(got, want, den)


def test_config5a_shape_sampled_outputs():
    """The 8192^3 product at full size through the benchmark's entry point; the oracle
    evaluates a sample of rows and columns exactly."""
    size = 8192
    cfg = synth.config5a(size=size)
    a_fmt, w_fmt = (8, True), (4, True)
    sa, qa = oracle_codes(cfg["A"], a_fmt)
    sw, qw = oracle_codes(cfg["W"], w_fmt)
    c = B.dybit_gemm(size, size, size, pack_rows_dev(qa, 8), a_fmt, scalar(sa),
                     pack_rows_dev(qw, 4), w_fmt, scalar(sw))
    torch.cuda.synchronize()
    rng = np.random.default_rng(0)
    rows = np.unique(np.concatenate([[0, 127, 128, size - 1], rng.integers(0, size, 60)]))
    cols = np.unique(np.concatenate([[0, 127, 128, size - 1], rng.integers(0, size, 508)]))
    want, den = R.gemm(qa[rows], a_fmt, sa, qw[cols], w_fmt, sw)
    got = c[torch.from_numpy(rows).cuda()][:, torch.from_numpy(cols).cuda()].cpu().numpy()
    assert_within(got, want, den)


def test_8192_cubed_4bit_w_a_sampled_outputs():
    """The same 8192^3 product with 4-bit activations, as bench.py times it (fp8 matrix path,
    256 x 256 tiles); the oracle evaluates a sample of rows and columns exactly."""
    size = 8192
    cfg = synth.config5a(size=size)
    a_fmt, w_fmt = (4, True), (4, True)
    sa, qa = oracle_codes(cfg["A"], a_fmt)
    sw, qw = oracle_codes(cfg["W"], w_fmt)
    c = B.dybit_gemm(size, size, size, pack_rows_dev(qa, 4), a_fmt, scalar(sa),
                     pack_rows_dev(qw, 4), w_fmt, scalar(sw))
    torch.cuda.synchronize()
    rng = np.random.default_rng(1)
    rows = np.unique(np.concatenate([[0, 255, 256, size - 1], rng.integers(0, size, 60)]))
    cols = np.unique(np.concatenate([[0, 255, 256, size - 1], rng.integers(0, size, 508)]))
    want, den = R.gemm(qa[rows], a_fmt, sa, qw[cols], w_fmt, sw)
    got = c[torch.from_numpy(rows).cuda()][:, torch.from_numpy(cols).cuda()].cpu().numpy()
    assert_within(got, want, den)


# ---- tiled MFMA kernels (256 x 256 and 128 x 128 tiles, in-register decode) --------
TILED_PAIRS = [(a, w) for w in ((4, True), (8, True)) for a in ((4, True), (4, False), (8, True), (8, False))]
# pairs with a 6-bit operand (on the 256 x 256 fp16 kernel when K is a multiple of 128, else on the 128 x 128 one)
TILED_PAIRS += [(a, (6, True)) for a in ((4, False), (6, True), (6, False), (8, True))]
TILED_PAIRS += [((6, True), (4, True)), ((6, False), (4, True)), ((6, True), (8, True)), ((6, False), (8, True))]
# ... and the 2-bit formats of the {8, 4, 2} x {8, 4, 2} mode matrix
TILED_PAIRS += [((2, True), (2, True)), ((2, False), (2, True)), ((8, True), (2, True)), ((4, False), (2, True)),
                ((2, False), (4, True)), ((2, True), (8, True)), ((2, False), (6, True)), ((4, True), (2, True)),
                ((2, True), (4, True))]
# mid1 / mid2: the 128 x 128 kernel with one / two k-groups.  Two operands of 4 or 2 bits run on the fp8
# matrix path by default (256 x 256 tiles included); the "-f16" entries keep them on the fp16 kernels
# (and are skipped for other pairs, which are on the fp16 kernels anyway).
# mid64: the 64 x 64 tile of the fp8-path kernel (chosen by itself when 128 x 128 tiles are few).
KERNELS = ["large", "mid1", "mid2", "mid64", "large-f16", "mid1-f16", "mid2-f16"]


# kernels (binding.KERNEL_NAMES) that a forced family may legitimately run on, by matrix path
_FAMILY = {"large": ({"f16_256"}, {"f8_256"}), "mid1": ({"f16_128_kg1", "f16_128_rows"}, {"f8_128_kg1"}),
           "mid2": ({"f16_128_kg2", "f16_128_rows"}, {"f8_128_kg2"}), "mid": ({"f16_128_kg1", "f16_128_kg2", "f16_128_rows"}, set()),
           "mid64": (set(), {"f8_64"}), "ws": ({"f16_ws"}, {"f8_ws"}), "general": ({"general"}, {"general"})}
_expected_kernels = None


def assert_forced_kernel_ran():
    """The kernel the last matrix-product call launched is one the forced family allows."""
    if _expected_kernels is not None:
        ran = B.dybit_last_gemm_kernel()
        assert ran in _expected_kernels, f"forced {sorted(_expected_kernels)} but the call ran on {ran}"


@pytest.fixture
def force_kernel(request):
    """Forces a kernel family through dybit_set_option for one test and checks, after every run_gemm and at
    the end of the test, that the call really ran on it (dybit_last_gemm_kernel)."""
    global _expected_kernels
    name = request.param
    fmts = [request.getfixturevalue(k) for k in ("a_fmt", "w_fmt", "x_fmt") if k in request.fixturenames]
    low_pair = bool(fmts) and all(f[0] in (2, 4) for f in fmts)
    options = {}
    f16_only = name.endswith("-f16")
    if f16_only:
        if fmts and not low_pair:
            pytest.skip("only pairs of 4- and 2-bit formats have an fp8 path to switch off")
        options["gemm_mfma"] = "f16"
        name = name[:-4]
    family = name
    if name == "mid64":
        if fmts and not low_pair:
            pytest.skip("the 64 x 64 tile exists on the fp8 path only")
        options["mid_tile"] = "64"
        name = "mid"
    elif name.startswith("mid") and name != "mid":
        options["mid_kgroups"] = name[3:]
        options["mid_tile"] = "128"
        name = "mid"
    options["gemm_kernel"] = name
    f16_set, f8_set = _FAMILY[family]
    if family in ("ws", "general"):                         # one kernel for every pair
        _expected_kernels = f16_set | f8_set
    elif family == "large" and any(f[0] in (2, 6) for f in fmts) and (f16_only or not low_pair):
        # a 2- or 6-bit operand is on the 256 x 256 fp16 kernel only when K (Cin) is a multiple of 128; other shapes
        # go on to the 128 x 128 kernel (test_large_kernel_six_bit_operands pins the first case)
        _expected_kernels = f16_set | _FAMILY["mid"][0]
    elif f16_only or (fmts and not low_pair):
        _expected_kernels = set(f16_set)
    elif fmts:
        _expected_kernels = set(f8_set)
    else:                                                   # the test picks its own formats
        _expected_kernels = f16_set | f8_set
    for k, v in options.items():
        B.dybit_set_option(k, v)
    try:
        yield request.param
        assert_forced_kernel_ran()
    finally:
        _expected_kernels = None
        for k in options:
            B.dybit_set_option(k, "auto")


@pytest.mark.parametrize("force_kernel", KERNELS, indirect=True)
@pytest.mark.parametrize("a_fmt,w_fmt", TILED_PAIRS)
@pytest.mark.parametrize("shape", [(2100, 3900, 192), (256, 256, 64), (300, 520, 128), (1, 7, 64), (513, 255, 320)])
def test_tiled_kernels_ragged(force_kernel, a_fmt, w_fmt, shape):
    M, N, K = shape
    rng = np.random.default_rng(M + N + K)
    qa = random_codes(rng, (M, K), a_fmt)
    qw = random_codes(rng, (N, K), w_fmt)
    bias = rng.normal(0, 3, N).astype(np.float32)
    for b, relu in ((None, False), (bias, True)):
        got = run_gemm(qa, a_fmt, 0.37, qw, w_fmt, 0.011, b, relu)
        want, den = R.gemm(qa, a_fmt, 0.37, qw, w_fmt, 0.011, b, relu)
        assert_within(got, want, den)


@pytest.mark.parametrize("force_kernel", KERNELS, indirect=True)
@pytest.mark.parametrize("a_fmt,w_fmt", TILED_PAIRS)
def test_tiled_kernels_every_code_pair(force_kernel, a_fmt, w_fmt):
    """Each A code meets each W code exactly once per row pair, so a wrong table entry or a
    wrong k pairing between the two decoders cannot cancel."""
    na, nw = 1 << a_fmt[0], 1 << w_fmt[0]
    K = 64 * ((na * nw + 63) // 64)
    qa = np.zeros((260, K), np.uint8); qw = np.zeros((258, K), np.uint8)
    for r in range(260):
        qa[r] = np.resize(np.repeat(np.arange(na), nw), K)
        qa[r] = np.roll(qa[r], r)
    for r in range(258):
        qw[r] = np.resize(np.tile(np.arange(nw), na), K)
        qw[r] = np.roll(qw[r], 3 * r)
    got = run_gemm(qa, a_fmt, 1.0, qw, w_fmt, 1.0)
    want, den = R.gemm(qa, a_fmt, 1.0, qw, w_fmt, 1.0)
    assert_within(got, want, den)
    # one-hot rows: a single non-zero code per row pins every decoded value on its own,
    # first those of A against a unit weight, then those of W against a unit activation
    cba, cbw = R.codebook(*a_fmt), R.codebook(*w_fmt)
    one_w = int(np.where(cbw == 1.0)[0][0])
    one_a = int(np.where(cba == 1.0)[0][0])
    qa1 = np.zeros((na, 64), np.uint8); qw1 = np.zeros((64, 64), np.uint8)
    for c in range(na):
        qa1[c, c % 64] = c
    qw1[np.arange(64), np.arange(64)] = one_w
    got = run_gemm(qa1, a_fmt, 1.0, qw1, w_fmt, 1.0)
    want = np.zeros((na, 64)); want[np.arange(na), np.arange(na) % 64] = cba
    assert np.array_equal(got.astype(np.float64), want)
    qa2 = np.zeros((64, 64), np.uint8); qw2 = np.zeros((nw, 64), np.uint8)
    qa2[np.arange(64), np.arange(64)] = one_a
    for c in range(nw):
        qw2[c, c % 64] = c
    got = run_gemm(qa2, a_fmt, 1.0, qw2, w_fmt, 1.0)
    want = np.zeros((64, nw)); want[np.arange(nw) % 64, np.arange(nw)] = cbw
    assert np.array_equal(got.astype(np.float64), want)


@pytest.mark.parametrize("force_kernel", KERNELS, indirect=True)
@pytest.mark.parametrize("x_fmt,w_fmt", TILED_PAIRS)
@pytest.mark.parametrize("geom", [(3, 1, 1), (1, 1, 0), (3, 2, 1)])
def test_tiled_kernels_conv(force_kernel, x_fmt, w_fmt, geom):
    k, stride, pad = geom
    rng = np.random.default_rng(k * 7 + stride)
    Bn, H, W, Cin, Cout = 3, 13, 11, 64, 300
    qx = random_codes(rng, (Bn, H, W, Cin), x_fmt)
    qw = random_codes(rng, (Cout, k, k, Cin), w_fmt)
    bias = rng.normal(0, 1, Cout).astype(np.float32)
    got = run_conv(qx, x_fmt, 0.21, qw, w_fmt, 0.05, stride, pad, bias, True)
    want, den = R.conv2d(qx, x_fmt, 0.21, qw, w_fmt, 0.05, stride, pad, bias, True)
    assert_within(got, want, den)


SIX_PAIRS = [((6, True), (6, True)), ((6, False), (6, True)), ((8, True), (6, True)), ((4, False), (6, True)),
             ((6, True), (4, True)), ((6, False), (8, True)), ((2, True), (8, True)), ((2, False), (6, True)),
             ((8, False), (2, True)), ((6, True), (2, True))]


@pytest.mark.parametrize("a_fmt,w_fmt", SIX_PAIRS)
def test_large_kernel_six_bit_operands(a_fmt, w_fmt):
    """2- and 6-bit operands on the 256 x 256 fp16 kernel (K steps of 128: a lane's 64 codes are 16 / 48 bytes): ragged M and N,
    an odd number of K steps, every (A code, W code) pair, one-hot rows, a convolution with 128 channels;
    each call must really run on that kernel."""
    B.dybit_set_option("gemm_kernel", "large")
    try:
        rng = np.random.default_rng(a_fmt[0] * 10 + w_fmt[0])
        for (M, N, K) in ((300, 520, 384), (257, 255, 128), (2100, 300, 640)):
            qa = random_codes(rng, (M, K), a_fmt)
            qw = random_codes(rng, (N, K), w_fmt)
            bias = rng.normal(0, 3, N).astype(np.float32)
            got = run_gemm(qa, a_fmt, 0.37, qw, w_fmt, 0.011, bias, True)
            assert B.dybit_last_gemm_kernel() == "f16_256"
            want, den = R.gemm(qa, a_fmt, 0.37, qw, w_fmt, 0.011, bias, True)
            assert_within(got, want, den)
        na, nw = 1 << a_fmt[0], 1 << w_fmt[0]
        K = 128 * ((na * nw + 127) // 128)
        qa = np.zeros((260, K), np.uint8); qw = np.zeros((258, K), np.uint8)
        for r in range(260):
            qa[r] = np.roll(np.resize(np.repeat(np.arange(na), nw), K), r)
        for r in range(258):
            qw[r] = np.roll(np.resize(np.tile(np.arange(nw), na), K), 3 * r)
        got = run_gemm(qa, a_fmt, 1.0, qw, w_fmt, 1.0)
        assert B.dybit_last_gemm_kernel() == "f16_256"
        want, den = R.gemm(qa, a_fmt, 1.0, qw, w_fmt, 1.0)
        assert_within(got, want, den)
        cba = R.codebook(*a_fmt)
        one_w = int(np.where(R.codebook(*w_fmt) == 1.0)[0][0])
        qa1 = np.zeros((na, 128), np.uint8); qw1 = np.zeros((128, 128), np.uint8)
        qa1[np.arange(na), np.arange(na) % 128] = np.arange(na)
        qw1[np.arange(128), np.arange(128)] = one_w
        got = run_gemm(qa1, a_fmt, 1.0, qw1, w_fmt, 1.0)
        want = np.zeros((na, 128)); want[np.arange(na), np.arange(na) % 128] = cba
        assert np.array_equal(got.astype(np.float64), want)
        qx = random_codes(rng, (2, 9, 10, 128), a_fmt)
        qf = random_codes(rng, (140, 3, 3, 128), w_fmt)
        got = run_conv(qx, a_fmt, 0.3, qf, w_fmt, 0.02, 1, 1)
        assert B.dybit_last_gemm_kernel() == "f16_256"
        want, den = R.conv2d(qx, a_fmt, 0.3, qf, w_fmt, 0.02, 1, 1)
        assert_within(got, want, den)
    finally:
        B.dybit_set_option("gemm_kernel", "auto")


@pytest.mark.parametrize("force_kernel", ["mid1", "mid2", "mid64", "mid1-f16", "mid2-f16"], indirect=True)
def test_mid_kernel_wide_channels_conv(force_kernel):
    """Cin = 192: a 128-wide K step straddles two filter taps (each k-group follows its own tap)."""
    rng = np.random.default_rng(11)
    x_fmt, w_fmt = (4, False), (4, True)
    qx = random_codes(rng, (2, 9, 10, 192), x_fmt)
    qw = random_codes(rng, (130, 3, 3, 192), w_fmt)
    got = run_conv(qx, x_fmt, 0.3, qw, w_fmt, 0.02, 1, 1)
    want, den = R.conv2d(qx, x_fmt, 0.3, qw, w_fmt, 0.02, 1, 1)
    assert_within(got, want, den)


WS_PAIRS = [((4, False), (4, True)), ((8, True), (4, True)), ((8, False), (8, True)), ((6, False), (6, True)),
            ((6, True), (4, True)), ((4, True), (8, True)), ((2, False), (2, True)), ((8, True), (6, True)),
            ((2, True), (8, True)), ((4, False), (2, True))]


@pytest.mark.parametrize("force_kernel", ["ws"], indirect=True)
@pytest.mark.parametrize("a_fmt,w_fmt", WS_PAIRS)
@pytest.mark.parametrize("shape", [(1000, 64, 64), (300, 70, 192), (2049, 128, 576), (257, 100, 128), (5, 128, 256),
                                   (70000, 33, 64), (3000, 256, 64), (1500, 200, 128), (70000, 320, 64), (257, 1000, 192)])
def test_weight_stationary_kernel(force_kernel, a_fmt, w_fmt, shape):
    """The whole weight matrix decoded into LDS once, a persistent grid walking over the rows: N not a
    multiple of 32, ragged M, one to nine K steps, more slabs than workgroups (70000 rows), both
    column-block counts (N <= 64, <= 128); N > 128 in column groups of 64 (a whole number of groups, a last
    group of 8 columns, five groups with more slabs than slab walkers, sixteen groups with fewer);
    bias + ReLU and a leading dimension larger than N."""
    M, N, K = shape
    rng = np.random.default_rng(M + 7 * N + K)
    qa = random_codes(rng, (M, K), a_fmt)
    qw = random_codes(rng, (N, K), w_fmt)
    bias = rng.normal(0, 3, N).astype(np.float32)
    got = run_gemm(qa, a_fmt, 0.37, qw, w_fmt, 0.011, bias, True, ldc=N + 8)
    want, den = R.gemm(qa, a_fmt, 0.37, qw, w_fmt, 0.011, bias, True)
    assert_within(got[:, :N], want, den)
    assert np.all(got[:, N:] == -777.0)


@pytest.mark.parametrize("force_kernel", ["ws"], indirect=True)
@pytest.mark.parametrize("x_fmt,w_fmt", WS_PAIRS[:6])
@pytest.mark.parametrize("geom", [(3, 1, 1), (1, 1, 0), (3, 2, 1), (1, 2, 0)])
@pytest.mark.parametrize("Cout", [96, 264])
def test_weight_stationary_kernel_conv(force_kernel, x_fmt, w_fmt, geom, Cout):
    """Cout = 264: five column groups, the last of 8 channels."""
    k, stride, pad = geom
    rng = np.random.default_rng(k * 11 + stride)
    Bn, H, W, Cin = 3, 13, 11, 64
    qx = random_codes(rng, (Bn, H, W, Cin), x_fmt)
    qw = random_codes(rng, (Cout, k, k, Cin), w_fmt)
    bias = rng.normal(0, 1, Cout).astype(np.float32)
    got = run_conv(qx, x_fmt, 0.21, qw, w_fmt, 0.05, stride, pad, bias, False)
    want, den = R.conv2d(qx, x_fmt, 0.21, qw, w_fmt, 0.05, stride, pad, bias, False)
    assert_within(got, want, den)


@pytest.mark.parametrize("force_kernel", ["ws"], indirect=True)
@pytest.mark.parametrize("x_fmt,w_fmt,Cin,kw", [((8, True), (8, True), 4, 8), ((6, True), (4, True), 4, 8), ((4, False), (6, True), 8, 4),
                                                 ((2, True), (8, True), 4, 8), ((8, False), (4, True), 2, 16)])
@pytest.mark.parametrize("kh,stride,pad,shape", [(8, 2, 3, (3, 23, 21)), (2, 3, 4, (2, 12, 16)), (4, 1, 2, (2, 9, 27)), (6, 2, 5, (1, 30, 17))])
@pytest.mark.parametrize("Cout", [100, 200])
def test_weight_stationary_kernel_few_channels(force_kernel, x_fmt, w_fmt, Cin, kw, kh, stride, pad, shape, Cout):
    """Filter rows of exactly 32 codes fetched row by row (see test_conv_few_channels), weights resident
    (Cout = 200: in four column groups).
    The rows are fetched as aligned 32-bit words, so the kernel is only taken for image tensors of a
    whole number of words; the others must fall back to the general kernel (and still be right)."""
    global _expected_kernels
    Bn, H, W = shape
    if (Bn * H * W * Cin * x_fmt[0] // 8) % 4:
        _expected_kernels = {"general"}
    rng = np.random.default_rng(Cin * 100 + kw * 10 + kh + 1)
    qx = random_codes(rng, (Bn, H, W, Cin), x_fmt)
    qw = random_codes(rng, (Cout, kh, kw, Cin), w_fmt)
    bias = rng.normal(0, 1, Cout).astype(np.float32)
    got = run_conv(qx, x_fmt, 0.21, qw, w_fmt, 0.05, stride, pad, bias, False)
    want, den = R.conv2d(qx, x_fmt, 0.21, qw, w_fmt, 0.05, stride, pad, bias, False)
    assert got.shape == want.shape
    assert_within(got, want, den)


@pytest.mark.parametrize("force_kernel", ["general"], indirect=True)
@pytest.mark.parametrize("a_fmt,w_fmt", [((4, False), (4, True)), ((8, True), (4, True)), ((8, False), (8, True))])
def test_general_kernel_on_tiled_shapes(force_kernel, a_fmt, w_fmt):
    """The general kernel's vector path on shapes the tiled kernels would otherwise take."""
    rng = np.random.default_rng(3)
    qa = random_codes(rng, (257, 192), a_fmt)
    qw = random_codes(rng, (129, 192), w_fmt)
    got = run_gemm(qa, a_fmt, 0.37, qw, w_fmt, 0.011)
    want, den = R.gemm(qa, a_fmt, 0.37, qw, w_fmt, 0.011)
    assert_within(got, want, den)


# ---- running maximum of the outputs taken in the epilogue ---------------------------
@pytest.mark.parametrize("force_kernel", ["large", "mid1", "mid2", "mid64", "general"], indirect=True)
@pytest.mark.parametrize("relu", [False, True])
@pytest.mark.parametrize("a_fmt", [(8, True), (4, False)])
def test_gemm_absmax_matches_a_pass_over_the_output(force_kernel, relu, a_fmt):
    """max|C| from the epilogue is the maximum of the values actually written (ragged tiles, bias,
    ReLU), bit for bit, and the scale derived from it equals dybit_absmax_scale of C."""
    rng = np.random.default_rng(17)
    w_fmt = (4, True)
    M, N, K = 300, 261, 192
    qa = random_codes(rng, (M, K), a_fmt)
    qw = random_codes(rng, (N, K), w_fmt)
    bias = rng.normal(0, 3, N).astype(np.float32)
    mx = torch.zeros(1, dtype=torch.float32, device="cuda")
    c = B.dybit_gemm_ex(M, N, K, pack_rows_dev(qa, a_fmt[0]), a_fmt, scalar(0.37), pack_rows_dev(qw, 4), w_fmt,
                        scalar(0.011), dev(bias), None, relu, mx)
    torch.cuda.synchronize()
    want, den = R.gemm(qa, a_fmt, 0.37, qw, w_fmt, 0.011, bias, relu)
    assert_within(c.cpu().numpy(), want, den)
    assert mx.item() == c.abs().max().item()
    for fmt in ((4, False), (8, True)):
        s_fused = B.dybit_scale_from_absmax(mx, *fmt)
        s_pass = B.dybit_absmax_scale(c.reshape(-1), *fmt)
        assert s_fused.item() == s_pass.item()
    # a larger value already in the word stays; a smaller one is replaced
    big = torch.full((1,), 1.0e9, dtype=torch.float32, device="cuda")
    B.dybit_gemm_ex(M, N, K, pack_rows_dev(qa, a_fmt[0]), a_fmt, scalar(0.37), pack_rows_dev(qw, 4), w_fmt,
                    scalar(0.011), dev(bias), None, relu, big)
    assert big.item() == 1.0e9


@pytest.mark.parametrize("force_kernel", ["mid1", "mid2", "mid64", "mid1-f16", "general"], indirect=True)
@pytest.mark.parametrize("with_shortcut", [False, True])
def test_conv2d_ex_shortcut_and_absmax(force_kernel, with_shortcut):
    """Shortcut added before the ReLU, running maximum over the values written, ragged tiles."""
    rng = np.random.default_rng(23)
    x_fmt, w_fmt = (4, False), (4, True)
    qx = random_codes(rng, (2, 9, 10, 64), x_fmt)
    qw = random_codes(rng, (70, 3, 3, 64), w_fmt)
    bias = rng.normal(0, 1, 70).astype(np.float32)
    res = rng.normal(0, 20, (2, 9, 10, 70)).astype(np.float32) if with_shortcut else None
    mx = torch.zeros(1, dtype=torch.float32, device="cuda")
    y = B.dybit_conv2d_ex(2, 9, 10, 64, 70, 3, 3, 1, 1, pack_rows_dev(qx.reshape(-1, 64), 4), x_fmt, scalar(0.3),
                          pack_rows_dev(qw.reshape(-1, 64), 4), w_fmt, scalar(0.02), dev(bias),
                          None if res is None else dev(res), True, mx)
    torch.cuda.synchronize()
    want, den = R.conv2d(qx, x_fmt, 0.3, qw, w_fmt, 0.02, 1, 1, bias, True, res)
    assert_within(y.cpu().numpy(), want, den, shortcut=with_shortcut)
    assert mx.item() == y.abs().max().item()


@pytest.mark.parametrize("force_kernel", ["large", "mid1", "mid2", "mid64", "general"], indirect=True)
@pytest.mark.parametrize("a_fmt", [(8, True), (4, True)])
def test_gemm_ex_shortcut(force_kernel, a_fmt):
    """C = A W^T + bias + shortcut (no ReLU, so a wrong sign or a shortcut applied after the ReLU shows),
    with a leading dimension larger than N shared by output and shortcut."""
    rng = np.random.default_rng(29)
    w_fmt = (4, True)
    M, N, K, ldc = 290, 200, 128, 208
    qa = random_codes(rng, (M, K), a_fmt)
    qw = random_codes(rng, (N, K), w_fmt)
    bias = rng.normal(0, 3, N).astype(np.float32)
    res = rng.normal(0, 50, (M, ldc)).astype(np.float32)
    out = torch.full((M, ldc), -777.0, dtype=torch.float32, device="cuda")
    B.dybit_gemm_ex(M, N, K, pack_rows_dev(qa, a_fmt[0]), a_fmt, scalar(0.37), pack_rows_dev(qw, 4), w_fmt,
                    scalar(0.011), dev(bias), dev(res), False, None, out=out, ldc=ldc)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    want, den = R.gemm(qa, a_fmt, 0.37, qw, w_fmt, 0.011, bias, False, res[:, :N])
    assert_within(got[:, :N], want, den, shortcut=True)
    assert np.all(got[:, N:] == -777.0)


def test_scale_from_absmax_of_zero_is_one():
    z = torch.zeros(1, dtype=torch.float32, device="cuda")
    assert B.dybit_scale_from_absmax(z, 4, True).item() == 1.0
    v = torch.full((1,), 6.0, dtype=torch.float32, device="cuda")
    assert B.dybit_scale_from_absmax(v, 4, True).item() == 1.5       # 2^(m-1) = 4
    assert B.dybit_scale_from_absmax(v, 8, False).item() == 6.0 / 128


@pytest.mark.parametrize("force_kernel", ["large", "mid1", "mid2", "mid64", "ws", "general"], indirect=True)
@pytest.mark.parametrize("case", ["c_off4", "bias_off4", "res_off4", "ldc_odd", "n_mod4_2"])
def test_epilogue_alignment_cases(force_kernel, case):
    """The epilogue moves four neighbouring columns of a row as one 128-bit word only when every tensor it
    touches allows it; each case breaks one condition (an output, bias or shortcut that starts 4 bytes past a
    16-byte boundary, an odd leading dimension, N = 2 mod 4) and must give the same results element by element."""
    rng = np.random.default_rng(77)
    a_fmt, w_fmt = (4, False), (4, True)
    M, K = 200, 128
    N = 98 if case == "n_mod4_2" else 96
    ldc = 101 if case == "ldc_odd" else (N + 8 if case != "n_mod4_2" else N)
    qa = random_codes(rng, (M, K), a_fmt)
    qw = random_codes(rng, (N, K), w_fmt)
    bias = rng.normal(0, 2, N).astype(np.float32)
    res = rng.normal(0, 20, (M, ldc)).astype(np.float32)
    want, den = R.gemm(qa, a_fmt, 0.3, qw, w_fmt, 0.05, bias, True, res[:, :N])

    def shifted(a, on):          # the same values in a buffer that starts 4 bytes past a 16-byte boundary
        flat = torch.empty(a.size + 4, dtype=torch.float32, device="cuda")
        view = flat[1 if on else 0:][:a.size].view(a.shape)
        view.copy_(dev(a))
        return view
    out = shifted(np.full((M, ldc), -777.0, dtype=np.float32), case == "c_off4")
    mx = torch.zeros(1, dtype=torch.float32, device="cuda")
    c = B.dybit_gemm_ex(M, N, K, pack_rows_dev(qa, 4), a_fmt, scalar(0.3), pack_rows_dev(qw, 4), w_fmt, scalar(0.05),
                        shifted(bias, case == "bias_off4"), shifted(res, case == "res_off4"), True, mx, out=out, ldc=ldc)
    assert_forced_kernel_ran()
    torch.cuda.synchronize()
    got = c.cpu().numpy()
    assert_within(got[:, :N], want, den, shortcut=True)
    assert np.all(got[:, N:] == -777.0)                      # nothing written past column N
    assert mx.item() == np.abs(got[:, :N]).max()
