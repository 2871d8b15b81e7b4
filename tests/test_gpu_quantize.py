"""GPU parity: absmax scale, quantize and dequantize against the CPU oracle, bit for bit."""
import numpy as np
import pytest
import torch

from oracle import dybit_ref as R
from paper_2302_12510_amd import binding as B
from paper_2302_12510_amd import synth
from gpu_util import dev, scalar

pytestmark = pytest.mark.gpu
FORMATS = [(b, s) for b in (2, 4, 6, 8) for s in (True, False)]


def gpu_quantize(x: np.ndarray, s, fmt) -> np.ndarray:
    xd = dev(x.astype(np.float32).ravel())
    out = B.dybit_quantize(xd, scalar(s), *fmt)
    torch.cuda.synchronize()
    assert B.dybit_get_last_async_error() == B.OK
    return out.cpu().numpy()


def check_codes(x, s, fmt):
    got = gpu_quantize(x, s, fmt)
    want = R.pack(R.quantize(x.ravel(), s, *fmt), fmt[0])
    assert got.shape == want.shape
    if not np.array_equal(got, want):
        gu, wu = R.unpack(got, x.size, fmt[0]), R.unpack(want, x.size, fmt[0])
        bad = np.nonzero(gu != wu)[0]
        raise AssertionError(f"fmt {fmt} scale {s!r}: {bad.size} codes differ, first at {bad[0]}: "
                             f"x={x.ravel()[bad[0]]!r} got {gu[bad[0]]} want {wu[bad[0]]}")


@pytest.mark.parametrize("fmt", FORMATS)
def test_laplace_tensor_codes_scale_and_dequantize(fmt):
    n = (1 << 20) + 4099                      # several blocks plus a ragged tail
    x = synth.laplace((n,), 0.02, seed=1, stream=fmt[0])
    xd = dev(x)
    sd = B.dybit_absmax_scale(xd, *fmt)
    s = R.absmax_scale(x, *fmt)
    assert sd.cpu().numpy()[0] == s
    codes = B.dybit_quantize(xd, sd, *fmt)
    want = R.pack(R.quantize(x, s, *fmt), fmt[0])
    assert np.array_equal(codes.cpu().numpy(), want)
    y = B.dybit_dequantize(codes, n, sd, *fmt)
    assert np.array_equal(y.cpu().numpy(), R.dequantize(R.unpack(want, n, fmt[0]), s, *fmt))
    assert B.dybit_get_last_async_error() == B.OK


@pytest.mark.parametrize("fmt", FORMATS)
@pytest.mark.parametrize("s", [1.0, 0.75, 0.0123, 3.7, 2.0 ** -20, 1.9999999 * 2.0 ** 40, 1.1 * 2.0 ** -110,
                               1.3 * 2.0 ** 105, 2.0 ** -126])
def test_decision_points_and_neighbours(fmt, s):
    """Inputs on, just above and just below every decision point, both signs."""
    s = np.float32(s)
    m = R.magnitude_bits(*fmt)
    mids = (np.float64(s) * R.midpoints(m)).astype(np.float32)
    vals = (np.float64(s) * R.magnitude_table(m)).astype(np.float32)
    base = np.concatenate([mids, vals])
    with np.errstate(over="ignore"):
        x = np.concatenate([base, np.nextafter(base, np.float32(np.inf)), np.nextafter(base, np.float32(0)),
                            base * np.float32(1 + 2e-7), base * np.float32(1 - 2e-7)])
    x = np.concatenate([x, -x]).astype(np.float32)
    check_codes(x, s, fmt)


@pytest.mark.parametrize("fmt", FORMATS)
def test_dense_sweep_near_ties(fmt):
    """Random inputs concentrated within a few ulps of decision points for awkward scales."""
    rng = np.random.default_rng(17)
    m = R.magnitude_bits(*fmt)
    for s in (np.float32(0.3), np.float32(1.0 / 3.0), np.float32(7.77e-4), np.float32(123.456)):
        mids = np.float64(s) * R.midpoints(m)
        pick = rng.integers(0, mids.size, 200000)
        x = mids[pick].astype(np.float32)
        steps = rng.integers(-3, 4, x.size)
        for _ in range(3):
            x = np.where(steps > 0, np.nextafter(x, np.float32(np.inf)), x)
            x = np.where(steps < 0, np.nextafter(x, np.float32(0)), x)
            steps = steps - np.sign(steps)
        x = x * rng.choice([-1.0, 1.0], x.size).astype(np.float32)
        check_codes(x, s, fmt)


@pytest.mark.parametrize("fmt", FORMATS)
def test_special_values_and_sizes(fmt):
    vm = R.vmax(*fmt)
    special = np.array([np.nan, np.inf, -np.inf, 0.0, -0.0, 1e30, -1e30, 1e-45, -1e-45, 1e-38,
                        0.5 * vm, -0.5 * vm, 0.5 * vm * 0.999999, 0.49999 * 2.0 ** -(R.magnitude_bits(*fmt) - 1)],
                       dtype=np.float32)
    rng = np.random.default_rng(3)
    for n in (1, 2, 3, 4, 5, 7, 15, 16, 17, 31, 63, 64, 65, 1023, 1025, 4097):
        x = np.resize(special, n).astype(np.float32)
        x[rng.integers(0, n, n // 2)] = rng.normal(0, 0.3 * vm, n // 2).astype(np.float32)[: max(n // 2, 0)]
        check_codes(x, np.float32(0.5), fmt)
        # absmax ignores NaN; Inf makes the scale Inf (rejected by quantize)
        finite = np.where(np.isinf(x), np.float32(1.0), x)
        sd = B.dybit_absmax_scale(dev(finite), *fmt)
        assert sd.cpu().numpy()[0] == R.absmax_scale(finite, *fmt)


def test_empty_and_all_zero():
    fmt = (4, True)
    x = torch.zeros(0, dtype=torch.float32, device="cuda")
    assert B.dybit_absmax_scale(x, *fmt).item() == 1.0
    assert B.dybit_quantize(x, scalar(1.0), *fmt).numel() == 0
    z = torch.zeros(1000, dtype=torch.float32, device="cuda")
    assert B.dybit_absmax_scale(z, *fmt).item() == 1.0
    assert B.dybit_quantize(z, scalar(1.0), *fmt).sum().item() == 0


@pytest.mark.parametrize("bad", [0.0, -1.0, float("inf"), float("nan"), 1e-45])
def test_bad_scale_sets_flag_and_writes_nothing(bad):
    fmt = (8, True)
    x = dev(np.linspace(-1, 1, 4096, dtype=np.float32))
    out = torch.full((4096,), 0xAB, dtype=torch.uint8, device="cuda")
    B.dybit_quantize(x, scalar(bad), *fmt, out=out)
    assert B.dybit_get_last_async_error() == B.ERR_BAD_SCALE
    assert B.dybit_get_last_async_error() == B.OK            # cleared by the read
    assert int((out != 0xAB).sum().item()) == 0


def test_quantize_is_deterministic_and_leaves_guard_bytes():
    fmt = (4, True)
    n = 100003
    x = dev(synth.laplace((n,), 0.02, seed=2))
    s = B.dybit_absmax_scale(x, *fmt)
    nb = B.dybit_packed_bytes(*fmt, n)
    buf = torch.full((nb + 64,), 0x5A, dtype=torch.uint8, device="cuda")
    B.dybit_quantize(x, s, *fmt, out=buf[:nb])
    a = buf.clone()
    B.dybit_quantize(x, s, *fmt, out=buf[:nb])
    assert torch.equal(a, buf)
    assert int((buf[nb:] != 0x5A).sum().item()) == 0


@pytest.mark.parametrize("fmt", FORMATS)
@pytest.mark.parametrize("n", [1, 5, 16, 4099, (1 << 18) + 21])
def test_quantize_with_a_known_maximum(fmt, n):
    """dybit_quantize_absmax = dybit_scale_from_absmax + dybit_quantize in one launch: scale and codes
    are those of the oracle for the tensor's own maximum; an all-zero tensor gets scale 1."""
    rng = np.random.default_rng(n + fmt[0])
    x = rng.laplace(0, 0.02, n).astype(np.float32)
    if not fmt[1]:
        x = np.abs(x)
    for arr in (x, np.zeros(n, np.float32)):
        xd = torch.from_numpy(arr).cuda()
        mx = torch.tensor([float(np.abs(arr).max())], dtype=torch.float32, device="cuda")
        scale, codes = B.dybit_quantize_absmax(xd, mx, *fmt)
        torch.cuda.synchronize()
        s = R.absmax_scale(arr, *fmt)
        assert scale.item() == s
        assert np.array_equal(codes.cpu().numpy(), R.pack(R.quantize(arr, s, *fmt), fmt[0]))
    assert B.dybit_get_last_async_error() == B.OK


@pytest.mark.parametrize("fmt", FORMATS)
@pytest.mark.parametrize("n", [1, 3, 4, 5, 1023, 4099, (1 << 20) + 7])
def test_fake_quant_equals_quantize_then_dequantize(fmt, n):
    """dybit_fake_quant against the oracle's dequantize(quantize(x)), bit for bit, with special values,
    saturation and (signed formats) negative values that round to zero."""
    rng = np.random.default_rng(n + fmt[0])
    x = rng.laplace(0, 0.02, n).astype(np.float32)
    x[:: max(n // 7, 1)] *= np.float32(30.0)
    if n > 4:
        x[1], x[2], x[3], x[4] = np.nan, np.inf, -np.inf, -1e-9
    s = np.float32(0.6) * R.absmax_scale(np.nan_to_num(x, nan=0.0, posinf=0.0, neginf=0.0), *fmt)
    want = R.dequantize(R.quantize(x, s, *fmt), s, *fmt)
    got = B.dybit_fake_quant(dev(x), scalar(s), *fmt)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy().view(np.uint32), want.view(np.uint32))


def test_fake_quant_in_place_and_bad_scale():
    x = dev(np.linspace(-3, 3, 1001, dtype=np.float32))
    want = B.dybit_fake_quant(x, scalar(0.25), 4, True).clone()
    B.dybit_fake_quant(x, scalar(0.25), 4, True, out=x)
    assert torch.equal(x, want)
    assert B.dybit_get_last_async_error() == B.OK
    y = torch.full((1001,), 7.0, device="cuda")
    B.dybit_fake_quant(x, scalar(0.0), 4, True, out=y)
    assert B.dybit_get_last_async_error() == B.ERR_BAD_SCALE
    assert bool((y == 7.0).all())


def test_config5b_full_size():
    """The standalone quantize workload at its stated size (2^28 Laplace floats), i.e. the launch the
    benchmark times: four loads in flight per lane and more than one trip round the grid-stride loop.
    Scale bit-equal, packed codes byte for byte against the C oracle (plain loops, OpenMP) at 4 bits
    signed, 8 bits signed and 6 bits signed, and the decoder on the 8-bit codes at that size."""
    from oracle import c_ref
    n = 1 << 28
    x = synth.config5b(n=n)
    xd = torch.from_numpy(x).cuda()
    for fmt in ((4, True), (8, True), (6, True)):
        sd = B.dybit_absmax_scale(xd, *fmt)
        s = c_ref.absmax_scale(x, *fmt)
        assert sd.item() == s, fmt
        codes = B.dybit_quantize(xd, sd, *fmt)
        torch.cuda.synchronize()
        q = c_ref.quantize(x, s, *fmt)
        want = c_ref.pack(q, fmt[0])
        got = codes.cpu().numpy()
        assert got.shape == want.shape
        if not np.array_equal(got, want):
            bad = np.nonzero(got != want)[0]
            raise AssertionError(f"fmt {fmt}: {bad.size} packed bytes differ, first at byte {bad[0]}")
        if fmt == (8, True):
            y = B.dybit_dequantize(codes, n, sd, *fmt)
            torch.cuda.synchronize()
            assert np.array_equal(y.cpu().numpy().view(np.uint32), c_ref.dequantize(q, s, *fmt).view(np.uint32))
            del y
        del codes, q, want, got
    assert B.dybit_get_last_async_error() == B.OK


def test_caller_owned_error_word():
    """dybit_set_async_error_word: this thread's kernels report into the caller's word, the library's flag stays
    clear; NULL restores the library's flag."""
    x = torch.randn(4096, device="cuda")
    word = torch.zeros(1, dtype=torch.int32, device="cuda")
    assert B.dybit_get_last_async_error() == B.OK
    B.dybit_set_async_error_word(word)
    try:
        B.dybit_quantize(x, scalar(0.0), 4, True)
        torch.cuda.synchronize()
        assert word.item() == B.ERR_BAD_SCALE
        word.zero_()
        B.dybit_fake_quant(x, scalar(float("nan")), 8, True)
        torch.cuda.synchronize()
        assert word.item() == B.ERR_BAD_SCALE
        word.zero_()
        a = torch.zeros(64 * 64, dtype=torch.uint8, device="cuda")
        B.dybit_gemm_wb(64, 64, 64, a, (8, False), scalar(1.0), a, (8, True), scalar(1.0), (8, False), scalar(-1.0))
        torch.cuda.synchronize()
        assert word.item() == B.ERR_BAD_SCALE
        word.zero_()
        B.dybit_quantize(x, scalar(0.5), 4, True)
        torch.cuda.synchronize()
        assert word.item() == B.OK
        assert B.dybit_get_last_async_error() == B.OK
    finally:
        B.dybit_set_async_error_word(None)
    B.dybit_quantize(x, scalar(0.0), 4, True)
    assert B.dybit_get_last_async_error() == B.ERR_BAD_SCALE
    assert B.dybit_get_last_async_error() == B.OK


@pytest.mark.parametrize("fmt", [(2, False), (2, True), (4, False), (4, True), (6, False), (6, True), (8, False), (8, True)])
@pytest.mark.parametrize("shape", [(1000, 3, 4), (37, 1, 4), (513, 5, 8), (64, 4, 4), (9, 7, 16)])
def test_quantize_pad(fmt, shape):
    """dybit_quantize_pad: the codes of dybit_quantize on the zero-padded tensor, byte for byte against the
    oracle (special values and exact ties included)."""
    rows, cols, cpad = shape
    rng = np.random.default_rng(rows + fmt[0])
    x = rng.laplace(0, 1.0, (rows, cols)).astype(np.float32)
    x.reshape(-1)[:6] = [0.0, -0.0, np.inf, -np.inf, np.nan, 1e-30][: min(6, x.size)]
    s = R.absmax_scale(np.where(np.isfinite(x), x, 0), *fmt)
    mids = R.midpoints(R.magnitude_bits(*fmt)) * np.float64(s)
    k = min(mids.size, x.size - 6)
    if k > 0:
        x.reshape(-1)[6:6 + k] = mids[:k].astype(np.float32)          # decision points (exact where representable)
    xp = np.zeros((rows, cpad), dtype=np.float32)
    xp[:, :cols] = x
    want = R.pack_rows(R.quantize(xp, s, *fmt).reshape(rows, cpad), fmt[0])
    got = B.dybit_quantize_pad(dev(x), cpad, scalar(s), *fmt)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), want)
    assert B.dybit_get_last_async_error() == B.OK


def test_quantize_pad_refusals_and_bad_scale():
    x = torch.randn(16, 3, device="cuda")
    with pytest.raises(B.DybitError) as e:
        B.dybit_quantize_pad(x, 6, scalar(1.0), 4, False)
    assert e.value.status == B.ERR_ALIGNMENT
    with pytest.raises(B.DybitError) as e:
        B.dybit_quantize_pad(x, 0, scalar(1.0), 4, False)
    assert e.value.status == B.ERR_INVALID_ARG
    B.dybit_quantize_pad(x, 4, scalar(0.0), 4, False)
    assert B.dybit_get_last_async_error() == B.ERR_BAD_SCALE
