"""Pins for the oracle's quantizer, dequantizer and bit packing.  CPU only.

The rank-search quantizer is checked against an exact-rational brute force,
against a closed form that is written here independently, against numpy's
round-half-even in the special case where the format is a plain fixed-point
grid, and against the properties any nearest-value rounding must have."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import c_ref, dybit_ref as R

FORMATS = [(b, s) for b in (2, 4, 6, 8) for s in (True, False)]
SCALES = [np.float32(1.0), np.float32(0.25), np.float32(0.75), np.float32(0.0123), np.float32(3.7)]


def _tie_inputs(bits, signed, s):
    """Inputs that sit exactly on decision points (only exact for short scales)."""
    m = R.magnitude_bits(bits, signed)
    mids = R.midpoints(m)
    x = (np.float64(s) * mids).astype(np.float32)
    exact = x.astype(np.float64) == np.float64(s) * mids
    return x[exact]


@pytest.mark.parametrize("bits,signed", FORMATS)
def test_bruteforce_fraction_small(bits, signed):
    rng = np.random.default_rng(bits * 2 + signed)
    for s in SCALES:
        vm = R.vmax(bits, signed)
        x = np.concatenate([
            rng.normal(0, float(s) * vm / 3, 40).astype(np.float32),
            rng.uniform(-1.2, 1.2, 20).astype(np.float32) * np.float32(s * vm),
            _tie_inputs(bits, signed, s)[:24], -_tie_inputs(bits, signed, s)[:24],
            np.nextafter(_tie_inputs(bits, signed, s)[:12], np.float32(np.inf)),
            np.nextafter(_tie_inputs(bits, signed, s)[:12], np.float32(0)),
            np.array([0.0, -0.0, np.inf, -np.inf, np.nan, 1e-30, -1e-30, 3e38, -3e38], dtype=np.float32),
        ])
        got = R.quantize(x, s, bits, signed)
        want = R.quantize_bruteforce(x, s, bits, signed)
        assert got.tolist() == want
        assert c_ref.quantize(x, s, bits, signed).tolist() == want


@pytest.mark.parametrize("bits,signed", FORMATS)
def test_ties_go_to_even_code(bits, signed):
    m = R.magnitude_bits(bits, signed)
    for s in (np.float32(1.0), np.float32(0.5), np.float32(0.75)):
        x = _tie_inputs(bits, signed, s)
        assert x.size == (1 << m) - 1           # all exact for these scales
        q = R.quantize(x, s, bits, signed).astype(int)
        j = np.arange(x.size)
        assert np.array_equal(q, np.where(j % 2 == 0, j, j + 1))
        assert np.all(q % 2 == 0)


def _closed_form(t: Fraction, m: int) -> int:
    """Independent statement of round-to-nearest-even onto the tapered grid:
    below 1 the grid is uniform with step 2^-(m-1); in [2^e, 2^(e+1)) the code is
    (e+1) ones, a zero and the rounded (m-e-2)-bit fraction, carries propagating."""
    def rne(q: Fraction) -> int:
        f = q.numerator // q.denominator
        r = q - f
        if r > Fraction(1, 2) or (r == Fraction(1, 2) and f % 2 == 1):
            f += 1
        return f
    if t >= 2 ** (m - 1):
        return (1 << m) - 1
    if t < 1:
        return rne(t * 2 ** (m - 1))
    e = 0
    while t >= 2 ** (e + 1):
        e += 1
    i, k = e + 1, m - e - 2
    return (((1 << i) - 1) << (m - i)) + rne((t / 2 ** e - 1) * 2 ** k)


@pytest.mark.parametrize("bits,signed", FORMATS)
def test_closed_form_agrees(bits, signed):
    m = R.magnitude_bits(bits, signed)
    rng = np.random.default_rng(7)
    for s in (np.float32(1.0), np.float32(0.0123)):
        x = np.abs(rng.normal(0, float(s) * R.vmax(bits, signed) / 2.5, 4000)).astype(np.float32)
        x = np.concatenate([x, _tie_inputs(bits, signed, np.float32(1.0)) * s])
        q = R.quantize(x, s, bits, signed).astype(int)
        sf = Fraction(float(s))
        for xv, qv in zip(x.tolist(), q.tolist()):
            assert qv == _closed_form(Fraction(xv) / sf, m)


@pytest.mark.parametrize("bits,signed", [(4, False), (6, False), (8, False), (4, True), (8, True)])
def test_linear_region_is_round_half_even(bits, signed):
    """With a power-of-two scale and |x| < s the format is a uniform grid, so the
    code is numpy's rint (round half to even) of |x|/s * 2^(m-1)."""
    m = R.magnitude_bits(bits, signed)
    rng = np.random.default_rng(3)
    for j in (-3, 0, 5):
        s = np.float32(2.0 ** j)
        x = (rng.uniform(0, 1, 5000).astype(np.float32) * s).astype(np.float32)
        x = x[x < s]
        grid = np.arange(0, 1 << (m - 1)) + 0.5           # exact half-way points
        x = np.concatenate([x, (grid * 2.0 ** (j - (m - 1))).astype(np.float32)])
        want = np.rint(x.astype(np.float64) / float(s) * 2.0 ** (m - 1)).astype(int)
        assert np.array_equal(R.quantize(x, s, bits, signed).astype(int), want)


@pytest.mark.parametrize("bits,signed", FORMATS)
def test_monotone_and_error_bound(bits, signed):
    m = R.magnitude_bits(bits, signed)
    cb = R.codebook(bits, signed)
    mag = R.magnitude_table(m)
    rng = np.random.default_rng(11)
    s = np.float32(0.037)
    x = np.sort(rng.normal(0, float(s) * R.vmax(bits, signed) / 2, 20000).astype(np.float32))
    q = R.quantize(x, s, bits, signed)
    val = cb[q]
    assert np.all(np.diff(val) >= 0)                      # monotone in x
    inside = np.abs(x.astype(np.float64)) <= float(s) * mag[-1]
    if not signed:
        inside &= x >= 0
    err = np.abs(x.astype(np.float64) - float(s) * val)
    idx = (q & ((1 << m) - 1)).astype(int)
    gap_up = np.where(idx < mag.size - 1, mag[np.minimum(idx + 1, mag.size - 1)] - mag[idx], np.inf)
    gap_dn = np.where(idx > 0, mag[idx] - mag[np.maximum(idx - 1, 0)], np.inf)
    above = np.abs(x.astype(np.float64)) >= float(s) * mag[idx]
    half_gap = 0.5 * float(s) * np.where(above, gap_up, gap_dn)
    assert np.all(err[inside] <= half_gap[inside])
    # no other code is strictly closer
    for xv, e in zip(x[::997].astype(np.float64), err[::997]):
        assert e <= np.min(np.abs(xv - float(s) * cb)) + 0.0


@pytest.mark.parametrize("bits,signed", FORMATS)
def test_special_inputs(bits, signed):
    m = R.magnitude_bits(bits, signed)
    top = (1 << m) - 1
    sgn = 1 << (bits - 1)
    s = np.float32(0.5)
    x = np.array([np.nan, np.inf, -np.inf, 0.0, -0.0, 1e30, -1e30,
                  0.5 * R.vmax(bits, signed), -1e-38], dtype=np.float32)
    q = R.quantize(x, s, bits, signed).tolist()
    if signed:
        assert q == [0, top, top | sgn, 0, 0, top, top | sgn, top, 0]
    else:
        assert q == [0, top, 0, 0, 0, top, 0, top, 0]
    for bad in (0.0, -1.0, np.inf, np.nan):
        with pytest.raises(ValueError):
            R.quantize(x, bad, bits, signed)


@pytest.mark.parametrize("bits,signed", FORMATS)
def test_c_and_numpy_quantizers_agree(bits, signed):
    rng = np.random.default_rng(5)
    x = rng.laplace(0, 0.02, 200000).astype(np.float32)
    s = R.absmax_scale(x, bits, signed)
    assert s == c_ref.absmax_scale(x, bits, signed)
    assert s == np.float32(np.abs(x).max() / R.vmax(bits, signed))
    q = R.quantize(x, s, bits, signed)
    assert np.array_equal(q, c_ref.quantize(x, s, bits, signed))
    assert int((q & ((1 << R.magnitude_bits(bits, signed)) - 1)).max()) == (1 << R.magnitude_bits(bits, signed)) - 1
    y = R.dequantize(q, s, bits, signed)
    assert np.array_equal(y, c_ref.dequantize(q, s, bits, signed))
    assert np.array_equal(y, np.float32(s) * R.codebook(bits, signed).astype(np.float32)[q])


def test_absmax_scale_cases():
    assert R.absmax_scale(np.zeros(5, np.float32), 4, True) == 1.0
    assert R.absmax_scale(np.array([], np.float32), 8, True) == 1.0
    assert R.absmax_scale(np.array([np.nan, -3.0, 2.0], np.float32), 4, True) == np.float32(0.75)
    assert c_ref.absmax_scale(np.array([np.nan, -3.0, 2.0], np.float32), 4, True) == np.float32(0.75)
    assert R.absmax_scale(np.array([-3.0, 2.0], np.float32), 4, False) == np.float32(0.375)


# ---- packing ---------------------------------------------------------------
def test_pack_layout_examples():
    # 4-bit: element 2j in the low nibble, 2j+1 in the high nibble
    assert R.pack(np.array([1, 2, 3]), 4).tolist() == [0x21, 0x03]
    # 8-bit: identity
    assert R.pack(np.array([7, 200]), 8).tolist() == [7, 200]
    # 6-bit: four codes in three bytes, LSB first
    codes = [0b000001, 0b100000, 0b111111, 0b010101]
    stream = sum(c << (6 * j) for j, c in enumerate(codes))
    assert R.pack(np.array(codes), 6).tolist() == [stream & 255, (stream >> 8) & 255, stream >> 16]
    # 2-bit: four per byte
    assert R.pack(np.array([1, 2, 3, 0, 1]), 2).tolist() == [0b00111001, 0b01]


@pytest.mark.parametrize("bits", [2, 4, 6, 8])
def test_pack_roundtrip_and_c(bits):
    rng = np.random.default_rng(bits)
    for n in (0, 1, 3, 4, 17, 1000):
        codes = rng.integers(0, 1 << bits, n).astype(np.uint8)
        buf = R.pack(codes, bits)
        assert buf.size == R.packed_bytes(n, bits)
        assert np.array_equal(R.unpack(buf, n, bits), codes)
        assert np.array_equal(c_ref.pack(codes, bits), buf)
        assert np.array_equal(c_ref.unpack(buf, n, bits), codes)
        # generic definition: bit b of code j is bit (j*bits + b) of the stream
        big = int.from_bytes(buf.tobytes(), "little")
        for j in range(min(n, 9)):
            assert (big >> (j * bits)) & ((1 << bits) - 1) == codes[j]


def test_rmse_definition():
    """Eq. 2 against a hand computation."""
    x = np.array([1.0, -1.0, 3.0, -3.0])
    xq = np.array([1.0, -1.0, 2.0, -2.0])
    sigma = np.sqrt(5.0)
    assert R.rmse(x, xq) == pytest.approx(np.sqrt((0 + 0 + 1 + 1) / 4) / sigma)
