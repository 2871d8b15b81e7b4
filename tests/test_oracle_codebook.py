"""Pins for the oracle's number format: the paper's printed examples and the
invariants that Eq. 1 / Table I imply.  CPU only."""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import c_ref, dybit_ref as R
from oracle import minifloat as MF

FORMATS = [(b, s) for b in (2, 4, 6, 8) for s in (True, False)]


def _read_rows(path):
    rows = []
    with open(path) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


def test_table1_all_16_values(golden_dir):
    """Table I (Sec. III-A): every row of the 4-bit unsigned truth table."""
    rows = _read_rows(os.path.join(golden_dir, "table1_4bit_unsigned.txt"))
    assert len(rows) == 16
    cb = R.codebook(4, False)
    cbc = c_ref.codebook(4, False)
    for code_s, val_s in rows:
        c = int(code_s, 2)
        assert cb[c] == float(val_s), (code_s, cb[c])
        assert cbc[c] == float(val_s)
        assert R.magnitude_value_exact(c, 4) == Fraction(val_s)


def test_decoder_worked_example(golden_dir):
    """Sec. III-B decoder example: 11001010 -> exponent 001, mantissa 10101000."""
    (code_s, exp_s, man_s), = _read_rows(os.path.join(golden_dir, "decoder_example_8bit_unsigned.txt"))
    c = int(code_s, 2)
    exp, man = R.decode_fields(c, 8)
    assert exp == int(exp_s, 2)
    assert man == int(man_s, 2)
    # the two fields determine the value: 2^1 * 1.0101b = 2.625
    assert R.codebook(8, False)[c] == 2.0 ** exp * man / 128.0 == 2.625


@pytest.mark.parametrize("bits,signed", FORMATS)
def test_fields_reproduce_values(bits, signed):
    """value = 2^exp * mantissa / 2^(m-1) for every code (decoder description)."""
    m = R.magnitude_bits(bits, signed)
    tab = R.magnitude_table(m)
    for c in range(1 << m):
        e, man = R.decode_fields(c, m)
        assert tab[c] == 2.0 ** e * man / 2.0 ** (m - 1)
        if c >> (m - 1):                     # hidden one present at the MSB
            assert man >> (m - 1) == 1


@pytest.mark.parametrize("bits,signed", FORMATS)
def test_eq1_third_case_by_construction(bits, signed):
    """Build codes as i ones, a zero, then the k-bit fraction x and compare with
    (-1)^s 2^(i-1) (1 + x/2^k) (Eq. 1)."""
    m = R.magnitude_bits(bits, signed)
    cb = R.codebook(bits, signed)
    for i in range(1, m):
        k = m - i - 1
        for x in range(1 << k):
            s = "1" * i + "0" + (format(x, f"0{k}b") if k else "")
            c = int(s, 2)
            want = Fraction(2) ** (i - 1) * (1 + Fraction(x, 1 << k))
            assert Fraction(cb[c]) == want
            if signed:
                assert Fraction(cb[(1 << (bits - 1)) | c]) == -want


@pytest.mark.parametrize("bits,signed", FORMATS)
def test_enumeration_invariants(bits, signed):
    m = R.magnitude_bits(bits, signed)
    mag = R.magnitude_table(m)
    # ascending codes <-> ascending values (visible in Table I)
    assert np.all(np.diff(mag) > 0)
    assert mag[0] == 0 and mag[-1] == 2.0 ** (m - 1) == R.vmax(bits, signed)
    if m > 1:
        assert mag[1] == 2.0 ** -(m - 1)
    # start bit 0 <=> magnitude < 1
    assert np.all(mag[: 1 << (m - 1)] < 1) and np.all(mag[1 << (m - 1):] >= 1)
    assert np.count_nonzero(mag < 1) == 1 << (m - 1)
    for i in range(1, m):
        n_in = np.count_nonzero((mag >= 2.0 ** (i - 1)) & (mag < 2.0 ** i))
        assert n_in == 1 << (m - i - 1)
    # all values are integer multiples of 2^-(m-1)
    scaled = mag * 2.0 ** (m - 1)
    assert np.all(scaled == np.rint(scaled))
    cb = R.codebook(bits, signed)
    assert cb.size == 1 << bits
    if signed:
        half = 1 << (bits - 1)
        assert np.all(cb[half + 1:] == -cb[1:half])        # sign symmetry
        assert cb[half] == 0 and not np.signbit(cb[half])  # "negative zero" pattern is +0
        assert np.unique(cb).size == cb.size - 1           # distinct except the two zeros
    else:
        assert np.unique(cb).size == cb.size
    assert np.array_equal(cb, c_ref.codebook(bits, signed))
    assert [Fraction(v) for v in cb[: 1 << m]] == R.codebook_exact(bits, signed)[: 1 << m]


def test_known_small_codebooks():
    assert list(R.codebook(2, True)) == [0, 1, 0, -1]
    assert list(R.magnitude_table(3)) == [0, .25, .5, .75, 1, 1.5, 2, 4]
    assert [R.vmax(b, s) for b, s in [(4, True), (4, False), (6, True), (6, False), (8, True), (8, False)]] \
        == [4, 8, 16, 32, 64, 128]


@pytest.mark.parametrize("bits,signed", FORMATS)
def test_encode_inverts_decode(bits, signed):
    """Quantizing an exactly representable value returns its own code."""
    cb = R.codebook(bits, signed)
    half = 1 << (bits - 1)
    for s in (np.float32(1.0), np.float32(0.75), np.float32(5 / 4096), np.float32(40961 / 2 ** 20)):
        x = (np.float64(s) * cb).astype(np.float32)       # exact: <= 7-bit value times <= 16-bit s
        assert np.array_equal(x.astype(np.float64), np.float64(s) * cb)
        want = np.arange(1 << bits)
        if signed:
            want[half] = 0
        assert np.array_equal(R.quantize(x, s, bits, signed), want)


# ---- exact embedding into matrix-core input types -------------------------
EXPECTED_EMBED = {
    # format: types in which every value is exact
    (2, True): {"fp16", "bf16", "fp8_e4m3", "fp8_e5m2", "fp6_e2m3", "fp6_e3m2", "fp4_e2m1"},
    (4, True): {"fp16", "bf16", "fp8_e4m3", "fp8_e5m2", "fp6_e2m3", "fp6_e3m2"},
    (4, False): {"fp16", "bf16", "fp8_e4m3", "fp8_e5m2", "fp6_e3m2"},
    (6, True): {"fp16", "bf16", "fp8_e4m3"},
    (6, False): {"fp16", "bf16"},
    (8, True): {"fp16", "bf16"},
    (8, False): {"fp16", "bf16"},
}


@pytest.mark.parametrize("fmt", sorted(EXPECTED_EMBED))
def test_exact_embedding_by_enumeration(fmt):
    vals = R.codebook_exact(*fmt)
    got = {t for t in MF.TYPES if MF.embeds_exactly(vals, t)}
    assert got == EXPECTED_EMBED[fmt]
    m = R.magnitude_bits(*fmt)
    # an int8 operand holds value * 2^(m-1) only while 2^(2m-2) <= 127
    assert (max(abs(v) for v in vals) * 2 ** (m - 1) <= 127) == (m <= 4)


def test_minifloat_models_against_known_constants():
    """Pin the enumeration models themselves to published constants of each type."""
    assert max(MF.finite_values("fp16")) == 65504
    assert max(MF.finite_values("fp8_e4m3")) == 448
    assert max(MF.finite_values("fp8_e5m2")) == 57344
    assert max(MF.finite_values("fp6_e2m3")) == Fraction(15, 2)
    assert max(MF.finite_values("fp6_e3m2")) == 28
    assert max(MF.finite_values("fp4_e2m1")) == 6
    assert min(v for v in MF.finite_values("fp16") if v > 0) == Fraction(1, 1 << 24)
    assert min(v for v in MF.finite_values("fp8_e4m3") if v > 0) == Fraction(1, 512)
    # numpy's own float16 agrees with the model on every DyBit value
    for fmt in EXPECTED_EMBED:
        for v in R.codebook(*fmt):
            h = np.float16(v)
            assert float(h) == v
            assert MF.encode("fp16", Fraction(v)) == int(h.view(np.uint16)) or v == 0
