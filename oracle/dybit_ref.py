"""Plain numpy / pure-Python oracle for DyBit.  TEST INFRASTRUCTURE ONLY.

Everything here is the definition written out, in float64 or exact rational
arithmetic, with no blocking, fusion or reordering.  Nothing in the HIP library
imports this file and this file imports nothing from the HIP library.

Notation (Sec. III-A): an N-bit *signed* code is one sign bit followed by
m = N-1 magnitude bits; an N-bit *unsigned* code is m = N magnitude bits (the
truth table, Table I, and the decoder example in Sec. III-B are both unsigned).

Readings of the paper taken here (each one is also listed in the design notes):
  * The largest magnitude is 2^(m-1): Table I prints 1111 -> 8 for m = 4, which
    overrides the "2^n" written in the max case of Eq. 1.
  * Magnitude codes whose first bit is 0 are a pure fraction c / 2^(m-1) with no
    hidden one (Sec. III-A, "start bit 0"; Table I rows 0000..0111).
  * Otherwise i = number of leading ones before the first zero, the k = m-i-1
    bits after that zero are the fraction field x, value = 2^(i-1) (1 + x/2^k)
    (Eq. 1, third case).
  * Signed codes are sign-magnitude; the pattern sign=1, magnitude=0 decodes to
    +0 and is never produced by the quantizer.
  * Quantization is round-to-nearest in exact real arithmetic with ties going to
    the even magnitude code; the paper's encoder (Sec. III-B) truncates, this
    build rounds.
  * Packed storage is a little-endian bit stream: code j occupies bits
    [j*bits, (j+1)*bits) of the byte stream, least significant bit first.

Parity pins (tests/test_oracle_*.py): Table I, the Sec. III-B decoder example,
enumeration invariants, Fraction brute force, closed forms and library routines.
Unpinned: nothing in this file.
"""
from __future__ import annotations

from fractions import Fraction

import numpy as np

SUPPORTED_BITS = (2, 4, 6, 8)


# --------------------------------------------------------------------------
# Number format (Sec. III-A, Eq. 1, Table I)
# --------------------------------------------------------------------------
def magnitude_bits(bits: int, signed: bool) -> int:
    """m = number of magnitude bits of an N-bit code (Sec. III-A)."""
    if bits not in SUPPORTED_BITS:
        raise ValueError(f"unsupported bitwidth {bits}")
    m = bits - 1 if signed else bits
    if m < 1:
        raise ValueError("format has no magnitude bits")
    return m


def leading_ones(c: int, m: int) -> int:
    """Number of 1s before the first 0, scanning from the MSB of an m-bit field
    (the leading-one detector of Sec. III-A / III-B)."""
    i = 0
    for pos in range(m - 1, -1, -1):
        if (c >> pos) & 1:
            i += 1
        else:
            break
    return i


def magnitude_value_exact(c: int, m: int) -> Fraction:
    """Exact value of magnitude code c in an m-bit field (Eq. 1 + Table I)."""
    if not 0 <= c < (1 << m):
        raise ValueError("magnitude code out of range")
    if c == 0:                                   # Eq. 1, zero case
        return Fraction(0)
    if c == (1 << m) - 1:                        # Eq. 1, max case (Table I: 1111 -> 8)
        return Fraction(1 << (m - 1))
    if (c >> (m - 1)) == 0:                      # start bit 0: fraction only
        return Fraction(c, 1 << (m - 1))
    i = leading_ones(c, m)                       # 1 <= i <= m-1
    k = m - i - 1                                # fraction length
    x = c & ((1 << k) - 1)                       # fraction field
    return Fraction(1 << (i - 1)) * (1 + Fraction(x, 1 << k))   # Eq. 1, third case


def decode_fields(c: int, m: int) -> tuple[int, int]:
    """(exp, mantissa) as the mixed-precision decoder of Sec. III-B produces them.

    The mantissa is an m-bit integer with the binary point after its MSB, so
    value = 2^exp * mantissa / 2^(m-1).  For codes that start with 1 the decoder
    counts the leading ones (exp = i - 1), shifts them and the terminating zero
    out and inserts the hidden one at the MSB.  Codes that start with 0 carry no
    hidden one (exp = 0, mantissa = c); the all-ones code is 1.0 x 2^(m-1).
    """
    if c == (1 << m) - 1:
        return m - 1, 1 << (m - 1)
    if (c >> (m - 1)) == 0:
        return 0, c
    i = leading_ones(c, m)
    k = m - i - 1
    x = c & ((1 << k) - 1)
    return i - 1, (1 << (m - 1)) | (x << (m - 1 - k))


def magnitude_table(m: int) -> np.ndarray:
    """float64 values of all 2^m magnitude codes (every value is dyadic, so exact)."""
    return np.array([float(magnitude_value_exact(c, m)) for c in range(1 << m)],
                    dtype=np.float64)


def vmax(bits: int, signed: bool) -> float:
    """Largest representable magnitude, 2^(m-1)."""
    return float(1 << (magnitude_bits(bits, signed) - 1))


def codebook(bits: int, signed: bool) -> np.ndarray:
    """float64 value of every one of the 2^bits codes, indexed by the code.

    Signed: code = (s << (bits-1)) | c and value = (-1)^s * magnitude(c)
    (Eq. 1); the pattern s=1, c=0 is +0.0.
    """
    m = magnitude_bits(bits, signed)
    mag = magnitude_table(m)
    if not signed:
        return mag.copy()
    neg = -mag
    neg[0] = 0.0
    return np.concatenate([mag, neg])


def codebook_exact(bits: int, signed: bool) -> list[Fraction]:
    m = magnitude_bits(bits, signed)
    mag = [magnitude_value_exact(c, m) for c in range(1 << m)]
    if not signed:
        return mag
    return mag + [-v for v in mag]


def midpoints(m: int) -> np.ndarray:
    """The 2^m - 1 decision points between consecutive magnitudes (dyadic, exact)."""
    v = magnitude_table(m)
    return (v[:-1] + v[1:]) * 0.5


# --------------------------------------------------------------------------
# Per-tensor scale ("adjust its precision at the tensor level", Sec. I)
# --------------------------------------------------------------------------
def absmax_scale(x: np.ndarray, bits: int, signed: bool) -> np.float32:
    """s = max|x| / 2^(m-1) as a float32; NaNs are ignored; an all-zero (or
    empty) tensor gets s = 1.  Dividing by a power of two is exact unless the
    quotient is subnormal."""
    x = np.asarray(x, dtype=np.float32).ravel()
    a = np.abs(x)
    a = a[~np.isnan(a)]
    mx = np.float32(a.max()) if a.size else np.float32(0)
    if mx == 0:
        return np.float32(1.0)
    return np.float32(np.float32(mx) / np.float32(vmax(bits, signed)))


# --------------------------------------------------------------------------
# Quantize: nearest code of the real quotient x / s
# --------------------------------------------------------------------------
def quantize(x: np.ndarray, scale, bits: int, signed: bool) -> np.ndarray:
    """Codes (uint8, one per element, unpacked) nearest to x in exact arithmetic.

    The represented real of code q is s * value(q).  Magnitude codes increase
    with their value, so the magnitude code is the rank of |x| among the
    thresholds T_j = s * mid_j.  Each T_j is exact in float64 (a 24-bit by at
    most 9-bit significand product) and |x| converts exactly, so every
    comparison below is exact.  A tie goes to the even magnitude code.
    NaN -> code 0; |x| >= s*vmax (including Inf) -> all-ones magnitude;
    negative x in an unsigned format -> code 0; a zero magnitude never carries
    the sign bit.
    """
    m = magnitude_bits(bits, signed)
    s = np.float32(scale)
    if not (np.isfinite(s) and s > 0):
        raise ValueError("scale must be a finite positive float32")
    x = np.asarray(x, dtype=np.float32)
    T = np.float64(s) * midpoints(m)                       # exact products
    ax = np.abs(x.astype(np.float64))                      # exact conversion
    nan = np.isnan(ax)
    ax = np.where(nan, 0.0, ax)
    rank = np.searchsorted(T, ax, side="left")             # #{j : T_j < |x|}
    at_tie = rank < T.size
    at_tie &= ax == T[np.minimum(rank, T.size - 1)]
    rank = np.where(at_tie & (rank % 2 == 1), rank + 1, rank)
    mag = rank.astype(np.int64)
    negative = np.signbit(x) & ~nan
    if signed:
        code = np.where(negative & (mag != 0), mag | (1 << (bits - 1)), mag)
    else:
        code = np.where(negative, 0, mag)
    code = np.where(nan, 0, code)
    return code.astype(np.uint8)


def quantize_bruteforce(x, scale, bits: int, signed: bool) -> list[int]:
    """Second, independent definition for tiny inputs: argmin over all codes of
    |x - s*value(q)| in exact rational arithmetic (pure Python)."""
    m = magnitude_bits(bits, signed)
    s = Fraction(float(np.float32(scale)))
    out = []
    for xv in np.asarray(x, dtype=np.float32).ravel().tolist():
        if xv != xv:
            out.append(0)
            continue
        if xv in (float("inf"), float("-inf")):
            neg = xv < 0
            if signed:
                out.append(((1 << m) - 1) | ((1 << (bits - 1)) if neg else 0))
            else:
                out.append(0 if neg else (1 << m) - 1)
            continue
        xf = Fraction(xv)
        best = None
        for s_bit in ((0, 1) if signed else (0,)):
            for c in range(1 << m):
                if s_bit == 1 and c == 0:
                    continue                      # never emitted
                v = magnitude_value_exact(c, m) * (-1 if s_bit else 1)
                err = abs(xf - s * v)
                key = (err, c % 2, c)             # nearest, then even magnitude code
                cand = (key, (s_bit << (bits - 1)) | c if signed else c)
                if best is None or cand[0] < best[0]:
                    best = cand
        out.append(best[1])
    return out


def dequantize(codes: np.ndarray, scale, bits: int, signed: bool) -> np.ndarray:
    """y = float32(s) * float32(value(code)): one correctly rounded multiply."""
    cb = codebook(bits, signed).astype(np.float32)
    return (np.float32(scale) * cb[np.asarray(codes, dtype=np.int64)]).astype(np.float32)


# --------------------------------------------------------------------------
# Packed storage
# --------------------------------------------------------------------------
def packed_bytes(n: int, bits: int) -> int:
    return (n * bits + 7) // 8


def pack(codes: np.ndarray, bits: int) -> np.ndarray:
    """Little-endian bit stream of `bits`-wide codes; tail bits are zero."""
    codes = np.asarray(codes, dtype=np.uint8).ravel()
    n = codes.size
    bitmat = ((codes[:, None] >> np.arange(bits, dtype=np.uint8)[None, :]) & 1).astype(np.uint8)
    stream = bitmat.ravel()
    pad = (-stream.size) % 8
    if pad:
        stream = np.concatenate([stream, np.zeros(pad, dtype=np.uint8)])
    out = np.packbits(stream, bitorder="little")
    assert out.size == packed_bytes(n, bits)
    return out


def unpack(buf: np.ndarray, n: int, bits: int) -> np.ndarray:
    stream = np.unpackbits(np.asarray(buf, dtype=np.uint8).ravel(), bitorder="little")
    stream = stream[: n * bits].reshape(n, bits)
    w = (1 << np.arange(bits)).astype(np.uint16)
    return (stream.astype(np.uint16) * w[None, :]).sum(axis=1).astype(np.uint8)


def pack_rows(codes2d: np.ndarray, bits: int) -> np.ndarray:
    """Pack each row separately (rows start byte-aligned)."""
    codes2d = np.asarray(codes2d, dtype=np.uint8)
    rows, k = codes2d.shape
    if (k * bits) % 8:
        raise ValueError("row length in bits must be a multiple of 8")
    return pack(codes2d.reshape(-1), bits).reshape(rows, k * bits // 8)


def unpack_rows(buf2d: np.ndarray, k: int, bits: int) -> np.ndarray:
    buf2d = np.asarray(buf2d, dtype=np.uint8)
    rows = buf2d.shape[0]
    return unpack(buf2d.reshape(-1), rows * k, bits).reshape(rows, k)


# --------------------------------------------------------------------------
# GEMM and convolution with FP accumulation (Sec. III-B architecture)
# --------------------------------------------------------------------------
def _decode_scaled_int(codes: np.ndarray, bits: int, signed: bool) -> np.ndarray:
    """value(code) * 2^(m-1) as exact integers held in float64."""
    m = magnitude_bits(bits, signed)
    cb = codebook(bits, signed) * float(1 << (m - 1))
    assert np.all(cb == np.rint(cb))
    return cb[np.asarray(codes, dtype=np.int64)]


def gemm(a_codes, a_fmt, a_scale, w_codes, w_fmt, w_scale, bias=None, relu=False, residual=None):
    """C[m,n] = sA*sW * sum_k value(A[m,k]) * value(W[n,k]) (+ bias[n]) (+ residual[m,n]) (ReLU).

    `residual` is the identity shortcut of the ResNet workloads of Sec. IV: an fp32 tensor of
    the output's shape added to the floating-point intermediate result before the ReLU (and
    before anything is written back).

    a_codes: [M][K] unpacked codes, w_codes: [N][K]; *_fmt = (bits, signed).  w_scale is one
    number (tensor-level precision, Sec. I) or N numbers, one per row of W (per-output-channel
    weight scales: column n of C then carries sW[n]).
    The sum is taken over exact integers (values times 2^(m-1)) in float64;
    every partial sum stays below 2^53, so the order of summation cannot matter.
    Returns (C float64, D float64) with D[m,n] = sA*sW*sum_k|a*w| (+|bias|), the tolerance
    denominator: the error bar of the product is stated relative to sum|a*w|; the bias joins it
    because it is added in the same rounding.  The shortcut does not: adding an exact fp32 input
    costs one more rounding of the result, which a test allows for separately (half an ulp of C).
    """
    ia = _decode_scaled_int(a_codes, *a_fmt)
    iw = _decode_scaled_int(w_codes, *w_fmt)
    ma = magnitude_bits(*a_fmt)
    mw = magnitude_bits(*w_fmt)
    sw = np.asarray(w_scale, dtype=np.float32).astype(np.float64)
    if sw.ndim not in (0, 1) or (sw.ndim == 1 and sw.size != iw.shape[0]):
        raise ValueError("w_scale is a scalar or one value per row of W")
    unit = np.float64(np.float32(a_scale)) * sw * 2.0 ** (-(ma - 1) - (mw - 1))     # scalar or [N]
    acc = ia @ iw.T
    den = np.abs(ia) @ np.abs(iw).T
    assert den.max(initial=0.0) < 2.0 ** 53
    c = acc * unit
    d = den * unit
    if bias is not None:
        b = np.asarray(bias, dtype=np.float32).astype(np.float64)
        c = c + b[None, :]
        d = d + np.abs(b)[None, :]
    if residual is not None:
        r = np.asarray(residual, dtype=np.float32).astype(np.float64).reshape(c.shape)
        c = c + r
    if relu:
        c = np.maximum(c, 0.0)
    return c, d


def gemm_loops(a_codes, a_fmt, a_scale, w_codes, w_fmt, w_scale, bias=None, relu=False):
    """The same contraction as three plain Python loops over exact Fractions
    (tiny shapes only)."""
    cba = codebook_exact(*a_fmt)
    cbw = codebook_exact(*w_fmt)
    a_codes = np.asarray(a_codes)
    w_codes = np.asarray(w_codes)
    M, K = a_codes.shape
    N = w_codes.shape[0]
    sa = Fraction(float(np.float32(a_scale)))
    sw = Fraction(float(np.float32(w_scale)))
    out = np.zeros((M, N), dtype=np.float64)
    for i in range(M):
        for j in range(N):
            acc = Fraction(0)
            for k in range(K):
                acc += cba[int(a_codes[i, k])] * cbw[int(w_codes[j, k])]
            acc = acc * sa * sw
            if bias is not None:
                acc += Fraction(float(np.float32(bias[j])))
            if relu and acc < 0:
                acc = Fraction(0)
            out[i, j] = float(acc)
    return out


def conv_out_size(h: int, k: int, stride: int, pad: int) -> int:
    return (h + 2 * pad - k) // stride + 1


def im2col(x_codes: np.ndarray, kh: int, kw: int, stride: int, pad: int) -> np.ndarray:
    """x_codes [B][H][W][C] -> [B*Ho*Wo][kh*kw*C]; taps outside the image read
    code 0, which is exactly 0.0 in every format."""
    x_codes = np.asarray(x_codes, dtype=np.uint8)
    B, H, W, C = x_codes.shape
    Ho = conv_out_size(H, kh, stride, pad)
    Wo = conv_out_size(W, kw, stride, pad)
    xp = np.zeros((B, H + 2 * pad, W + 2 * pad, C), dtype=np.uint8)
    xp[:, pad:pad + H, pad:pad + W, :] = x_codes
    cols = np.zeros((B, Ho, Wo, kh, kw, C), dtype=np.uint8)
    for r in range(kh):
        for s in range(kw):
            cols[:, :, :, r, s, :] = xp[:, r:r + stride * Ho:stride, s:s + stride * Wo:stride, :]
    return cols.reshape(B * Ho * Wo, kh * kw * C)


def conv2d(x_codes, x_fmt, x_scale, w_codes, w_fmt, w_scale, stride, pad,
           bias=None, relu=False, residual=None):
    """x_codes [B][H][W][Cin], w_codes [Cout][kh][kw][Cin] (unpacked codes); residual, if given,
    has the output's shape [B][Ho][Wo][Cout].
    Returns (Y float64 [B][Ho][Wo][Cout], D same shape)."""
    x_codes = np.asarray(x_codes, dtype=np.uint8)
    w_codes = np.asarray(w_codes, dtype=np.uint8)
    B, H, W, C = x_codes.shape
    Cout, kh, kw, C2 = w_codes.shape
    assert C == C2
    Ho = conv_out_size(H, kh, stride, pad)
    Wo = conv_out_size(W, kw, stride, pad)
    cols = im2col(x_codes, kh, kw, stride, pad)
    res = None if residual is None else np.asarray(residual, dtype=np.float32).reshape(B * Ho * Wo, Cout)
    c, d = gemm(cols, x_fmt, x_scale, w_codes.reshape(Cout, -1), w_fmt, w_scale, bias, relu, res)
    return c.reshape(B, Ho, Wo, Cout), d.reshape(B, Ho, Wo, Cout)


def dwconv2d(x_codes, x_fmt, x_scale, w_codes, w_fmt, w_scale, stride, pad, bias=None, relu=False):
    """Depthwise convolution (the layer type of the depthwise-separable network of Sec. IV): every
    channel is filtered on its own,
        Y[b,ho,wo,c] = sA*sW * sum_{r,s} value(X[b, ho*stride-pad+r, wo*stride-pad+s, c]) * value(Wt[r,s,c])
                       (+ bias[c]) (ReLU),
    taps outside the image contributing 0.  x_codes [B][H][W][C], w_codes [kh][kw][C] (unpacked
    codes, channel innermost like the image).  Exact integer sums as in gemm.
    Returns (Y float64 [B][Ho][Wo][C], D same shape: the tolerance denominator)."""
    x_codes = np.asarray(x_codes, dtype=np.uint8)
    w_codes = np.asarray(w_codes, dtype=np.uint8)
    B, H, W, C = x_codes.shape
    kh, kw, C2 = w_codes.shape
    assert C == C2
    Ho = conv_out_size(H, kh, stride, pad)
    Wo = conv_out_size(W, kw, stride, pad)
    ix = np.zeros((B, H + 2 * pad, W + 2 * pad, C), dtype=np.float64)
    ix[:, pad:pad + H, pad:pad + W, :] = _decode_scaled_int(x_codes, *x_fmt)
    iw = _decode_scaled_int(w_codes, *w_fmt)
    acc = np.zeros((B, Ho, Wo, C), dtype=np.float64)
    den = np.zeros((B, Ho, Wo, C), dtype=np.float64)
    for r in range(kh):
        for q in range(kw):
            win = ix[:, r:r + stride * Ho:stride, q:q + stride * Wo:stride, :]
            acc += win * iw[r, q, :]
            den += np.abs(win) * np.abs(iw[r, q, :])
    sw = np.asarray(w_scale, dtype=np.float32).astype(np.float64)            # one number, or one per channel
    if sw.ndim not in (0, 1) or (sw.ndim == 1 and sw.size != C):
        raise ValueError("w_scale is a scalar or one value per channel")
    unit = np.float64(np.float32(x_scale)) * sw * 2.0 ** (-(magnitude_bits(*x_fmt) - 1) - (magnitude_bits(*w_fmt) - 1))
    y, d = acc * unit, den * unit
    if bias is not None:
        b = np.asarray(bias, dtype=np.float32).astype(np.float64)
        y = y + b
        d = d + np.abs(b)
    if relu:
        y = np.maximum(y, 0.0)
    return y, d


def group_conv2d(x_codes, x_fmt, x_scale, w_codes, w_fmt, w_scale, stride, pad, groups,
                 bias=None, relu=False, residual=None):
    """Grouped convolution (the layer type between the dense and the depthwise convolution of the
    networks of Sec. IV): input channels and output channels are split into `groups` equal parts and
    part g of the output sees part g of the input only.  x_codes [B][H][W][Cin]; w_codes
    [Cout][kh][kw][Cin / groups]; output channel n belongs to group n // (Cout / groups).  w_scale is
    one number or one per output channel.  Written as the definition: one dense convolution per group
    on its channel slices, the results side by side.  Returns (Y, D) like conv2d."""
    x_codes = np.asarray(x_codes, dtype=np.uint8)
    w_codes = np.asarray(w_codes, dtype=np.uint8)
    B, H, W, Cin = x_codes.shape
    Cout, kh, kw, Cg = w_codes.shape
    if groups < 1 or Cin % groups or Cout % groups or Cg * groups != Cin:
        raise ValueError("groups must divide Cin and Cout, and the filters hold Cin / groups channels")
    Cog = Cout // groups
    sw = np.asarray(w_scale, dtype=np.float32)
    ys, ds = [], []
    for g in range(groups):
        n0, n1 = g * Cog, (g + 1) * Cog
        y, d = conv2d(x_codes[..., g * Cg:(g + 1) * Cg], x_fmt, x_scale, w_codes[n0:n1], w_fmt,
                      sw if sw.ndim == 0 else sw[n0:n1], stride, pad,
                      None if bias is None else np.asarray(bias)[n0:n1], relu,
                      None if residual is None else np.asarray(residual)[..., n0:n1])
        ys.append(y)
        ds.append(d)
    return np.concatenate(ys, axis=-1), np.concatenate(ds, axis=-1)


# --------------------------------------------------------------------------
# Quantization error metric (Eq. 2)
# --------------------------------------------------------------------------
def maxpool2d_codes(x_codes: np.ndarray, bits: int, signed: bool, k: int, stride: int, pad: int) -> np.ndarray:
    """Max pooling of a tensor of DyBit codes [B][H][W][C] (Sec. III-B: activations are stored as codes):
    per window and channel the code whose value is largest, taps outside the image left out; the value zero
    is reported as code 0.  Plain loops over windows."""
    cb = codebook(bits, signed)
    canon = {float(v): c for c, v in reversed(list(enumerate(cb)))}      # smallest code of every value
    Bn, H, W, C = x_codes.shape
    Ho, Wo = conv_out_size(H, k, stride, pad), conv_out_size(W, k, stride, pad)
    vals = cb[np.asarray(x_codes, dtype=np.int64)]
    out = np.zeros((Bn, Ho, Wo, C), dtype=np.uint8)
    for ho in range(Ho):
        for wo in range(Wo):
            r0, s0 = ho * stride - pad, wo * stride - pad
            win = vals[:, max(r0, 0):min(r0 + k, H), max(s0, 0):min(s0 + k, W), :]
            best = win.reshape(Bn, -1, C).max(axis=1)
            out[:, ho, wo, :] = np.vectorize(canon.__getitem__, otypes=[np.uint8])(best)
    return out


def rmse(x: np.ndarray, xq: np.ndarray) -> float:
    """sqrt(mean(((x - xq)/sigma)^2)), sigma = standard deviation of x (Eq. 2)."""
    x = np.asarray(x, dtype=np.float64).ravel()
    xq = np.asarray(xq, dtype=np.float64).ravel()
    sigma = x.std()
    return float(np.sqrt(np.mean(((x - xq) / sigma) ** 2)))


def quantization_rmse(x: np.ndarray, scale, bits: int, signed: bool) -> float:
    """Eq. 2 for one tensor in one DyBit format: x_hat = s * value(code of x) with the product taken
    in float64 (the quantized value itself, Sec. III-A, not its float32 rounding), sigma the standard
    deviation of x (one value for the whole tensor, population form)."""
    x = np.asarray(x, dtype=np.float32).ravel()
    codes = quantize(x, scale, bits, signed)
    x_hat = np.float64(np.float32(scale)) * codebook(bits, signed)[np.asarray(codes, dtype=np.int64)]
    return rmse(x, x_hat)


def quantize_rows(x2d: np.ndarray, bits: int, signed: bool):
    """Per-row (per-output-channel) max-abs scales and codes of a weight matrix [rows][cols]:
    absmax_scale and quantize applied to every row on its own.  Returns (scales float32 [rows],
    codes [rows][cols])."""
    x2d = np.asarray(x2d, dtype=np.float32)
    scales = np.array([absmax_scale(row, bits, signed) for row in x2d], dtype=np.float32)
    codes = np.stack([quantize(row, scales[i], bits, signed) for i, row in enumerate(x2d)]) if len(x2d) else \
        np.zeros(x2d.shape, dtype=np.uint8)
    return scales, codes


def quantize_cols(x2d: np.ndarray, bits: int, signed: bool):
    """Per-column max-abs scales and codes of a matrix [rows][cols]: the per-channel scales of a
    depthwise filter, whose layout [kh*kw][C] has the channel innermost.  absmax_scale and quantize
    applied to every column on its own.  Returns (scales float32 [cols], codes [rows][cols])."""
    x2d = np.asarray(x2d, dtype=np.float32)
    scales, codes = quantize_rows(np.ascontiguousarray(x2d.T), bits, signed)
    return scales, np.ascontiguousarray(codes.T)


def fake_quant_grad(x: np.ndarray, grad: np.ndarray, scale, bits: int, signed: bool) -> np.ndarray:
    """Backward of the quantize-then-decode operator of the fine-tuning step (Sec. III-C) under the
    straight-through estimator: the rounding is treated as the identity and the saturation as the
    clamp it is, so d x_hat / d x = 1 where x lies inside the representable range
    [-s vmax, s vmax] (unsigned formats: [0, s vmax]), bounds included, and 0 outside (and for NaN).
    Returns grad * mask as float32."""
    x = np.asarray(x, dtype=np.float32)
    g = np.asarray(grad, dtype=np.float32)
    hi = np.float64(np.float32(scale)) * vmax(bits, signed)
    lo = -hi if signed else 0.0
    xd = x.astype(np.float64)
    inside = (xd >= lo) & (xd <= hi)                                         # False for NaN
    return np.where(inside, g, np.float32(0.0)).astype(np.float32)

