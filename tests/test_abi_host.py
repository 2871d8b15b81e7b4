"""The C-ABI library loads, exports what include/dybit.h declares, and rejects bad
arguments on the host before touching a GPU.  CPU only: no compute entry point is
called with valid arguments here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from oracle import dybit_ref as R
from paper_2302_12510_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "dybit.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dybit_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert {"dybit_codebook", "dybit_quantize", "dybit_dequantize", "dybit_gemm", "dybit_conv2d"} <= set(names)
    L = B.lib()
    for n in names:
        assert hasattr(L, n), n


@pytest.mark.parametrize("bits", [2, 4, 6, 8])
@pytest.mark.parametrize("signed", [True, False])
def test_codebook_matches_oracle(bits, signed):
    got = B.dybit_codebook(bits, signed)
    want = R.codebook(bits, signed)
    assert got.dtype == np.float32 and got.size == 1 << bits
    assert np.array_equal(got.astype(np.float64), want)
    assert not np.signbit(got[1 << (bits - 1)]) or not signed


def test_packed_bytes():
    for bits in (2, 4, 6, 8):
        for n in (0, 1, 3, 4, 5, 1000, 2 ** 28):
            assert B.dybit_packed_bytes(bits, True, n) == R.packed_bytes(n, bits)
    assert B.dybit_packed_bytes(5, True, 10) == 0


def test_status_strings():
    seen = {B.status_string(s) for s in range(7)}
    assert len(seen) == 7 and "ok" in seen


def _st(fn, *args):
    return fn(*args)


def test_argument_errors_without_gpu():
    L = B.lib()
    f4, f8, bad = B.fmt(4, True), B.fmt(8, False), B.fmt(5, True)
    p = C.c_void_p(0x1000)          # never dereferenced: all calls below fail validation first
    odd = C.c_void_p(0x1004)
    null = C.c_void_p(0)
    # codebook
    buf = (C.c_float * 256)()
    assert L.dybit_codebook(bad, buf, None) == B.ERR_UNSUPPORTED_BITS
    assert L.dybit_codebook(B.Fmt(4, 2), buf, None) == B.ERR_INVALID_ARG
    assert L.dybit_codebook(f4, None, None) == B.ERR_NULL
    # quantize / dequantize / absmax
    assert L.dybit_quantize(p, 16, bad, p, p, None) == B.ERR_UNSUPPORTED_BITS
    assert L.dybit_quantize(null, 16, f4, p, p, None) == B.ERR_NULL
    assert L.dybit_quantize(p, 16, f4, null, p, None) == B.ERR_NULL
    assert L.dybit_quantize(odd, 16, f4, p, p, None) == B.ERR_ALIGNMENT
    assert L.dybit_quantize(p, 16, f4, p, odd, None) == B.ERR_ALIGNMENT
    assert L.dybit_dequantize(p, 16, bad, p, p, None) == B.ERR_UNSUPPORTED_BITS
    assert L.dybit_dequantize(null, 16, f8, p, p, None) == B.ERR_NULL
    assert L.dybit_dequantize(p, 16, f8, p, odd, None) == B.ERR_ALIGNMENT
    assert L.dybit_absmax_scale(p, 16, bad, p, None) == B.ERR_UNSUPPORTED_BITS
    assert L.dybit_absmax_scale(p, 16, f4, null, None) == B.ERR_NULL
    assert L.dybit_absmax_scale(odd, 16, f4, p, None) == B.ERR_ALIGNMENT
    # gemm
    g = lambda M, N, K, fa=f4, fw=f4, a=p, w=p, sa=p, sw=p, relu=0, c=p, ldc=None: \
        L.dybit_gemm(M, N, K, a, fa, sa, w, fw, sw, null, relu, c, N if ldc is None else ldc, None)
    assert g(8, 8, 16, fa=bad) == B.ERR_UNSUPPORTED_BITS
    assert g(-1, 8, 16) == B.ERR_INVALID_ARG
    assert g(8, 8, 16, ldc=4) == B.ERR_INVALID_ARG
    assert g(8, 8, 16, relu=3) == B.ERR_INVALID_ARG
    assert g(8, 8, 15) == B.ERR_ALIGNMENT                        # 15 nibbles: row not byte-aligned
    assert g(8, 8, 6, fa=B.fmt(6, True)) == B.ERR_ALIGNMENT      # 36 bits
    assert g(8, 8, 16, a=null) == B.ERR_NULL
    assert g(8, 8, 16, sa=null) == B.ERR_NULL
    assert g(8, 8, 16, c=null) == B.ERR_NULL
    assert g(0, 8, 16, a=null, w=null, c=null) == B.OK           # empty problem: nothing to do
    # conv2d
    cv = lambda Bn=1, H=8, W=8, Cin=16, Cout=8, kh=3, kw=3, s=1, pd=1, fx=f4, fw=f4, x=p, y=p: \
        L.dybit_conv2d(Bn, H, W, Cin, Cout, kh, kw, s, pd, x, fx, p, p, fw, p, null, 0, y, None)
    assert cv(fx=bad) == B.ERR_UNSUPPORTED_BITS
    assert cv(s=0) == B.ERR_INVALID_ARG
    assert cv(H=2, kh=7, pd=0) == B.ERR_INVALID_ARG
    assert cv(Cin=3) == B.ERR_ALIGNMENT                          # 12 bits per pixel
    assert cv(x=null) == B.ERR_NULL
    assert cv(Bn=0, x=null, y=null) == B.OK
    # the extended variants: the same checks; shortcut and running maximum are optional
    assert L.dybit_gemm_ex(8, 8, 16, p, f4, p, p, f4, p, null, null, 0, null, 8, null, None) == B.ERR_NULL
    assert L.dybit_gemm_ex(8, 8, 15, p, f4, p, p, f4, p, null, p, 0, p, 8, p, None) == B.ERR_ALIGNMENT
    assert L.dybit_gemm_ex(0, 8, 16, null, f4, p, null, f4, p, null, null, 0, null, 8, null, None) == B.OK
    assert L.dybit_conv2d_ex(1, 8, 8, 16, 8, 3, 3, 1, 1, null, f4, p, p, f4, p, null, null, 0, p, null, None) == B.ERR_NULL
    assert L.dybit_conv2d_ex(1, 8, 8, 16, 8, 3, 3, 0, 1, p, f4, p, p, f4, p, null, p, 0, p, p, None) == B.ERR_INVALID_ARG
    # the write-back variants: output format, whole words per row, at least one output
    f6, f2 = B.fmt(6, False), B.fmt(2, True)
    wb = lambda N=8, c=p, cf=f4, cs=p, cc=p: \
        L.dybit_gemm_wb(8, N, 16, p, f4, p, p, f4, p, null, null, 0, c, N, null, cf, cs, cc, None)
    assert wb(cf=f2) == B.ERR_UNSUPPORTED_BITS                   # the epilogue packs 4-, 6- and 8-bit codes
    assert wb(cf=bad) == B.ERR_UNSUPPORTED_BITS
    assert wb(cf=f6) == B.ERR_ALIGNMENT                          # 8 codes of 6 bits: a row is not whole words
    assert wb(N=4) == B.ERR_ALIGNMENT                            # 16 bits per row
    assert wb(cc=C.c_void_p(p.value + 1)) == B.ERR_ALIGNMENT
    assert wb(c=null, cc=null) == B.ERR_NULL
    assert wb(cs=null) == B.ERR_NULL
    assert L.dybit_conv2d_wb(1, 8, 8, 16, 8, 3, 3, 1, 1, p, f4, p, p, f4, p, null, null, 0, null, null,
                             f4, p, null, None) == B.ERR_NULL
    assert L.dybit_conv2d_wb(1, 8, 8, 16, 12, 3, 3, 1, 1, p, f4, p, p, f4, p, null, null, 0, p, null,
                             f4, p, p, None) == B.ERR_ALIGNMENT
    p2 = C.c_void_p(0x2000)
    assert L.dybit_quantize_absmax(p, 64, f4, null, p2, p, None) == B.ERR_NULL
    assert L.dybit_quantize_absmax(p, 64, f4, p, p, p, None) == B.ERR_INVALID_ARG     # maximum and scale in one word
    assert L.dybit_quantize_absmax(p, 64, bad, p, p2, p, None) == B.ERR_UNSUPPORTED_BITS
    assert L.dybit_quantize_absmax(C.c_void_p(0x1004), 64, f4, p, p2, p, None) == B.ERR_ALIGNMENT
    assert L.dybit_scale_from_absmax(null, f4, p, None) == B.ERR_NULL
    assert L.dybit_scale_from_absmax(p, bad, p, None) == B.ERR_UNSUPPORTED_BITS
    assert L.dybit_get_last_async_error(None, None) == B.ERR_NULL


def test_rmse_argument_errors_without_gpu():
    L = B.lib()
    f4, bad = B.fmt(4, True), B.fmt(3, False)
    p, null = C.c_void_p(0x1000), C.c_void_p(0)
    assert L.dybit_rmse(p, 64, bad, p, p, None) == B.ERR_UNSUPPORTED_BITS
    assert L.dybit_rmse(null, 64, f4, p, p, None) == B.ERR_NULL
    assert L.dybit_rmse(p, 64, f4, null, p, None) == B.ERR_NULL
    assert L.dybit_rmse(p, 64, f4, p, null, None) == B.ERR_NULL
    assert L.dybit_rmse(p, 0, f4, p, p, None) == B.ERR_INVALID_ARG
    assert L.dybit_rmse(C.c_void_p(0x1004), 64, f4, p, p, None) == B.ERR_ALIGNMENT
    assert L.dybit_rmse(p, 64, f4, p, C.c_void_p(0x1004), None) == B.ERR_ALIGNMENT
    assert L.dybit_fake_quant(p, 64, bad, p, p, None) == B.ERR_UNSUPPORTED_BITS
    assert L.dybit_fake_quant(null, 64, f4, p, p, None) == B.ERR_NULL
    assert L.dybit_fake_quant(p, 64, f4, null, p, None) == B.ERR_NULL
    assert L.dybit_fake_quant(p, 64, f4, p, C.c_void_p(0x1008), None) == B.ERR_ALIGNMENT
    assert L.dybit_fake_quant(null, 0, f4, p, null, None) == B.OK


# ---- the search is host code: checked in full against the oracle here ---------------------------------
from oracle import search_ref as S  # noqa: E402
from test_oracle_search import LAT, ERR, random_tables  # noqa: E402

STRATEGY = {"speedup": B.SEARCH_SPEEDUP, "rmse": B.SEARCH_RMSE}


def test_search_hand_traces():
    """The runs traced by hand in the oracle's tests (Alg. 1)."""
    assert B.dybit_search(LAT, ERR, ERR, B.SEARCH_SPEEDUP, 2.0, 2)[:2] == ([4, 4, 8], [8, 4, 8])
    assert B.dybit_search(LAT, ERR, ERR, B.SEARCH_SPEEDUP, 3.0, 2)[:2] == ([4, 4, 4], [4, 4, 8])
    assert B.dybit_search(LAT, ERR, ERR, B.SEARCH_RMSE, 5.0, 2)[:2] == ([4, 4, 8], [4, 4, 8])
    assert B.dybit_search(LAT, ERR, ERR, B.SEARCH_RMSE, 2.5, 1)[:2] == ([8, 4, 8], [8, 4, 8])


@pytest.mark.parametrize("seed", range(12))
def test_search_matches_oracle(seed):
    """Same tables, same sums in the same order: widths, ratio and verdict are identical, not close."""
    rng = np.random.default_rng(500 + seed)
    n = int(rng.integers(1, 40))
    lat, ew, ea = random_tables(rng, n)
    if seed % 3 == 0:                                   # ties: equal layers must come out in index order
        lat[n // 2:] = [lat[0]] * (n - n // 2)
        ew[n // 2:] = [ew[0]] * (n - n // 2)
    for strategy in ("speedup", "rmse"):
        for constraint in (0.7, 1.0, 1.2, 2.0, 3.5, 8.0, 1e6):
            for k in (1, 2, 5, n, n + 3):
                want = S.search(lat, ew, ea, strategy, constraint, k)
                got = B.dybit_search(lat, ew, ea, STRATEGY[strategy], constraint, k)
                assert got == tuple(want), (strategy, constraint, k)


def test_search_argument_errors():
    L = B.lib()
    n = 3
    lat = np.ones((n, 3, 3))
    e = np.ones((n, 3))
    w = np.zeros(n, dtype=np.int32)
    vp = lambda a: a.ctypes.data_as(C.c_void_p)
    call = lambda n_=n, lat_=lat, ew=e, ea=e, strat=0, c=2.0, k=1, wo=w, ao=w: L.dybit_search(
        n_, vp(lat_) if lat_ is not None else None, vp(ew) if ew is not None else None, vp(ea) if ea is not None else None,
        strat, c, k, vp(wo) if wo is not None else None, vp(ao) if ao is not None else None, None, None)
    assert call() == B.OK
    assert call(lat_=None) == B.ERR_NULL and call(ew=None) == B.ERR_NULL and call(wo=None) == B.ERR_NULL
    assert call(n_=0) == B.ERR_INVALID_ARG and call(k=0) == B.ERR_INVALID_ARG and call(strat=2) == B.ERR_INVALID_ARG
    assert call(c=float("nan")) == B.ERR_INVALID_ARG
    bad = lat.copy(); bad[1, 2, 0] = 0.0
    assert call(lat_=bad) == B.ERR_INVALID_ARG
    bad = lat.copy(); bad[0, 0, 0] = float("inf")
    assert call(lat_=bad) == B.ERR_INVALID_ARG
    neg = e.copy(); neg[2, 1] = -1e-9
    assert call(ea=neg) == B.ERR_INVALID_ARG
    assert call(ew=np.zeros((n, 3)), ea=np.zeros((n, 3)), strat=1) == B.ERR_INVALID_ARG     # zero error at (8, 8)


def test_per_channel_argument_errors_without_gpu():
    L = B.lib()
    f4, f6, bad = B.fmt(4, True), B.fmt(6, True), B.fmt(5, True)
    p, null = C.c_void_p(0x1000), C.c_void_p(0)
    assert L.dybit_quantize_rows(p, 4, 16, bad, p, p, None) == B.ERR_UNSUPPORTED_BITS
    assert L.dybit_quantize_rows(p, -1, 16, f4, p, p, None) == B.ERR_INVALID_ARG
    assert L.dybit_quantize_rows(p, 4, 3, f4, p, p, None) == B.ERR_ALIGNMENT          # a row of 12 bits
    assert L.dybit_quantize_rows(p, 4, 6, f6, p, p, None) == B.ERR_ALIGNMENT          # a row of 36 bits
    assert L.dybit_quantize_rows(p, 4, 16, f4, null, p, None) == B.ERR_NULL
    assert L.dybit_quantize_rows(null, 4, 16, f4, p, p, None) == B.ERR_NULL
    assert L.dybit_quantize_rows(null, 0, 16, f4, null, null, None) == B.OK
    pc = lambda w=p, c=p, cc=null, cf=f4: L.dybit_gemm_pc(8, 8, 16, p, f4, p, p, f4, w, null, null, 0, c, 8, null, cf, p, cc, None)
    assert pc(w=null) == B.ERR_NULL
    assert pc(c=null) == B.ERR_NULL                                                    # no codes asked for: fp32 output required
    assert pc(cc=p, cf=B.fmt(2, True)) == B.ERR_UNSUPPORTED_BITS
    assert pc(cc=p, cf=f6) == B.ERR_ALIGNMENT
    assert L.dybit_conv2d_pc(1, 8, 8, 16, 8, 3, 3, 1, 1, p, f4, p, p, f4, null, null, null, 0, p, null,
                             f4, p, null, None) == B.ERR_NULL


def test_dwconv_argument_errors_without_gpu():
    L = B.lib()
    f4, f6 = B.fmt(4, True), B.fmt(6, True)
    p, null = C.c_void_p(0x1000), C.c_void_p(0)
    dw = lambda Cn=32, xf=f4, wf=f4, k=3, st=1, x=p, y=p, bias=null: L.dybit_dwconv2d(
        1, 8, 8, Cn, k, k, st, 1, x, xf, p, p, wf, p, bias, 0, y, null, None)
    assert dw(xf=f6) == B.ERR_UNSUPPORTED_BITS and dw(wf=f6) == B.ERR_UNSUPPORTED_BITS
    assert dw(Cn=4) == B.ERR_ALIGNMENT
    assert dw(k=9, st=4) == B.ERR_INVALID_ARG
    assert dw(st=0) == B.ERR_INVALID_ARG
    assert dw(x=null) == B.ERR_NULL and dw(y=null) == B.ERR_NULL
    assert dw(bias=C.c_void_p(0x1004)) == B.ERR_ALIGNMENT
    assert dw(Cn=0) == B.OK



def test_code_chain_argument_errors_without_gpu():
    """Shortcut as codes, pooling on codes, caller-owned error word: refusals on the host."""
    L = B.lib()
    f2, f4, f6, f8 = B.fmt(2, False), B.fmt(4, False), B.fmt(6, False), B.fmt(8, True)
    p, null = C.c_void_p(0x1000), C.c_void_p(0)
    rc = lambda r=p, rf=f4, rs=p, codes=p, N=64: L.dybit_gemm_wb_rc(64, N, 64, p, f4, p, p, f8, p, null, r, rf, rs, 1,
                                                                     null, N, null, f4, p, codes, None)
    assert rc(rf=f2) == B.ERR_UNSUPPORTED_BITS
    assert rc(r=null) == B.ERR_NULL and rc(rs=null) == B.ERR_NULL and rc(codes=null) == B.ERR_NULL
    pool = lambda Cn=8, f=f4, k=3, st=2, pad=1, x=p, y=p: L.dybit_maxpool2d_codes(1, 8, 8, Cn, k, st, pad, x, f, y, None)
    assert pool(f=f6) == B.ERR_UNSUPPORTED_BITS
    assert pool(Cn=4) == B.ERR_ALIGNMENT and pool(x=C.c_void_p(0x1002)) == B.ERR_ALIGNMENT
    assert pool(pad=2) == B.ERR_INVALID_ARG and pool(st=0) == B.ERR_INVALID_ARG and pool(k=20, pad=3) == B.ERR_INVALID_ARG
    assert pool(x=null) == B.ERR_NULL and pool(y=null) == B.ERR_NULL
    assert L.dybit_set_async_error_word(C.c_void_p(0x1002)) == B.ERR_ALIGNMENT
    assert L.dybit_set_async_error_word(null) == B.OK
