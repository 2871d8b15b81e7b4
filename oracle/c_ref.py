"""ctypes front end of the plain C oracle (dybit_ref.c).  TEST INFRASTRUCTURE ONLY."""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dybit_ref.c")
_LIB = os.path.join(_HERE, "libdybit_ref.so")
_lib = None


def build(force: bool = True) -> str:
    """Compile dybit_ref.c with gcc (-O2, OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build(force=False)
        L = C.CDLL(_LIB)
        L.ref_magnitude.restype = C.c_double
        L.ref_magnitude.argtypes = [C.c_int, C.c_int]
        L.ref_num_threads.restype = C.c_int
        L.ref_absmax_scale.restype = C.c_float
        L.ref_absmax_scale.argtypes = [C.c_void_p, C.c_size_t, C.c_int, C.c_int]
        L.ref_codebook.argtypes = [C.c_int, C.c_int, C.c_void_p]
        L.ref_quantize.argtypes = [C.c_void_p, C.c_size_t, C.c_float, C.c_int, C.c_int, C.c_void_p]
        L.ref_dequantize.argtypes = [C.c_void_p, C.c_size_t, C.c_float, C.c_int, C.c_int, C.c_void_p]
        L.ref_pack.argtypes = [C.c_void_p, C.c_size_t, C.c_int, C.c_void_p]
        L.ref_unpack.argtypes = [C.c_void_p, C.c_size_t, C.c_int, C.c_void_p]
        L.ref_gemm.argtypes = [C.c_longlong] * 3 + \
            [C.c_void_p, C.c_int, C.c_int, C.c_float] * 2 + \
            [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
        L.ref_conv2d.argtypes = [C.c_longlong] * 5 + [C.c_int] * 4 + \
            [C.c_void_p, C.c_int, C.c_int, C.c_float] * 2 + \
            [C.c_void_p, C.c_int, C.c_void_p, C.c_void_p]
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def num_threads() -> int:
    return lib().ref_num_threads()


def codebook(bits: int, signed: bool) -> np.ndarray:
    out = np.zeros(1 << bits, dtype=np.float64)
    lib().ref_codebook(bits, int(signed), _p(out))
    return out


def absmax_scale(x: np.ndarray, bits: int, signed: bool) -> np.float32:
    x = np.ascontiguousarray(x, dtype=np.float32).ravel()
    return np.float32(lib().ref_absmax_scale(_p(x), x.size, bits, int(signed)))


def quantize(x: np.ndarray, scale, bits: int, signed: bool) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint8)
    lib().ref_quantize(_p(x), x.size, float(np.float32(scale)), bits, int(signed), _p(out))
    return out


def dequantize(codes: np.ndarray, scale, bits: int, signed: bool) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    out = np.empty(codes.shape, dtype=np.float32)
    lib().ref_dequantize(_p(codes), codes.size, float(np.float32(scale)), bits, int(signed), _p(out))
    return out


def pack(codes: np.ndarray, bits: int) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.uint8).ravel()
    out = np.empty((codes.size * bits + 7) // 8, dtype=np.uint8)
    lib().ref_pack(_p(codes), codes.size, bits, _p(out))
    return out


def unpack(buf: np.ndarray, n: int, bits: int) -> np.ndarray:
    buf = np.ascontiguousarray(buf, dtype=np.uint8).ravel()
    out = np.empty(n, dtype=np.uint8)
    lib().ref_unpack(_p(buf), n, bits, _p(out))
    return out


def gemm(a_codes, a_fmt, a_scale, w_codes, w_fmt, w_scale, bias=None, relu=False, want_den=True):
    a = np.ascontiguousarray(a_codes, dtype=np.uint8)
    w = np.ascontiguousarray(w_codes, dtype=np.uint8)
    M, K = a.shape
    N = w.shape[0]
    assert w.shape[1] == K
    c = np.empty((M, N), dtype=np.float64)
    d = np.empty((M, N), dtype=np.float64) if want_den else None
    b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float32)
    lib().ref_gemm(M, N, K, _p(a), a_fmt[0], int(a_fmt[1]), float(np.float32(a_scale)),
                   _p(w), w_fmt[0], int(w_fmt[1]), float(np.float32(w_scale)),
                   _p(b), int(relu), _p(c), _p(d))
    return c, d


def conv2d(x_codes, x_fmt, x_scale, w_codes, w_fmt, w_scale, stride, pad,
           bias=None, relu=False, want_den=True):
    x = np.ascontiguousarray(x_codes, dtype=np.uint8)
    w = np.ascontiguousarray(w_codes, dtype=np.uint8)
    B, H, W, Cin = x.shape
    Cout, kh, kw, _ = w.shape
    Ho = (H + 2 * pad - kh) // stride + 1
    Wo = (W + 2 * pad - kw) // stride + 1
    y = np.empty((B, Ho, Wo, Cout), dtype=np.float64)
    d = np.empty((B, Ho, Wo, Cout), dtype=np.float64) if want_den else None
    b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float32)
    lib().ref_conv2d(B, H, W, Cin, Cout, kh, kw, stride, pad,
                     _p(x), x_fmt[0], int(x_fmt[1]), float(np.float32(x_scale)),
                     _p(w), w_fmt[0], int(w_fmt[1]), float(np.float32(w_scale)),
                     _p(b), int(relu), _p(y), _p(d))
    return y, d
