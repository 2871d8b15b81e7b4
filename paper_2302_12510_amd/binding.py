"""Thin ctypes binding of libdybit.so: argument marshalling only.

PyTorch-ROCm supplies device memory and streams; every step of the path runs in the
library's HIP kernels.  Loading fails loudly when the library has not been built: there is
no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os

import torch  # imported first so that the library binds to the HIP runtime torch already loaded

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdybit.so")

OK = 0
ERR_INVALID_ARG, ERR_UNSUPPORTED_BITS, ERR_BAD_SCALE, ERR_ALIGNMENT, ERR_NULL, ERR_HIP = 1, 2, 3, 4, 5, 6


class Fmt(C.Structure):
    _fields_ = [("bits", C.c_int32), ("is_signed", C.c_int32)]


class DybitError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with "
                              "`python -m paper_2302_12510_amd.build` (needs hipcc); there is no fallback")
        L = C.CDLL(LIB_PATH)
        vp, sz, i32, i64 = C.c_void_p, C.c_size_t, C.c_int32, C.c_int64
        L.dybit_codebook.argtypes = [Fmt, vp, C.POINTER(i32)]
        L.dybit_packed_bytes.argtypes = [Fmt, sz]
        L.dybit_packed_bytes.restype = sz
        L.dybit_status_string.argtypes = [C.c_int]
        L.dybit_status_string.restype = C.c_char_p
        L.dybit_absmax_scale.argtypes = [vp, sz, Fmt, vp, vp]
        L.dybit_quantize.argtypes = [vp, sz, Fmt, vp, vp, vp]
        L.dybit_dequantize.argtypes = [vp, sz, Fmt, vp, vp, vp]
        L.dybit_quantize_absmax.argtypes = [vp, sz, Fmt, vp, vp, vp, vp]
        L.dybit_gemm.argtypes = [i64, i64, i64, vp, Fmt, vp, vp, Fmt, vp, vp, i32, vp, i64, vp]
        L.dybit_conv2d.argtypes = [i64] * 5 + [i32] * 4 + [vp, Fmt, vp, vp, Fmt, vp, vp, i32, vp, vp]
        L.dybit_gemm_ex.argtypes = [i64, i64, i64, vp, Fmt, vp, vp, Fmt, vp, vp, vp, i32, vp, i64, vp, vp]
        L.dybit_conv2d_ex.argtypes = [i64] * 5 + [i32] * 4 + [vp, Fmt, vp, vp, Fmt, vp, vp, vp, i32, vp, vp, vp]
        L.dybit_gemm_wb.argtypes = [i64, i64, i64, vp, Fmt, vp, vp, Fmt, vp, vp, vp, i32, vp, i64, vp, Fmt, vp, vp, vp]
        L.dybit_conv2d_wb.argtypes = [i64] * 5 + [i32] * 4 + [vp, Fmt, vp, vp, Fmt, vp, vp, vp, i32, vp, vp, Fmt, vp, vp, vp]
        L.dybit_gemm_wb_rc.argtypes = [i64, i64, i64, vp, Fmt, vp, vp, Fmt, vp, vp, vp, Fmt, vp, i32, vp, i64, vp, Fmt, vp, vp, vp]
        L.dybit_conv2d_wb_rc.argtypes = [i64] * 5 + [i32] * 4 + [vp, Fmt, vp, vp, Fmt, vp, vp, vp, Fmt, vp, i32, vp, vp, Fmt, vp, vp, vp]
        L.dybit_maxpool2d_codes.argtypes = [i64] * 4 + [i32] * 3 + [vp, Fmt, vp, vp]
        L.dybit_quantize_pad.argtypes = [vp, i64, i64, i64, Fmt, vp, vp, vp]
        L.dybit_scale_from_absmax.argtypes = [vp, Fmt, vp, vp]
        L.dybit_quantize_rows.argtypes = [vp, i64, i64, Fmt, vp, vp, vp]
        L.dybit_dwconv2d.argtypes = [i64] * 4 + [i32] * 4 + [vp, Fmt, vp, vp, Fmt, vp, vp, i32, vp, vp, vp]
        L.dybit_gemm_pc.argtypes = L.dybit_gemm_wb.argtypes
        L.dybit_conv2d_pc.argtypes = L.dybit_conv2d_wb.argtypes
        L.dybit_rmse.argtypes = [vp, sz, Fmt, vp, vp, vp]
        L.dybit_fake_quant.argtypes = [vp, sz, Fmt, vp, vp, vp]
        L.dybit_fake_quant_bwd.argtypes = [vp, vp, sz, Fmt, vp, vp, vp]
        L.dybit_quantize_cols.argtypes = [vp, i64, i64, Fmt, vp, vp, vp]
        L.dybit_dwconv2d_wb.argtypes = [i64] * 4 + [i32] * 4 + [vp, Fmt, vp, vp, Fmt, vp, i32, vp, i32, vp, vp, Fmt, vp, vp, vp]
        L.dybit_group_conv2d.argtypes = [i64] * 5 + [i32] * 5 + [vp, Fmt, vp, vp, Fmt, vp, i32, vp, vp, i32, vp, vp, vp]
        L.dybit_search.argtypes = [i32, vp, vp, vp, i32, C.c_double, i32, vp, vp, C.POINTER(C.c_double), C.POINTER(i32)]
        L.dybit_get_last_async_error.argtypes = [C.POINTER(i32), vp]
        L.dybit_set_async_error_word.argtypes = [vp]
        L.dybit_last_gemm_kernel.argtypes = []
        L.dybit_last_gemm_kernel.restype = i32
        L.dybit_set_option.argtypes = [C.c_char_p, C.c_char_p]
        L.dybit_diag_mfma_f16.argtypes = [vp, i32, i32, vp, C.POINTER(C.c_double), vp]
        L.dybit_diag_mfma_f8.argtypes = [vp, i32, i32, vp, C.POINTER(C.c_double), vp]
        _lib = L
    return _lib


def fmt(bits: int, signed: bool) -> Fmt:
    return Fmt(int(bits), int(bool(signed)))


def status_string(status: int) -> str:
    return lib().dybit_status_string(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != OK:
        raise DybitError(status, where)


def _stream(stream=None) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream)


def _ptr(t) -> int | None:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("expected a device tensor")
    if not t.is_contiguous():
        raise ValueError("expected a contiguous tensor")
    return t.data_ptr()


# ---- host-only --------------------------------------------------------------
KERNEL_NAMES = ("none", "general", "f16_256", "f16_128_kg1", "f16_128_kg2", "f16_128_rows", "f16_ws",
                "f8_256", "f8_128_kg1", "f8_128_kg2", "f8_64", "f8_ws")


def dybit_last_gemm_kernel() -> str:
    """Name (KERNEL_NAMES) of the kernel this thread's last matrix-product call launched."""
    return KERNEL_NAMES[lib().dybit_last_gemm_kernel()]


def dybit_set_option(name: str, value: str = "auto") -> None:
    _check(lib().dybit_set_option(name.encode(), value.encode()), "dybit_set_option")


def dybit_codebook(bits: int, signed: bool):
    """numpy float32 array of the 2^bits code values."""
    import numpy as np
    out = np.zeros(1 << max(bits, 0) if 0 <= bits <= 8 else 1, dtype=np.float32)
    cnt = C.c_int32(0)
    _check(lib().dybit_codebook(fmt(bits, signed), out.ctypes.data_as(C.c_void_p), C.byref(cnt)), "dybit_codebook")
    return out[: cnt.value]


def dybit_packed_bytes(bits: int, signed: bool, n: int) -> int:
    return int(lib().dybit_packed_bytes(fmt(bits, signed), n))


SEARCH_SPEEDUP, SEARCH_RMSE = 0, 1


def dybit_search(lat, rmse_w, rmse_a, strategy: int, constraint: float, k: int):
    """lat: [layers][3][3], rmse_w / rmse_a: [layers][3] (levels 8, 4, 2 bits).
    Returns (w_bits, a_bits, ratio, met)."""
    import numpy as np
    lat = np.ascontiguousarray(lat, dtype=np.float64)
    rmse_w = np.ascontiguousarray(rmse_w, dtype=np.float64)
    rmse_a = np.ascontiguousarray(rmse_a, dtype=np.float64)
    n = lat.shape[0] if lat.ndim == 3 else 0
    if lat.shape != (n, 3, 3) or rmse_w.shape != (n, 3) or rmse_a.shape != (n, 3):
        raise ValueError("expected tables of shape [layers][3][3] and [layers][3]")
    w = np.zeros(max(n, 1), dtype=np.int32)
    a = np.zeros(max(n, 1), dtype=np.int32)
    ratio, met = C.c_double(0.0), C.c_int32(0)
    vp = lambda arr: arr.ctypes.data_as(C.c_void_p)
    _check(lib().dybit_search(n, vp(lat), vp(rmse_w), vp(rmse_a), int(strategy), float(constraint), int(k),
                              vp(w), vp(a), C.byref(ratio), C.byref(met)), "dybit_search")
    return w[:n].tolist(), a[:n].tolist(), ratio.value, bool(met.value)


# ---- device -----------------------------------------------------------------
def dybit_rmse(x: torch.Tensor, scale: torch.Tensor, bits: int, signed: bool, out: torch.Tensor | None = None, stream=None):
    """Device tensor of 4 doubles: RMSE (Eq. 2), sum (x - x_hat)^2, sum x, sum x^2."""
    assert x.dtype == torch.float32 and scale.dtype == torch.float32
    if out is None:
        out = torch.empty(4, dtype=torch.float64, device=x.device)
    assert out.dtype == torch.float64 and out.numel() >= 4
    _check(lib().dybit_rmse(_ptr(x), x.numel(), fmt(bits, signed), _ptr(scale), _ptr(out), _stream(stream)), "dybit_rmse")
    return out


def dybit_absmax_scale(x: torch.Tensor, bits: int, signed: bool, out: torch.Tensor | None = None, stream=None):
    assert x.dtype == torch.float32
    if out is None:
        out = torch.empty(1, dtype=torch.float32, device=x.device)
    _check(lib().dybit_absmax_scale(_ptr(x), x.numel(), fmt(bits, signed), _ptr(out), _stream(stream)),
           "dybit_absmax_scale")
    return out


def dybit_quantize(x: torch.Tensor, scale: torch.Tensor, bits: int, signed: bool,
                   out: torch.Tensor | None = None, stream=None):
    """Packed codes (uint8 tensor of dybit_packed_bytes elements) of a flat float32 tensor."""
    assert x.dtype == torch.float32 and scale.dtype == torch.float32
    n = x.numel()
    if out is None:
        out = torch.empty(dybit_packed_bytes(bits, signed, n), dtype=torch.uint8, device=x.device)
    _check(lib().dybit_quantize(_ptr(x), n, fmt(bits, signed), _ptr(scale), _ptr(out), _stream(stream)),
           "dybit_quantize")
    return out


def dybit_quantize_absmax(x: torch.Tensor, absmax: torch.Tensor, bits: int, signed: bool,
                          out: torch.Tensor | None = None, scale_out: torch.Tensor | None = None, stream=None):
    """Scale from a known max|x| (device scalar) and packed codes in one launch; returns (scale, codes)."""
    assert x.dtype == torch.float32 and absmax.dtype == torch.float32
    n = x.numel()
    if out is None:
        out = torch.empty(dybit_packed_bytes(bits, signed, n), dtype=torch.uint8, device=x.device)
    if scale_out is None:
        scale_out = torch.empty(1, dtype=torch.float32, device=x.device)
    _check(lib().dybit_quantize_absmax(_ptr(x), n, fmt(bits, signed), _ptr(absmax), _ptr(scale_out), _ptr(out),
                                       _stream(stream)), "dybit_quantize_absmax")
    return scale_out, out


def dybit_fake_quant(x: torch.Tensor, scale: torch.Tensor, bits: int, signed: bool, out: torch.Tensor | None = None, stream=None):
    """y = scale * value(code of x): quantize and decode in one pass."""
    assert x.dtype == torch.float32 and scale.dtype == torch.float32
    if out is None:
        out = torch.empty_like(x)
    assert out.dtype == torch.float32 and out.numel() == x.numel()
    _check(lib().dybit_fake_quant(_ptr(x), x.numel(), fmt(bits, signed), _ptr(scale), _ptr(out), _stream(stream)),
           "dybit_fake_quant")
    return out


def dybit_fake_quant_bwd(x: torch.Tensor, grad_out: torch.Tensor, scale: torch.Tensor, bits: int, signed: bool,
                         out: torch.Tensor | None = None, stream=None):
    """Straight-through gradient of dybit_fake_quant: grad_out where x lies inside the format's range, else 0."""
    assert x.dtype == torch.float32 and grad_out.dtype == torch.float32 and grad_out.numel() == x.numel()
    if out is None:
        out = torch.empty_like(x)
    _check(lib().dybit_fake_quant_bwd(_ptr(x), _ptr(grad_out), x.numel(), fmt(bits, signed), _ptr(scale), _ptr(out),
                                      _stream(stream)), "dybit_fake_quant_bwd")
    return out


def dybit_dequantize(codes: torch.Tensor, n: int, scale: torch.Tensor, bits: int, signed: bool,
                     out: torch.Tensor | None = None, stream=None):
    assert codes.dtype == torch.uint8
    if out is None:
        out = torch.empty(n, dtype=torch.float32, device=codes.device)
    _check(lib().dybit_dequantize(_ptr(codes), n, fmt(bits, signed), _ptr(scale), _ptr(out), _stream(stream)),
           "dybit_dequantize")
    return out


def dybit_gemm(M: int, N: int, K: int, a_codes, a_fmt, a_scale, w_codes, w_fmt, w_scale,
               bias=None, relu: bool = False, out: torch.Tensor | None = None, ldc: int | None = None, stream=None):
    """C [M][N] float32 = sA sW A W^T (+bias)(ReLU); a_fmt / w_fmt are (bits, signed) pairs."""
    if out is None:
        out = torch.empty((M, N), dtype=torch.float32, device=a_scale.device)
    if ldc is None:
        ldc = N
    _check(lib().dybit_gemm(M, N, K, _ptr(a_codes), fmt(*a_fmt), _ptr(a_scale),
                            _ptr(w_codes), fmt(*w_fmt), _ptr(w_scale), _ptr(bias), int(bool(relu)),
                            _ptr(out), ldc, _stream(stream)), "dybit_gemm")
    return out


def dybit_conv2d(B: int, H: int, W: int, Cin: int, Cout: int, kh: int, kw: int, stride: int, pad: int,
                 x_codes, x_fmt, x_scale, w_codes, w_fmt, w_scale, bias=None, relu: bool = False,
                 out: torch.Tensor | None = None, stream=None):
    """Y [B][Ho][Wo][Cout] float32 from NHWC codes and [Cout][kh][kw][Cin] filter codes."""
    Ho = (H + 2 * pad - kh) // stride + 1
    Wo = (W + 2 * pad - kw) // stride + 1
    if out is None:
        out = torch.empty((B, Ho, Wo, Cout), dtype=torch.float32, device=x_scale.device)
    _check(lib().dybit_conv2d(B, H, W, Cin, Cout, kh, kw, stride, pad,
                              _ptr(x_codes), fmt(*x_fmt), _ptr(x_scale),
                              _ptr(w_codes), fmt(*w_fmt), _ptr(w_scale), _ptr(bias), int(bool(relu)),
                              _ptr(out), _stream(stream)), "dybit_conv2d")
    return out


def dybit_gemm_ex(M: int, N: int, K: int, a_codes, a_fmt, a_scale, w_codes, w_fmt, w_scale,
                  bias=None, residual=None, relu: bool = False, absmax=None,
                  out: torch.Tensor | None = None, ldc: int | None = None, stream=None):
    """dybit_gemm with the optional shortcut tensor `residual` (laid out like the output) and the
    optional running maximum `absmax` (device float32 scalar, >= 0 on entry)."""
    if out is None:
        out = torch.empty((M, N), dtype=torch.float32, device=a_scale.device)
    if ldc is None:
        ldc = N
    _check(lib().dybit_gemm_ex(M, N, K, _ptr(a_codes), fmt(*a_fmt), _ptr(a_scale),
                               _ptr(w_codes), fmt(*w_fmt), _ptr(w_scale), _ptr(bias), _ptr(residual), int(bool(relu)),
                               _ptr(out), ldc, _ptr(absmax), _stream(stream)), "dybit_gemm_ex")
    return out


def dybit_conv2d_ex(B: int, H: int, W: int, Cin: int, Cout: int, kh: int, kw: int, stride: int, pad: int,
                    x_codes, x_fmt, x_scale, w_codes, w_fmt, w_scale, bias=None, residual=None, relu: bool = False,
                    absmax=None, out: torch.Tensor | None = None, stream=None):
    """dybit_conv2d with the optional shortcut tensor `residual` ([B][Ho][Wo][Cout]) and the optional
    running maximum `absmax` (device float32 scalar, >= 0 on entry)."""
    Ho = (H + 2 * pad - kh) // stride + 1
    Wo = (W + 2 * pad - kw) // stride + 1
    if out is None:
        out = torch.empty((B, Ho, Wo, Cout), dtype=torch.float32, device=x_scale.device)
    _check(lib().dybit_conv2d_ex(B, H, W, Cin, Cout, kh, kw, stride, pad,
                                 _ptr(x_codes), fmt(*x_fmt), _ptr(x_scale),
                                 _ptr(w_codes), fmt(*w_fmt), _ptr(w_scale), _ptr(bias), _ptr(residual), int(bool(relu)),
                                 _ptr(out), _ptr(absmax), _stream(stream)), "dybit_conv2d_ex")
    return out


def dybit_gemm_wb(M: int, N: int, K: int, a_codes, a_fmt, a_scale, w_codes, w_fmt, w_scale, c_fmt, c_scale,
                  bias=None, residual=None, relu: bool = False, absmax=None, fp32: bool = True,
                  out: torch.Tensor | None = None, ldc: int | None = None,
                  codes_out: torch.Tensor | None = None, stream=None):
    """dybit_gemm_ex with the results also (fp32=True) or only (fp32=False) written back as packed
    DyBit codes of format c_fmt under the given device scale.  Returns (C or None, codes [M][N*bits/8])."""
    if ldc is None:
        ldc = N
    if fp32 and out is None:
        out = torch.empty((M, N), dtype=torch.float32, device=a_scale.device)
    if codes_out is None:
        codes_out = torch.empty((M, N * c_fmt[0] // 8), dtype=torch.uint8, device=a_scale.device)
    _check(lib().dybit_gemm_wb(M, N, K, _ptr(a_codes), fmt(*a_fmt), _ptr(a_scale),
                               _ptr(w_codes), fmt(*w_fmt), _ptr(w_scale), _ptr(bias), _ptr(residual), int(bool(relu)),
                               _ptr(out if fp32 else None), ldc, _ptr(absmax),
                               fmt(*c_fmt), _ptr(c_scale), _ptr(codes_out), _stream(stream)), "dybit_gemm_wb")
    return (out if fp32 else None), codes_out


def dybit_conv2d_wb(B: int, H: int, W: int, Cin: int, Cout: int, kh: int, kw: int, stride: int, pad: int,
                    x_codes, x_fmt, x_scale, w_codes, w_fmt, w_scale, y_fmt, y_scale,
                    bias=None, residual=None, relu: bool = False, absmax=None, fp32: bool = True,
                    out: torch.Tensor | None = None, codes_out: torch.Tensor | None = None, stream=None):
    """dybit_conv2d_ex with the results also (fp32=True) or only (fp32=False) written back as packed
    DyBit codes.  Returns (Y or None, codes [B][Ho][Wo][Cout*bits/8])."""
    Ho = (H + 2 * pad - kh) // stride + 1
    Wo = (W + 2 * pad - kw) // stride + 1
    if fp32 and out is None:
        out = torch.empty((B, Ho, Wo, Cout), dtype=torch.float32, device=x_scale.device)
    if codes_out is None:
        codes_out = torch.empty((B, Ho, Wo, Cout * y_fmt[0] // 8), dtype=torch.uint8, device=x_scale.device)
    _check(lib().dybit_conv2d_wb(B, H, W, Cin, Cout, kh, kw, stride, pad,
                                 _ptr(x_codes), fmt(*x_fmt), _ptr(x_scale),
                                 _ptr(w_codes), fmt(*w_fmt), _ptr(w_scale), _ptr(bias), _ptr(residual), int(bool(relu)),
                                 _ptr(out if fp32 else None), _ptr(absmax),
                                 fmt(*y_fmt), _ptr(y_scale), _ptr(codes_out), _stream(stream)), "dybit_conv2d_wb")
    return (out if fp32 else None), codes_out


def dybit_gemm_wb_rc(M: int, N: int, K: int, a_codes, a_fmt, a_scale, w_codes, w_fmt, w_scale, c_fmt, c_scale,
                     r_codes, r_fmt, r_scale, bias=None, relu: bool = False, absmax=None, fp32: bool = True,
                     out: torch.Tensor | None = None, codes_out: torch.Tensor | None = None, stream=None):
    """dybit_gemm_wb with the shortcut given as packed DyBit codes `r_codes` ([M][N*bits/8]) of format r_fmt
    and scale r_scale.  Returns (C or None, codes)."""
    if fp32 and out is None:
        out = torch.empty((M, N), dtype=torch.float32, device=a_scale.device)
    if codes_out is None:
        codes_out = torch.empty((M, N * c_fmt[0] // 8), dtype=torch.uint8, device=a_scale.device)
    _check(lib().dybit_gemm_wb_rc(M, N, K, _ptr(a_codes), fmt(*a_fmt), _ptr(a_scale),
                                  _ptr(w_codes), fmt(*w_fmt), _ptr(w_scale), _ptr(bias),
                                  _ptr(r_codes), fmt(*r_fmt), _ptr(r_scale), int(bool(relu)),
                                  _ptr(out if fp32 else None), N, _ptr(absmax),
                                  fmt(*c_fmt), _ptr(c_scale), _ptr(codes_out), _stream(stream)), "dybit_gemm_wb_rc")
    return (out if fp32 else None), codes_out


def dybit_conv2d_wb_rc(B: int, H: int, W: int, Cin: int, Cout: int, kh: int, kw: int, stride: int, pad: int,
                       x_codes, x_fmt, x_scale, w_codes, w_fmt, w_scale, y_fmt, y_scale,
                       r_codes, r_fmt, r_scale, bias=None, relu: bool = False, absmax=None, fp32: bool = True,
                       out: torch.Tensor | None = None, codes_out: torch.Tensor | None = None, stream=None):
    """dybit_conv2d_wb with the shortcut given as packed DyBit codes `r_codes` ([B][Ho][Wo][Cout*bits/8]).
    Returns (Y or None, codes)."""
    Ho = (H + 2 * pad - kh) // stride + 1
    Wo = (W + 2 * pad - kw) // stride + 1
    if fp32 and out is None:
        out = torch.empty((B, Ho, Wo, Cout), dtype=torch.float32, device=x_scale.device)
    if codes_out is None:
        codes_out = torch.empty((B, Ho, Wo, Cout * y_fmt[0] // 8), dtype=torch.uint8, device=x_scale.device)
    _check(lib().dybit_conv2d_wb_rc(B, H, W, Cin, Cout, kh, kw, stride, pad,
                                    _ptr(x_codes), fmt(*x_fmt), _ptr(x_scale),
                                    _ptr(w_codes), fmt(*w_fmt), _ptr(w_scale), _ptr(bias),
                                    _ptr(r_codes), fmt(*r_fmt), _ptr(r_scale), int(bool(relu)),
                                    _ptr(out if fp32 else None), _ptr(absmax),
                                    fmt(*y_fmt), _ptr(y_scale), _ptr(codes_out), _stream(stream)), "dybit_conv2d_wb_rc")
    return (out if fp32 else None), codes_out


def dybit_maxpool2d_codes(B: int, H: int, W: int, C: int, k: int, stride: int, pad: int, x_codes, x_fmt,
                          out: torch.Tensor | None = None, stream=None):
    """Max pooling of packed codes [B][H][W][C*bits/8] -> [B][Ho][Wo][C*bits/8] (same format, same scale)."""
    Ho = (H + 2 * pad - k) // stride + 1
    Wo = (W + 2 * pad - k) // stride + 1
    if out is None:
        out = torch.empty((B, Ho, Wo, C * x_fmt[0] // 8), dtype=torch.uint8, device=x_codes.device)
    _check(lib().dybit_maxpool2d_codes(B, H, W, C, k, stride, pad, _ptr(x_codes), fmt(*x_fmt), _ptr(out), _stream(stream)),
           "dybit_maxpool2d_codes")
    return out


def dybit_dwconv2d(B: int, H: int, W: int, C: int, kh: int, kw: int, stride: int, pad: int,
                   x_codes, x_fmt, x_scale, w_codes, w_fmt, w_scale, bias=None, relu: bool = False, absmax=None,
                   out: torch.Tensor | None = None, stream=None):
    """Depthwise convolution: x_codes [B][H][W][C], w_codes [kh][kw][C]; returns Y [B][Ho][Wo][C] float32."""
    Ho = (H + 2 * pad - kh) // stride + 1
    Wo = (W + 2 * pad - kw) // stride + 1
    if out is None:
        out = torch.empty((B, Ho, Wo, C), dtype=torch.float32, device=x_scale.device)
    _check(lib().dybit_dwconv2d(B, H, W, C, kh, kw, stride, pad, _ptr(x_codes), fmt(*x_fmt), _ptr(x_scale),
                                _ptr(w_codes), fmt(*w_fmt), _ptr(w_scale), _ptr(bias), int(bool(relu)),
                                _ptr(out), _ptr(absmax), _stream(stream)), "dybit_dwconv2d")
    return out


def dybit_dwconv2d_wb(B: int, H: int, W: int, C: int, kh: int, kw: int, stride: int, pad: int,
                      x_codes, x_fmt, x_scale, w_codes, w_fmt, w_scale, bias=None, relu: bool = False, absmax=None,
                      y_fmt=None, y_scale=None, per_channel: bool = False, fp32: bool = True,
                      out: torch.Tensor | None = None, stream=None):
    """dybit_dwconv2d with per-channel weight scales (per_channel: w_scale holds C floats) and, with y_fmt and
    y_scale, the results also (fp32=False: only) written back as codes.  Returns (Y or None, codes or None)."""
    Ho = (H + 2 * pad - kh) // stride + 1
    Wo = (W + 2 * pad - kw) // stride + 1
    if fp32 and out is None:
        out = torch.empty((B, Ho, Wo, C), dtype=torch.float32, device=x_scale.device)
    codes = None
    if y_fmt is not None:
        codes = torch.empty((B, Ho, Wo, C * y_fmt[0] // 8), dtype=torch.uint8, device=x_scale.device)
    _check(lib().dybit_dwconv2d_wb(B, H, W, C, kh, kw, stride, pad, _ptr(x_codes), fmt(*x_fmt), _ptr(x_scale),
                                   _ptr(w_codes), fmt(*w_fmt), _ptr(w_scale), int(bool(per_channel)), _ptr(bias), int(bool(relu)),
                                   _ptr(out) if fp32 else None, _ptr(absmax), fmt(*(y_fmt or (4, False))), _ptr(y_scale),
                                   _ptr(codes), _stream(stream)), "dybit_dwconv2d_wb")
    return (out if fp32 else None), codes


def dybit_group_conv2d(B: int, H: int, W: int, Cin: int, Cout: int, kh: int, kw: int, stride: int, pad: int, groups: int,
                       x_codes, x_fmt, x_scale, w_codes, w_fmt, w_scale, bias=None, residual=None, relu: bool = False,
                       absmax=None, per_channel: bool = False, out: torch.Tensor | None = None, stream=None):
    """Grouped convolution: x_codes [B][H][W][Cin], w_codes [Cout][kh][kw][Cin/groups]; returns Y [B][Ho][Wo][Cout]."""
    Ho = (H + 2 * pad - kh) // stride + 1
    Wo = (W + 2 * pad - kw) // stride + 1
    if out is None:
        out = torch.empty((B, Ho, Wo, Cout), dtype=torch.float32, device=x_scale.device)
    _check(lib().dybit_group_conv2d(B, H, W, Cin, Cout, kh, kw, stride, pad, groups, _ptr(x_codes), fmt(*x_fmt), _ptr(x_scale),
                                    _ptr(w_codes), fmt(*w_fmt), _ptr(w_scale), int(bool(per_channel)), _ptr(bias), _ptr(residual),
                                    int(bool(relu)), _ptr(out), _ptr(absmax), _stream(stream)), "dybit_group_conv2d")
    return out


def dybit_quantize_cols(x: torch.Tensor, bits: int, signed: bool, stream=None):
    """x: [rows][cols] float32.  Returns (scales [cols], codes [rows][cols*bits/8]): every column encoded under
    its own max-abs scale (a depthwise filter [kh*kw][C] with one scale per channel)."""
    assert x.dtype == torch.float32 and x.dim() == 2
    rows, cols = x.shape
    scales = torch.empty(cols, dtype=torch.float32, device=x.device)
    codes = torch.empty((rows, cols * bits // 8), dtype=torch.uint8, device=x.device)
    _check(lib().dybit_quantize_cols(_ptr(x), rows, cols, fmt(bits, signed), _ptr(scales), _ptr(codes), _stream(stream)),
           "dybit_quantize_cols")
    return scales, codes


def dybit_quantize_pad(x: torch.Tensor, cols_padded: int, scale: torch.Tensor, bits: int, signed: bool, stream=None):
    """Codes of the [rows][cols] matrix x with every row padded to cols_padded codes (zero codes)."""
    rows, cols = x.shape
    out = torch.empty((rows, cols_padded * bits // 8), dtype=torch.uint8, device=x.device)
    _check(lib().dybit_quantize_pad(_ptr(x), rows, cols, cols_padded, fmt(bits, signed), _ptr(scale), _ptr(out), _stream(stream)),
           "dybit_quantize_pad")
    return out


def dybit_quantize_rows(x: torch.Tensor, bits: int, signed: bool, stream=None):
    """x: [rows][cols] float32.  Returns (scales [rows], codes [rows][cols*bits/8]): every row encoded under
    its own max-abs scale."""
    assert x.dtype == torch.float32 and x.dim() == 2
    rows, cols = x.shape
    scales = torch.empty(rows, dtype=torch.float32, device=x.device)
    codes = torch.empty((rows, cols * bits // 8), dtype=torch.uint8, device=x.device)
    _check(lib().dybit_quantize_rows(_ptr(x), rows, cols, fmt(bits, signed), _ptr(scales), _ptr(codes), _stream(stream)),
           "dybit_quantize_rows")
    return scales, codes


def dybit_gemm_pc(M: int, N: int, K: int, a_codes, a_fmt, a_scale, w_codes, w_fmt, w_scales,
                  bias=None, residual=None, relu: bool = False, absmax=None, c_fmt=None, c_scale=None,
                  fp32: bool = True, out: torch.Tensor | None = None, ldc: int | None = None, stream=None):
    """The matrix product with one weight scale per output column (w_scales: N floats).  With c_fmt and
    c_scale the results are also (or, fp32=False, only) written back as codes.  Returns (C or None, codes or None)."""
    if ldc is None:
        ldc = N
    if fp32 and out is None:
        out = torch.empty((M, N), dtype=torch.float32, device=a_scale.device)
    codes = None
    if c_fmt is not None:
        codes = torch.empty((M, N * c_fmt[0] // 8), dtype=torch.uint8, device=a_scale.device)
    _check(lib().dybit_gemm_pc(M, N, K, _ptr(a_codes), fmt(*a_fmt), _ptr(a_scale),
                               _ptr(w_codes), fmt(*w_fmt), _ptr(w_scales), _ptr(bias), _ptr(residual), int(bool(relu)),
                               _ptr(out if fp32 else None), ldc, _ptr(absmax),
                               fmt(*(c_fmt or (8, False))), _ptr(c_scale), _ptr(codes), _stream(stream)), "dybit_gemm_pc")
    return (out if fp32 else None), codes


def dybit_conv2d_pc(B: int, H: int, W: int, Cin: int, Cout: int, kh: int, kw: int, stride: int, pad: int,
                    x_codes, x_fmt, x_scale, w_codes, w_fmt, w_scales,
                    bias=None, residual=None, relu: bool = False, absmax=None, y_fmt=None, y_scale=None,
                    fp32: bool = True, out: torch.Tensor | None = None, stream=None):
    """The convolution with one weight scale per output channel (w_scales: Cout floats); see dybit_gemm_pc."""
    Ho = (H + 2 * pad - kh) // stride + 1
    Wo = (W + 2 * pad - kw) // stride + 1
    if fp32 and out is None:
        out = torch.empty((B, Ho, Wo, Cout), dtype=torch.float32, device=x_scale.device)
    codes = None
    if y_fmt is not None:
        codes = torch.empty((B, Ho, Wo, Cout * y_fmt[0] // 8), dtype=torch.uint8, device=x_scale.device)
    _check(lib().dybit_conv2d_pc(B, H, W, Cin, Cout, kh, kw, stride, pad,
                                 _ptr(x_codes), fmt(*x_fmt), _ptr(x_scale),
                                 _ptr(w_codes), fmt(*w_fmt), _ptr(w_scales), _ptr(bias), _ptr(residual), int(bool(relu)),
                                 _ptr(out if fp32 else None), _ptr(absmax),
                                 fmt(*(y_fmt or (8, False))), _ptr(y_scale), _ptr(codes), _stream(stream)), "dybit_conv2d_pc")
    return (out if fp32 else None), codes


def dybit_scale_from_absmax(absmax: torch.Tensor, bits: int, signed: bool, out: torch.Tensor | None = None, stream=None):
    """scale = absmax / 2^(m-1) (1.0 for 0) on the device; returns the 1-element scale tensor."""
    if out is None:
        out = torch.empty(1, dtype=torch.float32, device=absmax.device)
    _check(lib().dybit_scale_from_absmax(_ptr(absmax), fmt(bits, signed), _ptr(out), _stream(stream)), "dybit_scale_from_absmax")
    return out


def dybit_get_last_async_error(stream=None) -> int:
    flag = C.c_int32(0)
    _check(lib().dybit_get_last_async_error(C.byref(flag), _stream(stream)), "dybit_get_last_async_error")
    return int(flag.value)


def dybit_set_async_error_word(word: torch.Tensor | None) -> None:
    """Asynchronous errors of this host thread's calls go to `word` (device int32 tensor of one element, kept
    alive by the caller) instead of the library's flag; None restores the library's flag."""
    _check(lib().dybit_set_async_error_word(_ptr(word)), "dybit_set_async_error_word")


def dybit_diag_mfma_f16(operands: torch.Tensor, workgroups: int, iters: int, sink: torch.Tensor, stream=None) -> float:
    """Launches the MFMA-only measurement kernel; returns the flops of the launch."""
    flops = C.c_double(0.0)
    _check(lib().dybit_diag_mfma_f16(_ptr(operands), workgroups, iters, _ptr(sink), C.byref(flops), _stream(stream)),
           "dybit_diag_mfma_f16")
    return float(flops.value)


def dybit_diag_mfma_f8(operands: torch.Tensor, workgroups: int, iters: int, sink: torch.Tensor, stream=None) -> float:
    """The same for the fp8 (e4m3) instruction; `operands` holds e4m3 bytes."""
    flops = C.c_double(0.0)
    _check(lib().dybit_diag_mfma_f8(_ptr(operands), workgroups, iters, _ptr(sink), C.byref(flops), _stream(stream)),
           "dybit_diag_mfma_f8")
    return float(flops.value)
