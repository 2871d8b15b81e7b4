"""Helpers for the GPU parity tests (not collected by pytest)."""
import numpy as np
import torch

from oracle import dybit_ref as R


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def scalar(v) -> torch.Tensor:
    return torch.tensor([float(np.float32(v))], dtype=torch.float32, device="cuda")


def oracle_codes(x: np.ndarray, fmt):
    """(scale, unpacked codes) from the oracle for a float tensor."""
    s = R.absmax_scale(x, *fmt)
    return s, R.quantize(x, s, *fmt)


def pack_rows_dev(codes2d: np.ndarray, bits: int) -> torch.Tensor:
    return dev(R.pack_rows(codes2d.reshape(-1, codes2d.shape[-1]), bits))


def assert_within(got: np.ndarray, want: np.ndarray, den: np.ndarray, rel: float = 1e-5, shortcut: bool = False):
    """|got - want| <= rel * sum|a*b| per element (the GEMM tolerance; `den` is the oracle's
    denominator, which holds no shortcut term).  shortcut=True: the call added an fp32 shortcut
    tensor to the result, i.e. one more fp32 rounding of the sum, at most 2^-24 |result|."""
    err = np.abs(got.astype(np.float64) - want)
    bound = rel * den + (2.0 ** -24 * np.abs(want) if shortcut else 0.0)
    bad = err > bound
    if bad.any():
        i = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError(f"{bad.sum()} of {bad.size} outputs outside tolerance; worst at {i}: "
                             f"got {got[i]!r} want {want[i]!r} err {err[i]:.3e} bound {bound[i]:.3e}")
