"""Enumeration models of small floating-point types.  TEST INFRASTRUCTURE ONLY.

Used to prove, by listing every finite value of a candidate matrix-core input
type, which DyBit formats embed exactly into it.  The types are described by
their public format definitions (IEEE 754 binary16, bfloat16, and the OCP
8-bit / microscaling 6- and 4-bit element formats), not by any library.
"""
from __future__ import annotations

from fractions import Fraction
from functools import lru_cache

# name -> (exponent bits, mantissa bits, bias, special-value convention)
#   "ieee":  top exponent is Inf/NaN
#   "ocp_e4m3": only S.1111.111 is NaN, no Inf, the rest of the top binade is finite
#   "none": no Inf/NaN at all (OCP MX element types)
TYPES = {
    "fp16": (5, 10, 15, "ieee"),
    "bf16": (8, 7, 127, "ieee"),
    "fp8_e4m3": (4, 3, 7, "ocp_e4m3"),
    "fp8_e5m2": (5, 2, 15, "ieee"),
    "fp6_e2m3": (2, 3, 1, "none"),
    "fp6_e3m2": (3, 2, 3, "none"),
    "fp4_e2m1": (2, 1, 1, "none"),
}


def _enumerate(name: str):
    """Yield (bit pattern, exact value) for every finite non-negative encoding."""
    e_bits, m_bits, bias, special = TYPES[name]
    for e in range(1 << e_bits):
        for f in range(1 << m_bits):
            if special == "ieee" and e == (1 << e_bits) - 1:
                continue
            if special == "ocp_e4m3" and e == (1 << e_bits) - 1 and f == (1 << m_bits) - 1:
                continue
            if e == 0:
                v = Fraction(f, 1 << m_bits) * Fraction(2) ** (1 - bias)
            else:
                v = (1 + Fraction(f, 1 << m_bits)) * Fraction(2) ** (e - bias)
            yield (e << m_bits) | f, v


@lru_cache(maxsize=None)
def _tables(name: str):
    pattern_of = {}
    for bits, v in _enumerate(name):
        pattern_of.setdefault(v, bits)
    return pattern_of


def finite_values(name: str) -> set[Fraction]:
    """Every finite value the type can hold (both signs), as exact rationals."""
    pos = _tables(name)
    return set(pos) | {-v for v in pos}


def encode(name: str, v: Fraction) -> int | None:
    """Bit pattern of v in the type, or None when v is not exactly representable."""
    e_bits, m_bits, _, _ = TYPES[name]
    a = -v if v < 0 else v
    pat = _tables(name).get(Fraction(a))
    if pat is None:
        return None
    return ((1 if v < 0 else 0) << (e_bits + m_bits)) | pat


def embeds_exactly(values, name: str) -> bool:
    pos = _tables(name)
    return all(abs(Fraction(v)) in pos for v in values)
