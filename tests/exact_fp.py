"""Exact-rational helpers for the oracle's pins (test code, CPU only).

IEEE-754 defines +, *, / and fma as "the exact result, rounded once".  These
helpers compute the exact result with Python fractions and round it to
binary32 by that definition, so that the tests can state what the arithmetic
of the method must produce without calling the code under test.
"""
from __future__ import annotations

from fractions import Fraction

import numpy as np

_MIN_EXP = -126          # exponent of the smallest normal binary32
_MANT = 23


def frac(x) -> Fraction:
    """Exact value of a finite float."""
    return Fraction(float(x))


def round_to_f32(v: Fraction) -> np.float32:
    """Round an exact rational to binary32: to nearest, ties to even (subnormals included)."""
    if v == 0:
        return np.float32(0.0)
    sign = -1 if v < 0 else 1
    a = abs(v)
    # exponent e with 2^e <= a < 2^(e+1)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    if Fraction(2) ** (e + 1) <= a:
        e += 1
    e = max(e, _MIN_EXP)
    quantum = Fraction(2) ** (e - _MANT)
    units = round(a / quantum)          # Fraction.__round__ rounds half to even
    r = units * quantum
    if r >= Fraction(2) ** 128:
        return np.float32(sign * np.inf)
    return np.float32(sign * float(r))  # r is representable: the conversion is exact


def bf16_bits_to_f32(u16: np.ndarray) -> np.ndarray:
    """Widen raw bf16 patterns with integer shifts only."""
    return (np.asarray(u16, np.uint16).astype(np.uint32) << 16).view(np.float32)


def rne_int(v: Fraction) -> int:
    return round(v)                     # half to even
