"""Exact-rational helpers for the oracle's pins, written with Python integers only.

Nothing here is used by the oracle or by the GPU path: these are the independent
yardsticks the oracle is measured against.
"""
from fractions import Fraction
import math


def round_half_even(x: Fraction) -> int:
    fl = math.floor(x)
    d = x - fl
    if d > Fraction(1, 2):
        return fl + 1
    if d < Fraction(1, 2):
        return fl
    return fl if fl % 2 == 0 else fl + 1


def fl32(x: Fraction) -> Fraction:
    """Nearest IEEE binary32 value (ties to even), as an exact Fraction. No overflow handling."""
    if x == 0:
        return Fraction(0)
    s = -1 if x < 0 else 1
    a = abs(x)
    # exponent e with 2^e <= a < 2^(e+1)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    if Fraction(2) ** (e + 1) <= a:
        e += 1
    e = max(e, -126)            # subnormals share the smallest normal exponent
    ulp = Fraction(2) ** (e - 23)
    n = round_half_even(a / ulp)
    return s * n * ulp


def fl64(x: Fraction) -> Fraction:
    if x == 0:
        return Fraction(0)
    s = -1 if x < 0 else 1
    a = abs(x)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    if Fraction(2) ** (e + 1) <= a:
        e += 1
    e = max(e, -1022)
    ulp = Fraction(2) ** (e - 52)
    n = round_half_even(a / ulp)
    return s * n * ulp


def clamp(v, lo, hi):
    return max(min(v, hi), lo)
