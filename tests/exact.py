"""Exact-arithmetic helpers for pins: correctly rounded binary32 results computed with
Python integers and Fractions only (no floating point on the way)."""
from fractions import Fraction
from math import isqrt

import numpy as np


def _scale(v: Fraction):
    """exponent e with 2^23 <= v / 2^e < 2^24 (v > 0)"""
    e = 0
    while v / Fraction(2) ** e >= 1 << 24:
        e += 1
    while v / Fraction(2) ** e < 1 << 23:
        e -= 1
    return e


def round_f32(v: Fraction) -> np.float32:
    """nearest binary32 (ties to even) of a positive rational in the normal range"""
    if v == 0:
        return np.float32(0.0)
    assert v > 0
    e = _scale(v)
    q = v / Fraction(2) ** e
    n = q.numerator // q.denominator
    rem = q - n
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and n & 1):
        n += 1
    out = Fraction(n) * Fraction(2) ** e
    f = np.float32(float(out))          # exact: n < 2^24+1 and a power of two
    assert Fraction(float(f)) == out
    return f


def sqrt_f32(v: Fraction) -> np.float32:
    """correctly rounded binary32 square root of a positive rational"""
    if v == 0:
        return np.float32(0.0)
    # find even-power scaling so the root has a 24-bit integer part
    k = 0
    while v * Fraction(4) ** k < Fraction(1 << 46):
        k += 1
    while v * Fraction(4) ** k >= Fraction(1 << 48):
        k -= 1
    y = v * Fraction(4) ** k                       # 2^46 <= y < 2^48  ->  2^23 <= sqrt(y) < 2^24
    n = isqrt(y.numerator // y.denominator)
    # sqrt(y) in [n, n+1); round to nearest (a tie would need sqrt(y) = n + 1/2, i.e. y = n^2+n+1/4)
    mid = Fraction(2 * n + 1, 2)
    if y > mid * mid or (y == mid * mid and n & 1):
        n += 1
    out = Fraction(n) / Fraction(2) ** k
    f = np.float32(float(out))
    assert Fraction(float(f)) == out
    return f
