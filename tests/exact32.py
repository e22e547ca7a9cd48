"""Exact-rational model of IEEE-754 binary32 rounding, used to pin the oracle's
arithmetic to the mathematics rather than to another float library.

rn(x) rounds a Fraction to the nearest binary32 value (ties to even, gradual
underflow) and returns it as a Fraction; every binary32 value is a Fraction, so
chains such as rn(rn(b*e) + d) state exactly which roundings happen.
"""
from fractions import Fraction

import numpy as np


def rn(x: Fraction) -> Fraction:
    x = Fraction(x)
    if x == 0:
        return Fraction(0)
    sign = -1 if x < 0 else 1
    a = abs(x)
    # exponent e with 2^e <= a < 2^(e+1)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    if Fraction(2) ** (e + 1) <= a:
        e += 1
    e = max(e, -126)                      # subnormal range shares the quantum of 2^-126
    quantum = Fraction(2) ** (e - 23)
    n = a / quantum
    lo = n.numerator // n.denominator
    rem = n - lo
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (lo & 1)):
        lo += 1
    r = lo * quantum
    assert r < Fraction(2) ** 128, "overflow is outside this model"
    return sign * r


def F(v) -> Fraction:
    """Exact value of a float32 (or python float holding one)."""
    return Fraction(float(np.float32(v)))


def f32(x: Fraction) -> np.float32:
    """A Fraction that is exactly representable -> np.float32."""
    v = np.float32(float(x))
    assert Fraction(float(v)) == x, "not a binary32 value"
    return v


def bits(v) -> int:
    return int(np.array(v, np.float32).view(np.uint32))
