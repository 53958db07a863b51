"""Exact rational arithmetic with explicit fp32 rounding, for pinning the oracle.

``rn32(q)`` rounds a ``Fraction`` to the nearest binary32 value, ties to even,
subnormals included -- written from the IEEE-754 definition, independent of
numpy's float32 arithmetic and of the oracle.
"""
from fractions import Fraction

import numpy as np


def rn32(q: Fraction) -> np.float32:
    q = Fraction(q)
    if q == 0:
        return np.float32(0.0)
    sign = -1 if q < 0 else 1
    a = abs(q)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    assert Fraction(2) ** e <= a < Fraction(2) ** (e + 1)
    e = max(e, -126)
    quantum = Fraction(2) ** (e - 23)
    n = a / quantum
    fl = n.numerator // n.denominator
    rem = n - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (fl & 1)):
        fl += 1
    v = fl * quantum
    assert v < Fraction(2) ** 128, "overflow"
    return np.float32(sign * float(v))


def F(x) -> Fraction:
    """Exact value of a float32/float."""
    return Fraction(float(x))


def add32(a, b):
    return rn32(F(a) + F(b))


def sub32(a, b):
    return rn32(F(a) - F(b))


def mul32(a, b):
    return rn32(F(a) * F(b))


def div32(a, b):
    return rn32(F(a) / F(b))
