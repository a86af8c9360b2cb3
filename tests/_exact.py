"""Exact-arithmetic helpers for the tests: IEEE binary32 rounding of rationals, done with
Python integers (no floating point), so hand-computed expectations do not depend on any
implementation under test."""
import math
from fractions import Fraction

import numpy as np


def f32_round(x: Fraction) -> np.float32:
    """Round an exact rational to binary32, to nearest, ties to even (overflow -> inf)."""
    x = Fraction(x)
    if x == 0:
        return np.float32(0.0)
    sign = -1 if x < 0 else 1
    a = abs(x)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    assert Fraction(2) ** e <= a < Fraction(2) ** (e + 1)
    e = max(e, -126)
    scaled = a / (Fraction(2) ** (e - 23))
    q = scaled.numerator // scaled.denominator
    rem = scaled - q
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (q & 1)):
        q += 1
    val = math.ldexp(q, e - 23)
    if val >= 2.0 ** 128:
        val = math.inf
    return np.float32(sign * val)


def frac(x) -> Fraction:
    """Exact value of a float."""
    return Fraction(float(x))


def fma32(a, b, c) -> np.float32:
    return f32_round(frac(a) * frac(b) + frac(c))


def mul32(a, b) -> np.float32:
    return f32_round(frac(a) * frac(b))


def sub32(a, b) -> np.float32:
    return f32_round(frac(a) - frac(b))


def div32(a, b) -> np.float32:
    return f32_round(frac(a) / frac(b))


def bits(x) -> int:
    return int(np.array([x], dtype=np.float32).view(np.uint32)[0])
