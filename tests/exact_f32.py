"""Exact-rational fp32 arithmetic for brute-force pins (tiny inputs only)."""
from fractions import Fraction

import numpy as np


def round_to_f32(v: Fraction) -> np.float32:
    """Correctly rounded (nearest, ties to even) fp32 of an exact rational."""
    if v == 0:
        return np.float32(0.0)
    sign = -1 if v < 0 else 1
    a = abs(v)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    assert Fraction(2) ** e <= a < Fraction(2) ** (e + 1)
    e = max(e, -126)
    quantum = Fraction(2) ** (e - 23)
    q = a / quantum
    n = q.numerator // q.denominator
    rem = q - n
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (n & 1)):
        n += 1
    return np.float32(sign * float(n * quantum))


def fma_f32(a, b, c) -> np.float32:
    return round_to_f32(Fraction(float(a)) * Fraction(float(b)) + Fraction(float(c)))


def add_f32(a, b) -> np.float32:
    return round_to_f32(Fraction(float(a)) + Fraction(float(b)))
