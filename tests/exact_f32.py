"""Exact-arithmetic model of IEEE-754 binary32 operations for the oracle pins.

An IEEE operation is the exact real result rounded once to the nearest
representable value, ties to even.  This file computes the exact result with
Python's Fraction and rounds it with integer arithmetic, so it shares nothing
with the C oracle's hardware float operations.  Values are carried as Python
floats that are exactly representable in binary32.
"""
from fractions import Fraction
import math
import struct

EMIN = -126          # exponent of the smallest normal
MANT = 23
F32_MAX = Fraction((2 ** 24 - 1) * 2 ** (127 - 23))


def is_f32(x: float) -> bool:
    return math.isnan(x) or struct.unpack("<f", struct.pack("<f", x))[0] == x


def round_f32(q: Fraction) -> float:
    """Nearest binary32 to the non-zero rational q, ties to even mantissa."""
    assert q != 0
    sign = -1.0 if q < 0 else 1.0
    a = -q if q < 0 else q
    # e with 2^e <= a < 2^(e+1)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    assert Fraction(2) ** e <= a < Fraction(2) ** (e + 1)
    e = max(e, EMIN)                       # denormals share the exponent of the smallest normal
    quantum = Fraction(2) ** (e - MANT)
    scaled = a / quantum
    n = scaled.numerator // scaled.denominator
    rem = scaled - n
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (n & 1)):
        n += 1
    val = n * quantum
    if val > F32_MAX:
        return sign * math.inf
    return sign * float(val)               # exact: val has at most 24 significant bits


def _op(exact_fn, double_fn, x: float, y: float) -> float:
    assert is_f32(x) and is_f32(y)
    if math.isinf(x) or math.isinf(y) or math.isnan(x) or math.isnan(y):
        return double_fn(x, y)
    q = exact_fn(Fraction(x), Fraction(y))
    if q == 0:
        return double_fn(x, y)             # the sign of an exact zero follows IEEE's rule, same in binary64
    return round_f32(q)


def add(x: float, y: float) -> float:
    return _op(lambda a, b: a + b, lambda a, b: a + b, x, y)


def div(x: float, y: float) -> float:
    assert y != 0
    return _op(lambda a, b: a / b, lambda a, b: a / b, x, y)


def bits_to_fraction(u: int) -> Fraction:
    """Value of a finite non-negative binary32 bit pattern (Inf's pattern maps to 2^128)."""
    assert 0 <= u <= 0x7F800000
    exp = u >> 23
    man = u & 0x7FFFFF
    if exp == 0:
        return Fraction(man) * Fraction(2) ** (EMIN - MANT)
    return Fraction(man + (1 << 23)) * Fraction(2) ** (exp - 127 - MANT)
