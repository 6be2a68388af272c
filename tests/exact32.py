"""Exact binary32 rounding from rational numbers, for pinning the oracle.

Independent of the oracle and of numpy's float arithmetic: a value is a
fractions.Fraction, and `round_f32` applies IEEE-754 round-to-nearest-even to
the binary32 grid (normal and subnormal), returning the rounded value again as
a Fraction (or +-inf as float).
"""
from fractions import Fraction
import struct

EMIN = -126
MANT = 23
MAXF = Fraction((2 ** 24 - 1) * 2 ** (127 - 23))


def f32_to_fraction(x):
    """Exact value of a python float that is representable in binary32."""
    return Fraction(float(x))


def round_f32(q):
    """Round Fraction q to binary32 (RNE).  Returns a Fraction, or float('inf')/-inf on overflow."""
    if q == 0:
        return Fraction(0)
    sign = -1 if q < 0 else 1
    a = abs(q)
    # exponent e with 2^e <= a < 2^(e+1)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    elif Fraction(2) ** (e + 1) <= a:
        e += 1
    e = max(e, EMIN)
    ulp = Fraction(2) ** (e - MANT)
    n = a / ulp
    lo = n.numerator // n.denominator
    rem = n - lo
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (lo & 1)):
        lo += 1
    r = lo * ulp
    if r > MAXF:
        # beyond the largest finite value by at least half an ulp
        return float("inf") * sign
    return sign * r


def fraction_to_bits(q):
    """Bit pattern (uint32) of a Fraction that is exactly representable in binary32 (0 -> +0)."""
    return struct.unpack("<I", struct.pack("<f", float(q)))[0]
