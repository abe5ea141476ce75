"""Exact-rational helpers used by the oracle's pins.

Written from the format definitions alone (IEEE binary32, bf16 = its upper half,
OCP e4m3), with Python integers and fractions.  Nothing here calls the oracle or
the HIP library: the pins compare those against this.
"""
from __future__ import annotations

from bisect import bisect_left
from fractions import Fraction


def bf16_bits_to_fraction(h: int) -> Fraction:
    s = -1 if (h >> 15) & 1 else 1
    e = (h >> 7) & 0xFF
    m = h & 0x7F
    assert e != 0xFF
    if e == 0:
        return s * Fraction(m, 1 << 7) * Fraction(2) ** (-126)
    return s * (1 + Fraction(m, 1 << 7)) * Fraction(2) ** (e - 127)


def round_to_binary32(q: Fraction) -> Fraction:
    """Nearest IEEE binary32 value (ties to even) of an exact rational, overflow not handled."""
    if q == 0:
        return Fraction(0)
    s = -1 if q < 0 else 1
    a = abs(q)
    # find e with 2^e <= a < 2^(e+1)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    if Fraction(2) ** (e + 1) <= a:
        e += 1
    e = max(e, -126)                       # subnormal spacing below 2^-126
    quantum = Fraction(2) ** (e - 23)
    n = a / quantum
    f = n.numerator // n.denominator
    r = n - f
    if r > Fraction(1, 2) or (r == Fraction(1, 2) and f % 2 == 1):
        f += 1
    return s * f * quantum


def e4m3_code_value(c: int) -> Fraction:
    """Exact value of a non-NaN e4m3 code."""
    s = -1 if c & 0x80 else 1
    e = (c >> 3) & 0xF
    m = c & 7
    assert not (e == 0xF and m == 7)
    if e == 0:
        return s * Fraction(m, 8) * Fraction(2) ** (-6)
    return s * (1 + Fraction(m, 8)) * Fraction(2) ** (e - 7)


_POS = [e4m3_code_value(c) for c in range(0x7F)]       # ascending: codes 0x00..0x7E


def e4m3_nearest_code(t: Fraction, negative_zero: bool = False) -> int:
    """Code of the representable value nearest to t; ties to the even code; saturates at 448."""
    sign = 0x80 if (t < 0 or (t == 0 and negative_zero)) else 0
    a = abs(t)
    if a >= _POS[-1]:
        return sign | 0x7E
    i = bisect_left(_POS, a)               # _POS[i-1] < a <= _POS[i]
    if _POS[i] == a:
        return sign | i
    lo, hi = i - 1, i
    dl, dh = a - _POS[lo], _POS[hi] - a
    if dl < dh:
        return sign | lo
    if dh < dl:
        return sign | hi
    return sign | (lo if lo % 2 == 0 else hi)


def e4m3_spacing(a: Fraction) -> Fraction:
    """Distance between the representable neighbours around magnitude a (a <= 448)."""
    a = abs(a)
    if a < Fraction(2) ** (-6):
        return Fraction(2) ** (-9)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    if Fraction(2) ** (e + 1) <= a:
        e += 1
    return Fraction(2) ** (e - 3)
