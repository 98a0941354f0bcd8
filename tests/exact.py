"""Exact-rational helpers used to pin the oracle (no floating point anywhere).

A bf16 bit pattern is decoded to a fractions.Fraction from its sign, exponent
and mantissa fields; the nearest bf16 to a rational is found by integer
arithmetic with ties to the even mantissa.  Independent of oracle/ and of numpy
floating point.
"""
from fractions import Fraction


def bf16_to_fraction(bits: int) -> Fraction:
    sign = -1 if bits & 0x8000 else 1
    exp = (bits >> 7) & 0xFF
    man = bits & 0x7F
    if exp == 0xFF:
        raise ValueError("inf/nan")
    if exp == 0:
        return sign * Fraction(man, 1 << 7) * Fraction(1, 1 << 126)
    v = Fraction((1 << 7) | man, 1 << 7)
    e = exp - 127
    return sign * (v * (1 << e) if e >= 0 else v / (1 << -e))


def fraction_to_bf16(x: Fraction) -> int:
    """Nearest bf16 bit pattern to x, ties to even, overflow to infinity."""
    if x == 0:
        return 0
    sign = 0x8000 if x < 0 else 0
    ax = -x if x < 0 else x
    # binary exponent e with 2^e <= ax < 2^(e+1)
    e = ax.numerator.bit_length() - ax.denominator.bit_length()
    if Fraction(2) ** e > ax:
        e -= 1
    if Fraction(2) ** (e + 1) <= ax:
        e += 1
    e = max(e, -126)
    q = Fraction(2) ** (e - 7)          # grid spacing in this binade
    t = ax / q                          # want nearest integer, ties to even
    n = t.numerator // t.denominator
    rem = t - n
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (n & 1)):
        n += 1
    # n in [0, 256]; n == 256 means the value rounded up into the next binade
    if n >= 256:
        n >>= 1
        e += 1
    if e > 127:
        return sign | 0x7F80
    if n < 128:                         # subnormal (only possible with e == -126)
        return sign | n
    return sign | ((e + 127) << 7) | (n - 128)
