"""Exact-rational model of IEEE binary32 arithmetic, for pinning the oracle.

Every operation is carried out on `fractions.Fraction` (no rounding at all) and
then rounded once to the binary32 grid, round-to-nearest-even, subnormals
included.  That is the IEEE-754 definition of a correctly rounded operation; it
uses no floating-point hardware, so it cannot share a contraction, an
extended-precision or a flush-to-zero mistake with compiled code.

Also: a decoder of a generic IEEE-style bit pattern given only its field
widths (Table 1 of arXiv 2309.12381).
"""
from fractions import Fraction
import math
import struct


def bits_of(x: float) -> int:
    return struct.unpack("<I", struct.pack("<f", x))[0]


def float_of(bits: int) -> float:
    return struct.unpack("<f", struct.pack("<I", bits & 0xFFFFFFFF))[0]


def decode(bits: int, ebits: int, mbits: int):
    """Value of an IEEE-style pattern with 1 sign bit, `ebits` exponent bits and
    `mbits` stored significand bits.  Returns a Fraction, or 'inf'/'-inf'/'nan'."""
    sign = -1 if (bits >> (ebits + mbits)) & 1 else 1
    e = (bits >> mbits) & ((1 << ebits) - 1)
    f = bits & ((1 << mbits) - 1)
    bias = (1 << (ebits - 1)) - 1
    if e == (1 << ebits) - 1:
        if f:
            return "nan"
        return "inf" if sign > 0 else "-inf"
    if e == 0:
        return sign * Fraction(f, 1 << mbits) * Fraction(2) ** (1 - bias)
    return sign * (1 + Fraction(f, 1 << mbits)) * Fraction(2) ** (e - bias)


def _floor_log2(q: Fraction) -> int:
    assert q > 0
    e = q.numerator.bit_length() - q.denominator.bit_length()
    # 2^(e-1) < q < 2^(e+1); fix up
    if Fraction(2) ** e > q:
        e -= 1
    assert Fraction(2) ** e <= q < Fraction(2) ** (e + 1)
    return e


def _round_half_even(k: Fraction) -> int:
    fl = k.numerator // k.denominator
    rem = k - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (fl & 1)):
        return fl + 1
    return fl


def rn(q) -> Fraction:
    """Round an exact rational to the nearest binary32 value (ties to even)."""
    q = Fraction(q)
    if q == 0:
        return q
    s = -1 if q < 0 else 1
    a = abs(q)
    e = max(_floor_log2(a), -126)
    quantum = Fraction(2) ** (e - 23)
    r = _round_half_even(a / quantum) * quantum
    assert r < Fraction(2) ** 128, "overflow is outside what these tests exercise"
    return s * r


def sqrt_rn(q) -> Fraction:
    """Correctly rounded binary32 square root of an exact non-negative rational."""
    q = Fraction(q)
    assert q >= 0
    if q == 0:
        return q
    e = _floor_log2(q) // 2            # floor(log2(sqrt(q)))
    e = max(e, -126)
    quantum = Fraction(2) ** (e - 23)
    s = q / (quantum * quantum)         # want round(sqrt(s))
    k = math.isqrt(s.numerator // s.denominator)
    half = Fraction(2 * k + 1, 2)
    if s > half * half or (s == half * half and (k & 1)):
        k += 1
    return k * quantum


def frac_of_f32(x: float) -> Fraction:
    return Fraction(x)                   # every binary32 is an exact rational


def f32_bits_of_frac(q: Fraction, negative_zero: bool = False) -> int:
    """Bit pattern of a rational that lies exactly on the binary32 grid."""
    if q == 0:
        return 0x80000000 if negative_zero else 0
    x = float(q)                         # exact: binary32 values are binary64 values
    assert Fraction(x) == q
    b = bits_of(x)
    assert Fraction(float_of(b)) == q, "value is not on the binary32 grid"
    return b
