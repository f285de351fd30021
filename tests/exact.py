"""Exact-rational helpers for the tests: correctly rounded binary32 / fp16 / bf16 from Fractions.

Independent of both the oracle and the GPU library (Python integers only)."""
from fractions import Fraction
import struct


def _round_to(fr: Fraction, precision: int, emin: int, emax: int):
    """Nearest-even rounding of a rational to a binary format with `precision` significand bits,
    minimum normal exponent `emin`, maximum exponent `emax`.  Returns (sign, exponent, integer
    significand) with value = (-1)^sign * sig * 2^(exponent - precision + 1); None for overflow."""
    sign = 1 if fr < 0 else 0
    a = -fr if fr < 0 else fr
    if a == 0:
        return sign, emin, 0
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    if Fraction(2) ** (e + 1) <= a:
        e += 1
    e = max(e, emin)
    scaled = a / Fraction(2) ** (e - precision + 1)
    sig = scaled.numerator // scaled.denominator
    rem = scaled - sig
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and sig % 2 == 1):
        sig += 1
    if sig == 1 << precision:
        sig >>= 1
        e += 1
    if e > emax:
        return None
    return sign, e, sig


def f32_round(fr: Fraction) -> Fraction:
    s, e, sig = _round_to(fr, 24, -126, 127)
    v = Fraction(sig) * Fraction(2) ** (e - 23)
    return -v if s else v


def f32_bits(fr: Fraction) -> int:
    """Bit pattern of the binary32 nearest to fr (fr must be in range)."""
    s, e, sig = _round_to(fr, 24, -126, 127)
    if sig < (1 << 23):                      # zero or subnormal
        return (s << 31) | sig
    return (s << 31) | ((e + 127) << 23) | (sig - (1 << 23))


def f16_bits(fr: Fraction) -> int:
    r = _round_to(fr, 11, -14, 15)
    if r is None:
        return (0x8000 if fr < 0 else 0) | 0x7C00
    s, e, sig = r
    if sig < (1 << 10):
        return (s << 15) | sig
    return (s << 15) | ((e + 15) << 10) | (sig - (1 << 10))


def bf16_bits(fr: Fraction) -> int:
    s, e, sig = _round_to(fr, 8, -126, 127)
    if sig < (1 << 7):
        return (s << 15) | sig
    return (s << 15) | ((e + 127) << 7) | (sig - (1 << 7))


def f16_value(bits: int) -> Fraction:
    s = bits >> 15
    e = (bits >> 10) & 0x1F
    m = bits & 0x3FF
    assert e != 0x1F
    v = Fraction(m, 1 << 24) if e == 0 else Fraction((1 << 10) + m) * Fraction(2) ** (e - 25)
    return -v if s else v


def f32_value(bits: int) -> Fraction:
    return Fraction(struct.unpack("<f", struct.pack("<I", bits))[0])
