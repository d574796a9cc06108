"""Exact rational arithmetic helpers for pinning the oracle (CPU only).

Everything here works on ``fractions.Fraction`` and Python integers, so there
is no floating-point rounding anywhere except the one being defined:
``round_to_format`` is round-to-nearest, ties-to-even, into a binary format
given by its precision and exponent range.
"""
from __future__ import annotations

import struct
from fractions import Fraction

# (precision bits incl. hidden one, min normal exponent, max exponent, exponent field bits)
FORMATS = {
    "f32": (24, -126, 127, 8),
    "f16": (11, -14, 15, 5),
    "bf16": (8, -126, 127, 8),
}


def _floor_log2(q: Fraction) -> int:
    """Largest e with 2**e <= q, for q > 0."""
    e = q.numerator.bit_length() - q.denominator.bit_length()
    if Fraction(2) ** e > q:
        e -= 1
    assert Fraction(2) ** e <= q < Fraction(2) ** (e + 1)
    return e


def round_to_format(q: Fraction, fmt: str):
    """RNE of the rational q; returns ('fin', Fraction) or ('inf', sign)."""
    p, emin, emax, _ = FORMATS[fmt]
    if q == 0:
        return ("fin", Fraction(0))
    sign = -1 if q < 0 else 1
    a = abs(q)
    e = max(_floor_log2(a), emin)
    ulp = Fraction(2) ** (e - (p - 1))
    n = a / ulp                      # exact rational; want nearest integer, ties to even
    lo = n.numerator // n.denominator
    frac = n - lo
    if frac > Fraction(1, 2) or (frac == Fraction(1, 2) and lo % 2 == 1):
        lo += 1
    val = lo * ulp
    if val >= Fraction(2) ** (emax + 1):
        return ("inf", sign)
    return ("fin", sign * val)


def bits_to_fraction(bits: int, fmt: str) -> Fraction:
    """Decode a finite bit pattern of the format into its exact value."""
    p, emin, emax, ebits = FORMATS[fmt]
    mbits = p - 1
    sign = -1 if (bits >> (ebits + mbits)) & 1 else 1
    e = (bits >> mbits) & ((1 << ebits) - 1)
    m = bits & ((1 << mbits) - 1)
    assert e != (1 << ebits) - 1, "not finite"
    if e == 0:
        return sign * m * Fraction(2) ** (emin - mbits)
    bias = (1 << (ebits - 1)) - 1
    return sign * (m + (1 << mbits)) * Fraction(2) ** (e - bias - mbits)


def fraction_to_bits(q: Fraction, fmt: str, negative_zero: bool = False) -> int:
    """Bit pattern of a value that is exactly representable in the format."""
    p, emin, emax, ebits = FORMATS[fmt]
    mbits = p - 1
    signbit = 1 << (ebits + mbits)
    if q == 0:
        return signbit if negative_zero else 0
    s = signbit if q < 0 else 0
    a = abs(q)
    e = _floor_log2(a)
    bias = (1 << (ebits - 1)) - 1
    if e < emin:
        m = a / Fraction(2) ** (emin - mbits)
        assert m.denominator == 1
        return s | int(m)
    m = a / Fraction(2) ** (e - mbits)
    assert m.denominator == 1 and (1 << mbits) <= m < (2 << mbits)
    return s | ((e + bias) << mbits) | (int(m) - (1 << mbits))


def f32_fraction(f: float) -> Fraction:
    """Exact value of the fp32 nearest to the Python float f (must be exact)."""
    (u,) = struct.unpack("<I", struct.pack("<f", f))
    return bits_to_fraction(u, "f32")


def is_correctly_rounded_rsqrt(f: Fraction, D: Fraction, fmt: str = "f32") -> bool:
    """True iff f is the RNE of 1/sqrt(D) in the format, decided exactly.

    t = 1/sqrt(D) is irrational in general; f is its rounding iff t lies
    strictly between the midpoints to f's neighbours, i.e. iff
    m_lo^2 * D < 1 < m_hi^2 * D (all rational).  Ties cannot occur unless t is
    itself a midpoint, in which case the strict test fails and the caller
    must pick another input.
    """
    p, emin, emax, _ = FORMATS[fmt]
    assert f > 0 and D > 0
    e = max(_floor_log2(f), emin)
    ulp = Fraction(2) ** (e - (p - 1))
    # the neighbour below has a smaller spacing when f is a power of two
    ulp_lo = ulp / 2 if (f == Fraction(2) ** e and e > emin) else ulp
    m_lo = f - ulp_lo / 2
    m_hi = f + ulp / 2
    return m_lo * m_lo * D < 1 < m_hi * m_hi * D
