"""Exact rational arithmetic used to pin the oracle (test-side only).

Nothing here is shared with oracle/ or with the HIP path: 16-bit patterns are decoded with
integer arithmetic into fractions.Fraction, rounding is done on integers, and fp32 values
enter as Fractions of numpy float32 scalars.
"""
from __future__ import annotations

from fractions import Fraction

import numpy as np


def frac_of_f16(bits: int) -> Fraction | None:
    sign = -1 if bits >> 15 else 1
    e, f = (bits >> 10) & 0x1F, bits & 0x3FF
    if e == 31:
        return None
    if e == 0:
        return sign * Fraction(f, 1 << 24)
    return sign * Fraction(1024 + f, 1024) * Fraction(2) ** (e - 15)


def frac_of_bf16(bits: int) -> Fraction | None:
    sign = -1 if bits >> 15 else 1
    e, f = (bits >> 7) & 0xFF, bits & 0x7F
    if e == 255:
        return None
    if e == 0:
        return sign * Fraction(f, 128) * Fraction(2) ** (-126)
    return sign * Fraction(128 + f, 128) * Fraction(2) ** (e - 127)


def frac_of(bits: int, dtype: str) -> Fraction | None:
    return frac_of_f16(bits) if dtype == "f16" else frac_of_bf16(bits)


def round_half_even(p: Fraction) -> int:
    n, d = p.numerator, p.denominator
    fl = n // d
    rem = p - fl
    if rem > Fraction(1, 2):
        return fl + 1
    if rem < Fraction(1, 2):
        return fl
    return fl if fl % 2 == 0 else fl + 1


def inv_scale_f32(s) -> Fraction:
    """fl32(1/s) via numpy's float32 division."""
    return Fraction(float(np.float32(1.0) / np.float32(s)))


def quantize_exact(bits: int, dtype: str, s, nbits: int):
    """(r, m, q, p) with p = x * fl32(1/s) exact; infinities saturate with m = 0."""
    Qn, Qp = -(1 << (nbits - 1)), (1 << (nbits - 1)) - 1
    x = frac_of(bits, dtype)
    inv = inv_scale_f32(s)
    if x is None:  # +-inf
        neg = bool(bits >> 15) != (inv < 0)
        return (None, 0, Qn if neg else Qp, None)
    p = x * inv
    r = round_half_even(p)
    m = 1 if Qn <= r <= Qp else 0
    q = min(max(r, Qn), Qp)
    return (r, m, q, p)


def quantize_ideal(bits: int, dtype: str, s, nbits: int) -> int | None:
    """clamp(RHE(x / s)) with the true quotient (no reciprocal), exact."""
    Qn, Qp = -(1 << (nbits - 1)), (1 << (nbits - 1)) - 1
    x = frac_of(bits, dtype)
    if x is None:
        return None
    r = round_half_even(x / Fraction(float(np.float32(s))))
    return min(max(r, Qn), Qp)
