"""Exact rational arithmetic used to pin the oracle (pure Python, tiny inputs only).

Two evaluators of the paper's formulas, both independent of the oracle's C:

* ``real_*``      -- the formulas over the rationals, no rounding of
                    intermediates at all.  Valid as an expected value whenever
                    every intermediate is a dyadic rational that binary32 holds
                    exactly (the brute-force grids are built that way).
* ``soft_*``      -- the same formulas with every single operation rounded to
                    the nearest binary32 (ties to even) by ``rn_f32``, a
                    software rounding built from integer arithmetic.  This is
                    what IEEE hardware must produce for any finite input, so it
                    also covers inexact scales such as 1/7.
"""
from fractions import Fraction
import math
import struct

F = Fraction


def rne_int(v: Fraction) -> int:
    """Round a rational to the nearest integer, ties to even (Eq. 1's bracket)."""
    fl = math.floor(v)
    rem = v - fl
    if rem > F(1, 2):
        return fl + 1
    if rem < F(1, 2):
        return fl
    return fl if fl % 2 == 0 else fl + 1


def rn_f32(v: Fraction) -> Fraction:
    """Nearest binary32 value (ties to even), subnormals included, no overflow handling."""
    if v == 0:
        return F(0)
    sign = -1 if v < 0 else 1
    a = abs(v)
    # exponent e with 2^e <= a < 2^(e+1)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if F(2) ** e > a:
        e -= 1
    elif F(2) ** (e + 1) <= a:
        e += 1
    e = max(e, -126)                     # subnormal range shares the exponent -126
    ulp = F(2) ** (e - 23)
    q = rne_int(a / ulp)
    r = q * ulp
    assert r < F(2) ** 128, "overflow"
    return sign * r


def f32_to_fraction(x) -> Fraction:
    """Exact value of a Python float that holds a binary32."""
    return F(float(x))


def fraction_to_float(v: Fraction) -> float:
    return float(v)


# ---------------------------------------------------------------------------
# the paper's formulas over the rationals
# ---------------------------------------------------------------------------

def real_prescale(mn: Fraction, mx: Fraction, bits: int):
    """Eq. 2 / Eq. 5, plus the degenerate-channel reading (s == 0 -> 1)."""
    qmax = 2 ** bits - 1
    s = (mx - mn) / qmax
    if s == 0:
        s = F(1)
    z = rne_int(-mn / s)
    return s, z


def real_code(x: Fraction, s: Fraction, z: int) -> int:
    """Eq. 1, unclamped."""
    return rne_int(x / s + z)


def real_fakequant(x: Fraction, s: Fraction, z: int, bits: int):
    """(clamped code, x_hat, in-range flag): Eq. 1, clamp, Eq. 6."""
    qmax = 2 ** bits - 1
    u = real_code(x, s, z)
    q = min(max(u, 0), qmax)
    return q, s * (q - z), 0 <= u <= qmax


# ---------------------------------------------------------------------------
# the same, every operation rounded to binary32
# ---------------------------------------------------------------------------

FLT_MIN = F(2) ** -126


def soft_prescale(mn: Fraction, mx: Fraction, bits: int):
    qmax = 2 ** bits - 1
    rng = rn_f32(mx - mn)
    s = rn_f32(rng / qmax)
    if not s >= FLT_MIN:
        s = F(1)
    z = rne_int(rn_f32(-mn / s))
    return s, z


def soft_fakequant(x: Fraction, s: Fraction, z: int, bits: int):
    qmax = 2 ** bits - 1
    t = rn_f32(x / s)
    v = rn_f32(t + z)
    u = rne_int(v)
    q = min(max(u, 0), qmax)
    d = rn_f32(F(q - z))
    return q, rn_f32(s * d), 0 <= u <= qmax


def rn_bf16(v: Fraction) -> Fraction:
    """Nearest bfloat16 (8 significant bits, ties to even); normal range only."""
    if v == 0:
        return F(0)
    sign = -1 if v < 0 else 1
    a = abs(v)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if F(2) ** e > a:
        e -= 1
    elif F(2) ** (e + 1) <= a:
        e += 1
    ulp = F(2) ** (e - 7)
    return sign * rne_int(a / ulp) * ulp


def is_f32(v: Fraction) -> bool:
    return rn_f32(v) == v


def f32_bits(x: float) -> int:
    return struct.unpack("<I", struct.pack("<f", x))[0]
