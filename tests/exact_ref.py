"""Exact rational arithmetic with explicit IEEE rounding, used to brute-force
the quantiser chain on tiny inputs.  Independent of oracle/: roundings are
done arithmetically (scale to an integer, round half to even), not by
searching a table of representable values."""
from fractions import Fraction
import math


def _floor_log2(v: Fraction) -> int:
    assert v > 0
    e = v.numerator.bit_length() - v.denominator.bit_length()
    if Fraction(2) ** e > v:
        e -= 1
    assert Fraction(2) ** e <= v < Fraction(2) ** (e + 1)
    return e


def _round_half_even(v: Fraction) -> int:
    f = math.floor(v)
    r = v - f
    if r > Fraction(1, 2) or (r == Fraction(1, 2) and f % 2 == 1):
        return f + 1
    return f


def round_minifloat(v: Fraction, mant_bits: int, emin: int, vmax: Fraction) -> Fraction:
    """Nearest-even value of a binary float format with `mant_bits` fraction
    bits and smallest normal exponent `emin` (subnormals below), saturating."""
    if v == 0:
        return Fraction(0)
    sign = -1 if v < 0 else 1
    v = abs(v)
    e = max(_floor_log2(v), emin)
    quantum = Fraction(2) ** (e - mant_bits)
    out = _round_half_even(v / quantum) * quantum
    return sign * min(out, vmax)


F32_MAX = (Fraction(2) - Fraction(2) ** -23) * Fraction(2) ** 127


def r32(v: Fraction) -> Fraction:
    return round_minifloat(v, 23, -126, F32_MAX)


def e4m3_value(v: Fraction) -> Fraction:
    return round_minifloat(v, 3, -6, Fraction(448))


def e2m1_value(v: Fraction) -> Fraction:
    return round_minifloat(v, 1, 0, Fraction(6))


def e4m3_byte(val: Fraction) -> int:
    if val == 0:
        return 0
    if val < Fraction(2) ** -6:
        m = val / Fraction(2) ** -9
        assert m.denominator == 1
        return int(m)
    e = _floor_log2(val)
    m = (val / Fraction(2) ** e - 1) * 8
    assert m.denominator == 1 and 0 <= m < 8
    return ((e + 7) << 3) | int(m)


def e2m1_index(val: Fraction) -> int:
    if val < 1:
        m = val * 2
        assert m.denominator == 1
        return int(m)
    e = _floor_log2(val)
    m = (val / Fraction(2) ** e - 1) * 2
    assert m.denominator == 1
    return ((e + 1) << 1) | int(m)


def quantize_exact(rows):
    """rows: list of lists of Python floats (bf16 values).  Returns
    (code nibbles [N][K], scale bytes [N][K/16], tensor scale Fraction)
    following  S32 = amax/2688 ; S8 = E4M3(bamax/6/S32) ; code = E2M1(w/(S32*S8)),
    every operation rounded to fp32."""
    W = [[Fraction(w) for w in row] for row in rows]
    neg = [[math.copysign(1.0, w) < 0 for w in row] for row in rows]
    amax = max(abs(w) for row in W for w in row)
    S32 = Fraction(1) if amax == 0 else r32(amax / 2688)
    codes, scales = [], []
    for row, nrow in zip(W, neg):
        crow, srow = [], []
        for j in range(0, len(row), 16):
            blk = row[j:j + 16]
            bamax = max(abs(w) for w in blk)
            v = r32(r32(bamax / 6) / S32)
            s8 = e4m3_value(v)
            srow.append(e4m3_byte(s8))
            d = r32(S32 * s8)
            for w, ng in zip(blk, nrow[j:j + 16]):
                mag = Fraction(0) if d == 0 else e2m1_value(r32(abs(w) / d))
                crow.append(e2m1_index(mag) | (8 if ng else 0))
        codes.append(crow)
        scales.append(srow)
    return codes, scales, S32
