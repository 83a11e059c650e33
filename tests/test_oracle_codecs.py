"""Pins for the oracle's number formats: what the paper prints (tests/golden),
closed forms, exhaustive enumeration and an exact-arithmetic brute force."""
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import nvfp4_oracle as o
from tests import exact_ref as ex

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _facts():
    out = {}
    for line in open(os.path.join(GOLDEN, "paper_facts.txt")):
        line = line.split("#")[0].strip()
        if line:
            k, v = [t.strip() for t in line.split("=")]
            out[k] = float(v)
    return out


def test_e2m1_table_matches_printed_magnitudes():
    rows = [l for l in open(os.path.join(GOLDEN, "e2m1_magnitudes.txt")) if not l.startswith("#")]
    want = [float(t) for t in rows[0].split()]
    got = [float(o.e2m1_decode(c)) for c in range(8)]
    assert got == want
    assert [float(o.e2m1_decode(c | 8)) for c in range(1, 8)] == [-w for w in want[1:]]
    assert np.signbit(o.e2m1_decode(8))            # code 8 is -0
    f = _facts()
    assert max(got) == f["e2m1_qmax"]
    assert o.BLOCK == f["nvfp4_block"]
    # structure: 2 exponent bits, 1 mantissa bit  =>  8 magnitudes, spacing doubles per binade
    assert len(got) == 2 ** int(f["e2m1_exponent_bits"] + f["e2m1_mantissa_bits"])


def test_e4m3_landmarks():
    for line in open(os.path.join(GOLDEN, "e4m3_landmarks.txt")):
        if line.startswith("#") or not line.strip():
            continue
        b, v = line.split()
        assert float(o.e4m3_decode(int(b, 16))) == float(v)


def test_e4m3_closed_form_exhaustive_and_monotone():
    vals = []
    for b in range(0x7F):
        e, m = b >> 3, b & 7
        want = Fraction(m, 8) * Fraction(2) ** -6 if e == 0 else (1 + Fraction(m, 8)) * Fraction(2) ** (e - 7)
        got = Fraction(float(o.e4m3_decode(b)))
        assert got == want
        assert int(o.e4m3_encode(np.float32(float(want)))) == b      # enc(dec(b)) == b
        vals.append(want)
    assert all(a < b for a, b in zip(vals, vals[1:]))
    with pytest.raises(ValueError):
        o.e4m3_decode(0x7F)
    with pytest.raises(ValueError):
        o.e4m3_decode(0x80)


def test_e4m3_encode_against_exact_rounding():
    rng = np.random.default_rng(0)
    v = np.concatenate([
        np.exp2(rng.uniform(-14, 9.2, 4000)),
        np.array([0.0, 2.0 ** -10, 2.0 ** -10 * 1.0001, 2.0 ** -10 * 0.9999, 3 * 2.0 ** -10,
                  447.9, 448.0, 464.0, 463.9, 480.0, 1e6, 2.0 ** -9, 2.0 ** -20]),
    ]).astype(np.float32)
    # all midpoints between neighbouring values, and their fp32 neighbours
    g = o.E4M3_GRID
    mid = ((g[:-1] + g[1:]) / 2).astype(np.float32)
    v = np.concatenate([v, mid, np.nextafter(mid, np.float32(0)), np.nextafter(mid, np.float32(1e9))])
    got = o.e4m3_encode(v)
    for x, b in zip(v, got):
        assert int(b) == ex.e4m3_byte(ex.e4m3_value(Fraction(float(x)))), float(x)


def test_e2m1_tie_table_and_saturation():
    # ties go to the value whose mantissa bit is 0
    tie = {0.25: 0.0, 0.75: 1.0, 1.25: 1.0, 1.75: 2.0, 2.5: 2.0, 3.5: 4.0, 5.0: 4.0}
    for q, want in tie.items():
        assert float(o.E2M1_GRID[o.e2m1_encode_magnitude(np.float32(q))]) == want
        lo = np.nextafter(np.float32(q), np.float32(0))
        hi = np.nextafter(np.float32(q), np.float32(10))
        assert float(o.E2M1_GRID[o.e2m1_encode_magnitude(lo)]) < q
        assert float(o.E2M1_GRID[o.e2m1_encode_magnitude(hi)]) > q
    for q in [6.0, 6.2, 6.4, 100.0]:
        assert int(o.e2m1_encode_magnitude(np.float32(q))) == 7


def test_e2m1_encode_minimises_distance_dense_sweep():
    q = np.linspace(0, 7, 28001).astype(np.float32)
    idx = o.e2m1_encode_magnitude(q)
    grid = np.array([0, .5, 1, 1.5, 2, 3, 4, 6])
    dist = np.abs(q.astype(np.float64)[:, None] - grid[None, :])
    best = dist.min(axis=1)
    assert np.all(np.abs(q - grid[idx]) == best)
    for x, i in zip(q[::97], idx[::97]):
        assert int(i) == ex.e2m1_index(ex.e2m1_value(Fraction(float(x))))


def test_sigma_schedule():
    f = _facts()
    K = int(f["sigma_stages"])
    s = [o.aqn_sigma(k, K, f["sigma_start"], f["sigma_end"]) for k in range(K + 1)]
    assert s[0] == 0.0                                    # stage 0: quantisation noise only
    assert s[1] == 1e-2                                   # Eq. (8) at k = 1
    assert abs(s[K] - 5e-4) < 1e-18                       # Eq. (8) at k = K
    # geometric: constant ratio (sigma_end/sigma_start)^(1/(K-1)), independent high-precision value
    from decimal import Decimal, getcontext
    getcontext().prec = 40
    ratio = (Decimal("5e-4") / Decimal("1e-2")).ln() / Decimal(K - 1)
    for k in range(1, K + 1):
        want = Decimal("1e-2") * (ratio * (k - 1)).exp()
        assert abs(Decimal(s[k]) - want) < Decimal("1e-17")
    assert all(a > b for a, b in zip(s[1:], s[2:]))
    with pytest.raises(ValueError):
        o.aqn_sigma(K + 1, K, 1e-2, 5e-4)
