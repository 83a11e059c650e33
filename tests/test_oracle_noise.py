"""Pins for the oracle's noise generator and sigma schedulers (CPU only)."""
import math
import os

import numpy as np
import pytest
from scipy import stats

from oracle import nvfp4_oracle as o

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def _kat():
    rows = []
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        c, k, r = (part.split() for part in line.split("|"))
        rows.append(([int(v, 16) for v in c], [int(v, 16) for v in k], [int(v, 16) for v in r]))
    return rows


def test_philox_known_answers():
    rows = _kat()
    assert len(rows) == 3
    for c, k, want in rows:
        got = o.philox4x32_10(np.array([c], dtype=np.uint32), k)[0]
        assert [int(v) for v in got] == want


def test_philox_is_a_bijection_of_the_counter_and_vectorises():
    # distinct counters -> distinct outputs (a keyed permutation); batch call == one at a time
    rng = np.random.default_rng(0)
    ctr = rng.integers(0, 2 ** 32, size=(500, 4), dtype=np.uint64).astype(np.uint32)
    key = (0x12345678, 0x9ABCDEF0)
    out = o.philox4x32_10(ctr, key)
    assert len({tuple(r) for r in out.tolist()}) == len({tuple(r) for r in ctr.tolist()})
    for i in (0, 17, 499):
        assert (o.philox4x32_10(ctr[i:i + 1], key)[0] == out[i]).all()


def test_noise_groups_follow_the_documented_construction():
    """Element 4 b + j comes from counter (b, 0, subsequence) and key = seed: rebuilt here by
    hand for one group from the raw generator output with the Box-Muller identities
    z0^2 + z1^2 = -2 ln u1 and atan2(z1, z0) = 2 pi u2."""
    seed, sub, sigma = 0x1122334455667788, 0x0000000300000009, 0.25
    z = o.aqn_noise_philox(23, sigma, seed, sub) / sigma
    assert z.shape == (23,)
    b = 4
    r = o.philox4x32_10(np.array([[b, 0, sub & 0xFFFFFFFF, sub >> 32]], dtype=np.uint32),
                        (seed & 0xFFFFFFFF, seed >> 32))[0]
    for pair in range(2):
        u1 = ((int(r[2 * pair]) >> 8) + 1) / 2.0 ** 24
        u2 = (int(r[2 * pair + 1]) >> 8) / 2.0 ** 24
        z0, z1 = z[4 * b + 2 * pair], z[4 * b + 2 * pair + 1]
        assert math.isclose(z0 * z0 + z1 * z1, -2.0 * math.log(u1), rel_tol=1e-12)
        ang = math.atan2(z1, z0) % (2 * math.pi)
        assert math.isclose(ang, 2 * math.pi * u2, rel_tol=1e-9, abs_tol=1e-12)
    # a prefix of a longer vector is the shorter vector; other subsequence / seed -> other values
    assert (o.aqn_noise_philox(23, sigma, seed, sub) == o.aqn_noise_philox(64, sigma, seed, sub)[:23]).all()
    assert not np.allclose(z, o.aqn_noise_philox(23, 1.0, seed, sub + 1))
    assert not np.allclose(z, o.aqn_noise_philox(23, 1.0, seed + 1, sub))
    assert o.aqn_noise_philox(0, sigma, seed, sub).shape == (0,)


def test_noise_is_standard_normal_scaled_by_sigma():
    n, sigma = 400_000, 1e-2
    z = o.aqn_noise_philox(n, sigma, 42, 7) / sigma
    assert abs(z.mean()) < 4 / math.sqrt(n)
    assert abs(z.var() - 1.0) < 4 * math.sqrt(2.0 / n)
    assert abs(stats.skew(z)) < 0.02 and abs(stats.kurtosis(z)) < 0.04
    assert stats.kstest(z, "norm").pvalue > 1e-3
    # neighbours, the two halves of a pair, and consecutive forward passes are uncorrelated
    assert abs(np.corrcoef(z[:-1], z[1:])[0, 1]) < 0.01
    assert abs(np.corrcoef(z[0::2], z[1::2])[0, 1]) < 0.01
    z2 = o.aqn_noise_philox(n, sigma, 42, 8) / sigma
    assert abs(np.corrcoef(z, z2)[0, 1]) < 0.01
    # 24-bit uniforms bound the radius: |z| <= sqrt(2 * 24 * ln 2)
    assert np.abs(z).max() <= math.sqrt(48 * math.log(2.0)) + 1e-12


@pytest.mark.parametrize("kind", o.SCHEDULE_KINDS)
def test_schedules_run_from_start_to_end_and_decrease(kind):
    K, s0, s1 = 10, 1e-2, 5e-4
    vals = [o.aqn_sigma_schedule(kind, k, K, s0, s1) for k in range(K + 1)]
    assert vals[0] == 0.0
    assert math.isclose(vals[1], s0, rel_tol=1e-15) and math.isclose(vals[K], s1, rel_tol=1e-12)
    assert all(a > b for a, b in zip(vals[1:], vals[2:]))
    assert o.aqn_sigma_schedule(kind, 1, 1, s0, s1) == s0
    with pytest.raises(ValueError):
        o.aqn_sigma_schedule(kind, K + 1, K, s0, s1)


def test_schedule_shapes():
    K, s0, s1 = 9, 8.0, 2.0
    mid = (K + 1) // 2                                  # u = 1/2
    assert o.aqn_sigma_schedule("exponential", mid, K, s0, s1) == pytest.approx(4.0)      # geometric mean
    assert o.aqn_sigma_schedule("linear", mid, K, s0, s1) == pytest.approx(5.0)           # arithmetic mean
    assert o.aqn_sigma_schedule("cosine", mid, K, s0, s1) == pytest.approx(5.0)           # symmetric about the middle
    assert o.aqn_sigma_schedule("cosine", 2, K, s0, s1) > o.aqn_sigma_schedule("linear", 2, K, s0, s1)   # flat start
    assert o.aqn_sigma_schedule("cosine", K - 1, K, s0, s1) < o.aqn_sigma_schedule("linear", K - 1, K, s0, s1)
    # logarithmic: stage k sits at ln(k) / ln(K) of the way; K = 9 -> stage 3 is half way
    assert o.aqn_sigma_schedule("logarithmic", 3, K, s0, s1) == pytest.approx(5.0)
    assert o.aqn_sigma_schedule("logarithmic", 2, K, s0, s1) < o.aqn_sigma_schedule("linear", 2, K, s0, s1)
    # exponential through the general entry point is Eq. 8
    for k in range(K + 1):
        assert o.aqn_sigma_schedule("exponential", k, K, s0, s1) == o.aqn_sigma(k, K, s0, s1)
    with pytest.raises(ValueError):
        o.aqn_sigma_schedule("stepwise", 1, K, s0, s1)
