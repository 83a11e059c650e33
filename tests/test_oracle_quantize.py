"""Pins for the oracle's NVFP4 quantiser / dequantiser (CPU only)."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import nvfp4_oracle as o
from tests import cases
from tests import exact_ref as ex


def _unpack(codes):
    N, K2 = codes.shape
    c = np.empty((N, 2 * K2), dtype=np.uint8)
    c[:, 0::2] = codes & 15
    c[:, 1::2] = codes >> 4
    return c


@pytest.mark.parametrize("name", list(cases.quantizer_cases(3, 32).keys()))
def test_quantize_matches_exact_rational_chain(name):
    """Brute force: the fp32 chain re-evaluated in exact rationals with
    arithmetic roundings must give the same bytes."""
    W = cases.quantizer_cases(3, 32, seed=11)[name]
    codes, scales, S32 = o.nvfp4_quantize(W)
    ecodes, escales, eS32 = ex.quantize_exact(W.tolist())
    assert Fraction(float(S32)) == eS32
    assert scales.tolist() == escales
    assert _unpack(codes).tolist() == ecodes


def test_worked_example_scale_chain():
    """amax = 0.09375: S32 = amax/2688; a block with maximum 0.0625 gets
    v = 298.67 -> E4M3 288 (0x79, rounded down), so its maximum saturates at 6."""
    W = np.zeros((1, 32), dtype=np.float32)
    W[0, 0] = 0.09375
    W[0, 16] = 0.0625
    W[0, 17] = -0.03125
    codes, scales, S32 = o.nvfp4_quantize(W)
    assert float(S32) == float.fromhex("0x1.24924ap-15")
    assert scales.tolist() == [[0x7E, 0x79]]
    c = _unpack(codes)
    assert c[0, 0] == 7 and c[0, 16] == 7          # both saturate / hit 6
    d = np.float32(S32) * np.float32(288.0)
    assert abs(float(d) - 0.010044643) < 1e-9
    Wh = o.nvfp4_dequantize(codes, scales, S32)
    assert abs(float(Wh[0, 16]) - 0.06026786) < 1e-8
    # -0.03125/d = -3.11 -> -3  (code 8|5)
    assert c[0, 17] == (8 | 5)


def test_representable_roundtrip_is_exact():
    for p in (-9, 0, 5):
        W, sbytes, S32 = cases.representable(16, 256, seed=3, p=p)
        codes, scales, ts = o.nvfp4_quantize(W)
        assert ts == S32
        assert np.array_equal(scales, sbytes)
        assert np.array_equal(o.nvfp4_dequantize(codes, scales, ts), W)


def test_error_bound_per_element():
    """|W_hat - W| <= d * half the local E2M1 spacing; saturated elements
    (|q| > 6, possible because the block scale is rounded to nearest) are off
    by at most 0.4 d."""
    W = cases.gaussian(64, 512, seed=5)
    codes, scales, S32 = o.nvfp4_quantize(W)
    Wh = o.nvfp4_dequantize(codes, scales, S32).astype(np.float64)
    d = np.repeat(np.float64(S32) * o.e4m3_decode(scales).astype(np.float64), 16, axis=1)
    assert np.all(d > 0)
    q = np.abs(W.astype(np.float64)) / d
    err = np.abs(Wh - W.astype(np.float64)) / d
    slack = 1e-6
    assert np.all(err[q <= 2] <= 0.25 + slack)
    assert np.all(err[(q > 2) & (q <= 4)] <= 0.5 + slack)
    assert np.all(err[(q > 4) & (q <= 6)] <= 1.0 + slack)
    assert q.max() <= 6.0 / (1 - 2.0 ** -4) + 1e-3
    assert np.all(err[q > 6] <= 0.4 + 1e-3)
    assert (q > 6).sum() > 0                       # the case does occur
    # block maxima map to |code| >= 4 (they are within rounding of 6)
    blk_max_code = (_unpack(codes) & 7).reshape(64, 32, 16).max(axis=2)
    assert np.all(blk_max_code >= 6)


def test_sign_symmetry_and_pow2_scaling_and_row_permutation():
    W = cases.gaussian(8, 128, seed=9)
    c0, s0, t0 = o.nvfp4_quantize(W)
    c1, s1, t1 = o.nvfp4_quantize(-W)
    assert np.array_equal(s0, s1) and t0 == t1
    assert np.array_equal(c0 ^ 0x88, c1)
    for p in (-20, 7):
        c2, s2, t2 = o.nvfp4_quantize(W * np.float32(2.0 ** p))
        assert np.array_equal(c0, c2) and np.array_equal(s0, s2)
        assert t2 == np.float32(t0 * np.float32(2.0 ** p))
    perm = np.random.default_rng(1).permutation(8)
    c3, s3, t3 = o.nvfp4_quantize(W[perm])
    assert np.array_equal(c3, c0[perm]) and np.array_equal(s3, s0[perm]) and t3 == t0


def test_layout_nibbles_and_scale_plane():
    W = np.zeros((2, 48), dtype=np.float32)
    W[0, 0] = 6.0       # amax -> S32 = 6/2688, block (0,0) scale 448
    W[1, 33] = -3.0     # row 1, block 2, odd k -> high nibble of byte 16
    codes, scales, S32 = o.nvfp4_quantize(W)
    assert codes.shape == (2, 24) and scales.shape == (2, 3)
    assert codes[0, 0] == 0x07                      # even k in the low nibble
    assert scales[0, 0] == 0x7E and scales[1, 2] == 0x76   # 224 = 1.75 * 2^7
    assert codes[1, 16] == ((8 | 7) << 4)
    nz = np.argwhere(codes)
    assert nz.tolist() == [[0, 0], [1, 16]]
    assert np.argwhere(scales).tolist() == [[0, 0], [1, 2]]


def test_zero_tensor_and_zero_blocks_and_signed_zero():
    W = cases.all_zero(2, 32)
    codes, scales, S32 = o.nvfp4_quantize(W)
    assert S32 == np.float32(1.0) and not scales.any()
    assert codes[0, 0] == 0x80 and codes.sum() == 0x80      # only the -0 sign bit
    Wh = o.nvfp4_dequantize(codes, scales, S32)
    assert not Wh.any() and np.signbit(Wh[0, 1])
    W = cases.outlier(8, 128, seed=2)
    codes, scales, S32 = o.nvfp4_quantize(W)
    assert (scales == 0).sum() > 0                 # flushed blocks exist
    mags = (_unpack(codes) & 7).reshape(8, 8, 16)
    assert not mags[scales == 0].any()             # and hold only zeros


def test_rejects_bad_input():
    with pytest.raises(ValueError):
        o.nvfp4_quantize(np.zeros((2, 24), dtype=np.float32))
    W = np.zeros((1, 16), dtype=np.float32)
    W[0, 3] = np.inf
    with pytest.raises(ValueError):
        o.nvfp4_quantize(W)


def test_dequantize_is_eq6_elementwise():
    rng = np.random.default_rng(4)
    codes = rng.integers(0, 256, size=(3, 16)).astype(np.uint8)
    scales = rng.integers(0, 0x7F, size=(3, 2)).astype(np.uint8)
    S32 = np.float32(0.37)
    Wh = o.nvfp4_dequantize(codes, scales, S32)
    mags = [0, .5, 1, 1.5, 2, 3, 4, 6]
    for n in range(3):
        for k in range(32):
            b = int(codes[n, k // 2])
            c = (b >> 4) if k % 2 else (b & 15)
            sb = int(scales[n, k // 16])
            e, m = sb >> 3, sb & 7
            s = (m / 8) * 2.0 ** -6 if e == 0 else (1 + m / 8) * 2.0 ** (e - 7)
            val = mags[c & 7] * (-1 if c & 8 else 1)
            want = np.float32(S32) * np.float32(s * val)
            assert Wh[n, k] == want


# (tensor amax, block amax) pairs, found by scanning bf16 values, on which the
# order of the two divisions changes the scale byte: (bamax/6)/S32 as specified
# versus (bamax/S32)/6 or bamax/(6*S32).
ORDER_SENSITIVE = [
    (0.0064697265625, 0.004852294921875),
    (0.008544921875, 0.00762939453125),
    (0.0093994140625, 0.006378173828125),
    (0.0111083984375, 0.007537841796875),
    (0.013671875, 0.005615234375),
    (0.013671875, 0.01123046875),
]


def test_division_order_of_scale_chain_is_pinned():
    r32, F = ex.r32, Fraction
    discriminating = 0
    for amax, bamax in ORDER_SENSITIVE:
        W = np.zeros((1, 32), dtype=np.float32)
        W[0, 5] = -amax
        W[0, 20] = bamax
        codes, scales, S32 = o.nvfp4_quantize(W)
        S = r32(F(amax) / 2688)
        spec = ex.e4m3_byte(ex.e4m3_value(r32(r32(F(bamax) / 6) / S)))
        alt1 = ex.e4m3_byte(ex.e4m3_value(r32(r32(F(bamax) / S) / 6)))
        alt2 = ex.e4m3_byte(ex.e4m3_value(r32(F(bamax) / r32(6 * S))))
        alt3 = ex.e4m3_byte(ex.e4m3_value(F(bamax) / 6 / S))          # unrounded quotient
        assert int(scales[0, 1]) == spec
        discriminating += (spec != alt1) + (spec != alt2) + (spec != alt3)
        assert spec != alt1 or spec != alt2
    assert discriminating >= len(ORDER_SENSITIVE)
