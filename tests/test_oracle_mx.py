"""Pins for the MXFP4 / MXFP8 oracle (CPU only)."""
import numpy as np
import pytest

from oracle import mx_oracle as mx
from oracle import nvfp4_oracle as o


def _block(vals):
    v = np.zeros((1, 32), dtype=np.float32)
    v[0, :len(vals)] = vals
    return v


def test_e8m0_is_a_bare_power_of_two():
    assert mx.e8m0_decode(np.array([127, 0, 254, 128, 126], dtype=np.uint8)).tolist() == \
        [1.0, 2.0 ** -127, 2.0 ** 127, 2.0, 0.5]
    with pytest.raises(ValueError):
        mx.e8m0_decode(np.array([255], dtype=np.uint8))


@pytest.mark.parametrize("amax,byte,top_code", [
    (6.0, 127, 7),      # floor(log2 6) = 2, X = 0: the block maximum is exactly the largest element
    (4.0, 127, 6),      # X = 0, 4 is an element
    (3.9, 126, 7),      # floor(log2 3.9) = 1, X = -1: 3.9 / 0.5 = 7.8 saturates at 6 (the rule's known clamp)
    (8.0, 128, 6),      # X = 1: 8 / 2 = 4
    (7.0, 127, 7),      # X = 0: 7 rounds... saturates to 6
    (0.5, 124, 6),      # floor(log2 .5) = -1, X = -3: .5 * 8 = 4
    (1.0, 125, 6),      # X = -2: 1 * 4 = 4
])
def test_mxfp4_shared_exponent_worked_examples(amax, byte, top_code):
    """Hand-derived from the MX conversion rule: X = floor(log2(amax)) - 2."""
    codes, scales = mx.mxfp4_quantize(_block([amax, -amax / 2]))
    assert scales[0, 0] == byte
    assert codes[0, 0] & 0x7 == top_code and (codes[0, 0] >> 4) & 0x8 == 0x8     # second element negative


def test_mxfp4_zero_block_and_signed_zero():
    codes, scales = mx.mxfp4_quantize(_block([0.0, -0.0]))
    assert scales[0, 0] == 0 and codes[0, 0] == 0x80 and not codes[0, 1:].any()   # -0 keeps its sign bit


def test_mxfp4_representable_tensors_round_trip_exactly():
    rng = np.random.default_rng(1)
    N, K = 6, 128
    exps = rng.integers(-20, 20, size=(N, K // 32))
    codes = rng.integers(0, 16, size=(N, K)).astype(np.uint8)
    codes[:, 0::32] = 7                       # every block holds a 6: its shared exponent is the block's own
    W = (o.e2m1_decode(codes).astype(np.float64).reshape(N, K // 32, 32) * np.ldexp(1.0, exps)[:, :, None]).reshape(N, K)
    c, s = mx.mxfp4_quantize(W.astype(np.float32))
    assert (s.astype(int) - 127 == exps).all()
    assert (mx.mxfp4_dequantize(c, s) == W).all()
    # nibble order: low nibble = even k
    assert c[0, 0] & 0xF == codes[0, 0] and c[0, 0] >> 4 == codes[0, 1]


def test_mxfp4_error_bound_and_ties():
    rng = np.random.default_rng(2)
    W = (rng.standard_normal((8, 256)) * 0.02).astype(np.float32)
    c, s = mx.mxfp4_quantize(W)
    What = mx.mxfp4_dequantize(c, s)
    scale = np.repeat(mx.e8m0_decode(s), 32, axis=1)
    q = np.abs(W.astype(np.float64)) / scale
    # below the saturation point the error is at most half a grid step (steps 0.5 up to 2, 1 up to 4, 2 up to 6)
    step = np.where(q < 2, 0.5, np.where(q < 4, 1.0, 2.0))
    ok = q <= 6
    assert (np.abs(What - W)[ok] <= (step * scale / 2)[ok] + 1e-30).all()
    assert (np.abs(What)[~ok] == (6 * scale)[~ok]).all()
    # ties go to the even code: 2.5 -> 2 (code 4), 3.5 -> 4 (code 6), 0.25 -> 0, 0.75 -> 1
    c, s = mx.mxfp4_quantize(_block([6.0, 2.5, 3.5, 0.25, 0.75, 5.0]))
    nib = [c[0, 0] & 0xF, c[0, 0] >> 4, c[0, 1] & 0xF, c[0, 1] >> 4, c[0, 2] & 0xF, c[0, 2] >> 4]
    assert nib == [7, 4, 6, 0, 2, 6]          # 5.0 ties between 4 and 6 -> 4 (code 6, even index)


def test_mxfp8_worked_examples_and_round_trip():
    # amax 448 -> X = 8 - 8 = 0; 1.0 -> X = -8: 1 * 256 = 256 (E4M3 0x78); 500 -> X = 0, saturates at 448
    for amax, byte, top in [(448.0, 127, 0x7E), (1.0, 119, 0x78), (500.0, 127, 0x7E), (0.0, 0, 0x00)]:
        c, s = mx.mxfp8_quantize(_block([amax, -amax]))
        assert s[0, 0] == byte and c[0, 0] == top and c[0, 1] == (top | 0x80)
    rng = np.random.default_rng(3)
    codes = rng.integers(0, 0x7F, size=(4, 64)).astype(np.uint8) | (rng.integers(0, 2, size=(4, 64)).astype(np.uint8) << 7)
    codes[:, 0::32] = 0x7E
    exps = rng.integers(-30, 30, size=(4, 2))
    x = mx.mxfp8_dequantize(codes, (exps + 127).astype(np.uint8))
    c, s = mx.mxfp8_quantize(x.astype(np.float32))
    assert (s.astype(int) - 127 == exps).all()
    assert (mx.mxfp8_dequantize(c, s) == x).all()
    # relative error of an element is at most 2^-4 (3 mantissa bits) unless it falls into the block's subnormals
    x = rng.standard_normal((4, 128)).astype(np.float32)
    c, s = mx.mxfp8_quantize(x)
    xq = mx.mxfp8_dequantize(c, s)
    scale = np.repeat(mx.e8m0_decode(s), 32, axis=1)
    q = np.abs(x.astype(np.float64)) / scale
    normal = (q >= 2.0 ** -6) & (q <= 448)        # neither in the block's subnormal range nor beyond the largest element
    assert (np.abs(xq - x)[normal] <= 2.0 ** -4 * np.abs(x)[normal]).all()
    assert (np.abs(xq)[q > 448] == (448 * scale)[q > 448]).all()       # the rule's clamp: up to 12.5 % for a block maximum
    assert (q < 512).all()


def test_linears_are_the_products_of_their_dequantised_operands():
    rng = np.random.default_rng(4)
    W = (rng.standard_normal((5, 96)) * 0.02).astype(np.float32)
    x = rng.standard_normal((3, 96)).astype(np.float32)
    c, s = mx.mxfp4_quantize(W)
    # one-hot activations read dequantised columns; one-hot weights read (quantised) activations
    eye = np.zeros((1, 96), dtype=np.float32); eye[0, 37] = 1.0
    assert (mx.mx_linear_weight_only(eye, c, s)[0] == mx.mxfp4_dequantize(c, s)[:, 37]).all()
    assert (mx.mx_linear_native(eye, c, s)[0] == mx.mxfp4_dequantize(c, s)[:, 37]).all()       # 1.0 is exact in MXFP8
    ref = np.zeros((3, 5))
    What = mx.mxfp4_dequantize(c, s)
    for m in range(3):
        for n in range(5):
            ref[m, n] = sum(float(x[m, k]) * What[n, k] for k in range(96))
    assert np.allclose(mx.mx_linear_weight_only(x, c, s), ref, rtol=1e-13, atol=1e-15)
    xq = mx.mxfp8_dequantize(*mx.mxfp8_quantize(x))
    assert np.allclose(mx.mx_linear_native(x, c, s), xq @ What.T, rtol=1e-13, atol=1e-15)
    # the native path differs from the weight-only one by the activation rounding only: a few percent of a row's scale
    d = np.abs(mx.mx_linear_native(x, c, s) - mx.mx_linear_weight_only(x, c, s))
    assert d.max() <= 2.0 ** -4 * (np.abs(x) @ np.abs(What).T).max()


def test_native_linear_with_lora_and_bias_by_loops_and_special_cases():
    """Eq. (2) on top of the native product: brute-force loops; the adapter reads the UNquantised activations (a rank-1
    adapter that copies one activation shows it); zero B, zero scale and no adapter reduce to the plain native linear;
    the dense merge W_hat + s B A reproduces the weight-only variant of the same sum."""
    rng = np.random.default_rng(9)
    N, K, M, r = 6, 64, 4, 3
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    x = rng.standard_normal((M, K)).astype(np.float32)
    A = rng.standard_normal((r, K)).astype(np.float32)
    B = rng.standard_normal((N, r)).astype(np.float32)
    bias = rng.standard_normal(N).astype(np.float32)
    c, s = mx.mxfp4_quantize(W)
    base = mx.mx_linear_native(x, c, s)
    y = mx.mx_lora_linear_native(x, c, s, A, B, 0.5, bias)
    ref = np.zeros((M, N))
    for m in range(M):
        for n in range(N):
            t = [sum(float(x[m, k]) * float(A[j, k]) for k in range(K)) for j in range(r)]
            ref[m, n] = base[m, n] + 0.5 * sum(t[j] * float(B[n, j]) for j in range(r)) + float(bias[n])
    assert np.allclose(y, ref, rtol=1e-12, atol=1e-14)
    assert np.array_equal(mx.mx_lora_linear_native(x, c, s), base)
    assert np.array_equal(mx.mx_lora_linear_native(x, c, s, A, B, 0.0), base)
    assert np.array_equal(mx.mx_lora_linear_native(x, c, s, A, np.zeros_like(B), 2.0), base)
    # the adapter sees x itself, not MXFP8(x): A picks column 5, B feeds it to output 2
    A1 = np.zeros((1, K), dtype=np.float32); A1[0, 5] = 1.0
    B1 = np.zeros((N, 1), dtype=np.float32); B1[2, 0] = 1.0
    x2 = x.copy(); x2[:, 5] = np.float32(1.0 + 2.0 ** -7)          # representable in bf16, not in E4M3
    d = mx.mx_lora_linear_native(x2, c, s, A1, B1, 1.0) - mx.mx_linear_native(x2, c, s)
    assert np.array_equal(d[:, 2], x2[:, 5].astype(np.float64)) and not d[:, [0, 1, 3, 4, 5]].any()
    # dense merge, on the weight-only variant (where the base product is linear in x itself)
    What = mx.mxfp4_dequantize(c, s)
    merged = x.astype(np.float64) @ (What + 0.5 * B.astype(np.float64) @ A.astype(np.float64)).T
    assert np.allclose(mx.mx_linear_weight_only(x, c, s) + (y - base - bias[None, :]), merged, rtol=1e-12, atol=1e-13)


def _rel_rms(a, ref):
    return float(np.sqrt(np.mean((a - ref) ** 2)) / np.sqrt(np.mean(ref ** 2)))


def test_error_study_of_the_formats_on_gaussian_weights():
    """What each storage format costs on N(0, 0.02^2) weights (the synthetic stand-in for a trained matrix), as
    relative rms error of the dequantised weights: NVFP4 (E4M3 per 16 + tensor scale) < MXFP4 (a bare power of
    two per 32) < an NVFP4 tensor requantised to MXFP4 -- the only way to feed it to the block-scaled matrix
    instruction, whose scales are E8M0 per 32: an E4M3 scale is not a power of two, and the product of an E2M1
    code with an E4M3 mantissa needs five significand bits, one more than an FP8 E4M3 element holds, so no
    element format of the instruction carries NVFP4 exactly.  The ranges are the measured values +- 10 %."""
    rng = np.random.default_rng(11)
    W = (rng.standard_normal((128, 1024)) * 0.02).astype(np.float32)
    c, s, ts = o.nvfp4_quantize(W)
    Wn = o.nvfp4_dequantize(c, s, ts).astype(np.float64)
    Wm = mx.mxfp4_dequantize(*mx.mxfp4_quantize(W))
    Wr = mx.mxfp4_dequantize(*mx.mxfp4_quantize(Wn.astype(np.float32)))
    e_nv, e_mx, e_re = _rel_rms(Wn, W), _rel_rms(Wm, W), _rel_rms(Wr, W)
    assert 0.085 < e_nv < 0.105 and 0.102 < e_mx < 0.126 and 0.134 < e_re < 0.164
    assert e_nv < e_mx < e_re
    # exhaustive: some (code, scale mantissa) products are not E4M3 values
    grid8 = {float(o.e4m3_decode(np.uint8(b))) for b in range(0x7F)}
    products = {m * (8 + f) / 8 for m in (0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0) for f in range(8)}
    assert any(p not in grid8 for p in products)
    assert 1.5 * 1.125 not in grid8
    # activations in MXFP8 add a relative rms error of about 3 % of their own, nearly independent of the weights' error
    x = rng.standard_normal((8, 1024)).astype(np.float32)
    xq = mx.mxfp8_dequantize(*mx.mxfp8_quantize(x))
    assert 0.02 < _rel_rms(xq, x) < 0.04
    y = x.astype(np.float64) @ W.astype(np.float64).T
    wo, nat = _rel_rms(x.astype(np.float64) @ Wm.T, y), _rel_rms(xq @ Wm.T, y)
    assert wo < nat < wo * 1.1
