"""Adversarial weight tensors for the quantiser (shared by the oracle pins
and the GPU parity tests).  All return float32 numpy arrays of bf16 values."""
import numpy as np
import torch

import qerl_synth as qs

E2M1_VALUES = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]   # tests/golden/e2m1_magnitudes.txt


def to_bf16_f32(a):
    """Round a float array to bf16 (RNE) and return it as float32 numpy."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16).float().numpy()


def gaussian(N, K, seed, std=0.02):
    return qs.weights(N, K, seed, std).float().numpy()


def outlier(N, K, seed):
    """One huge element forces tiny / zero block scales elsewhere."""
    W = gaussian(N, K, seed)
    W[N // 2, K // 3] = 3.0e4
    return to_bf16_f32(W)


def zero_rows_and_blocks(N, K, seed):
    W = gaussian(N, K, seed)
    W[0, :] = 0.0
    if N > 1:
        W[N - 1, :] = -0.0
    if N > 2:
        W[1, 16:48] = 0.0
        W[2, 0:16] = -0.0
    return W


def all_zero(N, K):
    W = np.zeros((N, K), dtype=np.float32)
    W[0, 1] = -0.0
    return W


def representable(N, K, seed, p=-9):
    """W = 2^p * s * e with e an E2M1 value and s an E4M3 value per block;
    the tensor maximum is 2688 * 2^p so the tensor scale is exactly 2^p and
    each block's maximum is 6 * s * 2^p.  quantize -> dequantize must return W
    exactly and the scale bytes must encode s."""
    rng = np.random.default_rng(seed)
    nb = K // 16
    sbytes = rng.integers(0x08, 0x7F, size=(N, nb)).astype(np.uint8)  # normal E4M3, <= 448
    sbytes[0, 0] = 0x7E                                                # 448 -> holds amax
    e = (sbytes >> 3).astype(np.int64)
    m = (sbytes & 7).astype(np.float64)
    s = (1.0 + m / 8.0) * np.exp2(e - 7.0)
    idx = rng.integers(0, 8, size=(N, K))
    sign = rng.integers(0, 2, size=(N, K)) * 2.0 - 1.0
    mags = np.array(E2M1_VALUES)[idx]
    mags = mags.reshape(N, nb, 16)
    mags[:, :, 0] = 6.0                       # every block reaches 6 * s
    mags = mags.reshape(N, K)
    W = (2.0 ** p) * np.repeat(s, 16, axis=1) * mags * sign
    W32 = W.astype(np.float32)
    assert np.array_equal(to_bf16_f32(W32), W32), "construction must be bf16-exact"
    return W32, sbytes, np.float32(2.0 ** p)


def ties(N, K, p=-9):
    """Elements sitting exactly on the E2M1 rounding ties (0.25, 0.75, 1.25,
    1.75, 2.5, 3.5, 5) of a block whose scale is exactly 1 * 2^p."""
    tie_q = np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, 6.0,
                      -0.25, -0.75, -1.25, -1.75, -2.5, -3.5, -5.0, 0.125])
    W = np.tile(tie_q, (N, K // 16)) * (2.0 ** p)
    W[0, 0] = 2688.0 * 2.0 ** p      # tensor scale = 2^p; this block's scale is 448
    W = W.astype(np.float32)
    assert np.array_equal(to_bf16_f32(W), W)
    return W


def tiny_scale(N, K, seed):
    """Wide dynamic range: blocks whose scale is subnormal E4M3 or rounds to 0."""
    W = gaussian(N, K, seed, std=1.0)
    expo = np.linspace(0, -14, K // 16)
    W = W * np.repeat(np.exp2(expo), 16)[None, :]
    return to_bf16_f32(W)


def quantizer_cases(N=8, K=128, seed=7):
    rep, _, _ = representable(N, K, seed)
    return {
        "gaussian": gaussian(N, K, seed),
        "outlier": outlier(N, K, seed + 1),
        "zero_rows_blocks": zero_rows_and_blocks(N, K, seed + 2),
        "all_zero": all_zero(N, K),
        "representable": rep,
        "ties": ties(N, K),
        "tiny_scale": tiny_scale(N, K, seed + 3),
        "scaled_up": to_bf16_f32(gaussian(N, K, seed + 4) * 2.0 ** 40),
        "scaled_down": to_bf16_f32(gaussian(N, K, seed + 5) * 2.0 ** -40),
    }
