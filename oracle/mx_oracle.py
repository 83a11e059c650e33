"""CPU oracle for the MXFP4 variant of the weight-only linear layer.

THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE (same rules as nvfp4_oracle: only the
test-suite, the smoke check and the benchmark's cpu_baseline leg may import it; it shares
nothing with the HIP library).

What it follows
---------------
* MXFP4 tensor: FP4 (E2M1) elements with one shared FP8 (E8M0, a bare power of two) scale per
  block of 32 elements: Preliminary, "Model Quantization" (the paper evaluates MXFP4 next to
  NVFP4 in its GSM8K table and reward curves).  Dequantisation is Eq. (1)'s  w_hat = scale * code.
* The paper does not state the quantisation rule.  Reading taken here -- the OCP Microscaling
  Formats (MX) v1.0 conversion: per block, shared exponent
        X = floor(log2(max |v|)) - emax_elem          (emax_elem = 2 for E2M1, 8 for E4M3)
  clamped to [-127, 127]; scale byte = X + 127; element = round-to-nearest-even of v / 2^X onto
  the element grid, saturating at its largest magnitude (6, 448).  An all-zero block gets the
  smallest scale (byte 0) and zero elements.  Byte 255 (NaN) is never produced.
* "Native" path: the same linear with the ACTIVATIONS quantised to MXFP8 (E4M3 elements, E8M0
  scale per 32 along K) so that both operands fit the scaled matrix instruction of the target:
        y[m,n] = sum_b 2^(Xx[m,b] + Xw[n,b]) * sum_{k in b} xq[m,k] * wq[n,k]
  This is NOT what the paper runs (its kernels keep activations in bf16); the oracle defines it
  so that the kernel can be checked exactly, and mx_linear_weight_only gives the paper's
  weight-only result to measure the difference against.

Blocks run along K (the input dimension), W is [N, K], x is [M, K]; bf16 inputs are float32
arrays with bf16-representable values.  Every function is pinned in tests/test_oracle_mx.py.
"""
from __future__ import annotations

import numpy as np

from .nvfp4_oracle import E2M1_GRID, E4M3_GRID, e2m1_decode, round_to_grid_rne

MX_BLOCK = 32


def e8m0_decode(byte):
    """E8M0 byte -> 2^(byte - 127) as float64 (byte 255 is NaN in the format and not accepted)."""
    byte = np.asarray(byte, dtype=np.uint8)
    if np.any(byte == 255):
        raise ValueError("E8M0 byte 255 is NaN")
    return np.ldexp(1.0, byte.astype(np.int32) - 127)


def _shared_exponent(amax, emax_elem):
    """floor(log2(amax)) - emax_elem, clamped to [-127, 127]; amax == 0 -> -127.  amax >= 0 finite."""
    amax = np.asarray(amax, dtype=np.float64)
    _, e = np.frexp(amax)                      # amax = m * 2^e with 0.5 <= m < 1  ->  floor(log2) = e - 1
    x = np.where(amax > 0, e.astype(np.int64) - 1 - emax_elem, -127)
    return np.clip(x, -127, 127)


def _mx_quantize(V, grid, emax_elem):
    V = np.asarray(V, dtype=np.float32).astype(np.float64)
    if V.ndim != 2 or V.shape[1] % MX_BLOCK != 0:
        raise ValueError("need [rows, K] with K a multiple of 32")
    if np.any(~np.isfinite(V)):
        raise ValueError("finite inputs only")
    R, K = V.shape
    blocks = V.reshape(R, K // MX_BLOCK, MX_BLOCK)
    X = _shared_exponent(np.abs(blocks).max(axis=2), emax_elem)            # [R, K/32]
    scaled = np.abs(blocks) * np.ldexp(1.0, -X)[:, :, None]                # exact: power-of-two scaling in float64
    idx = round_to_grid_rne(scaled.reshape(-1), grid).reshape(blocks.shape)
    sign = np.signbit(blocks)
    return idx.astype(np.uint8), sign, (X + 127).astype(np.uint8)


def mxfp4_quantize(W):
    """W[N,K] -> (codes[N,K/2] u8: low nibble = even k, bit 3 of a nibble = sign; scales[N,K/32] u8 E8M0)."""
    idx, sign, sbytes = _mx_quantize(W, E2M1_GRID, 2)
    nib = (idx | (sign.astype(np.uint8) << 3)).reshape(idx.shape[0], -1)
    codes = (nib[:, 0::2] | (nib[:, 1::2] << 4)).astype(np.uint8)
    return codes, sbytes


def mxfp4_dequantize(codes, scales):
    """-> W_hat[N,K] float64 = 2^(scale - 127) * E2M1(code), exact."""
    codes = np.asarray(codes, dtype=np.uint8)
    N, K = codes.shape[0], codes.shape[1] * 2
    nib = np.empty((N, K), dtype=np.uint8)
    nib[:, 0::2] = codes & 0xF
    nib[:, 1::2] = codes >> 4
    vals = e2m1_decode(nib).astype(np.float64).reshape(N, K // MX_BLOCK, MX_BLOCK)
    return (vals * e8m0_decode(scales)[:, :, None]).reshape(N, K)


def mxfp8_quantize(x):
    """x[M,K] -> (codes[M,K] u8 E4M3 with sign in bit 7; scales[M,K/32] u8 E8M0)."""
    idx, sign, sbytes = _mx_quantize(x, E4M3_GRID, 8)
    return (idx | (sign.astype(np.uint8) << 7)).reshape(idx.shape[0], -1), sbytes


def mxfp8_dequantize(codes, scales):
    codes = np.asarray(codes, dtype=np.uint8)
    M, K = codes.shape
    mag = E4M3_GRID[codes & 0x7F]
    vals = np.where(codes >> 7, -mag, mag).reshape(M, K // MX_BLOCK, MX_BLOCK)
    return (vals * e8m0_decode(scales)[:, :, None]).reshape(M, K)


def mx_linear_weight_only(x, wcodes, wscales):
    """The paper's setting: bf16 activations times dequantised MXFP4 weights, float64."""
    return np.asarray(x, dtype=np.float32).astype(np.float64) @ mxfp4_dequantize(wcodes, wscales).T


def mx_linear_native(x, wcodes, wscales):
    """Activations quantised to MXFP8 first, then the exact product of the two quantised operands."""
    xc, xs = mxfp8_quantize(x)
    return mxfp8_dequantize(xc, xs) @ mxfp4_dequantize(wcodes, wscales).T


def mx_lora_linear_native(x, wcodes, wscales, A=None, B=None, lora_scale=0.0, bias=None):
    """The native MXFP4 linear with the LoRA branch of Eq. (2) and an optional bias:
        y = MXFP8(x) . MXFP4(W)^T + lora_scale * (x A^T) B^T + bias
    The adapter reads the bf16 activations as they are (LoRA stays in bf16 in the paper: only the frozen base
    weights are quantised), only the base product goes through the quantised activations.  float64."""
    y = mx_linear_native(x, wcodes, wscales)
    if A is not None:
        x64 = np.asarray(x, dtype=np.float32).astype(np.float64)
        t = x64 @ np.asarray(A, dtype=np.float32).astype(np.float64).T
        y = y + float(lora_scale) * (t @ np.asarray(B, dtype=np.float32).astype(np.float64).T)
    if bias is not None:
        y = y + np.asarray(bias, dtype=np.float32).astype(np.float64)[None, :]
    return y
