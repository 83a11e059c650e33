"""Seeded generators for synthetic tensors.

The paper trains Qwen2.5 checkpoints on GSM8K / BigMath rollouts; neither is
available here, so Gaussian tensors of the same shapes stand in for them.
In every "N(0, s)" below s is the standard deviation.  All draws come from a
CPU `torch.Generator` so the same seed gives the same bytes on every
machine; the benchmark may instead draw on the device for tensors too large
to ship (it says so where it does).
"""
from __future__ import annotations

import torch

BASE_SEED = 20251011


def seed_for(config: int, tensor_index: int) -> int:
    """seed = BASE_SEED + 1000 * config number (1-based) + tensor index."""
    return BASE_SEED + 1000 * int(config) + int(tensor_index)


def _gen(seed: int) -> torch.Generator:
    g = torch.Generator(device="cpu")
    g.manual_seed(int(seed))
    return g


def normal_f32(shape, std: float, seed: int, mean: float = 0.0) -> torch.Tensor:
    return torch.randn(*shape, generator=_gen(seed), dtype=torch.float32) * std + mean


def normal_bf16(shape, std: float, seed: int, mean: float = 0.0) -> torch.Tensor:
    """fp32 draw, scaled, rounded to bf16 (round-to-nearest-even)."""
    return normal_f32(shape, std, seed, mean).to(torch.bfloat16)


def weights(N: int, K: int, seed: int, std: float = 0.02) -> torch.Tensor:
    """Pre-quantisation weight W[N, K] ~ N(0, 0.02), bf16."""
    return normal_bf16((N, K), std, seed)


def activations(M: int, K: int, seed: int, std: float = 1.0) -> torch.Tensor:
    """x[M, K] ~ N(0, 1), bf16."""
    return normal_bf16((M, K), std, seed)


def lora_pair(N: int, K: int, r: int, seed: int, b_std: float = 0.01):
    """A[r, K] ~ N(0, 1/r), B[N, r] ~ N(0, 0.01), both bf16."""
    A = normal_bf16((r, K), 1.0 / r, seed)
    B = normal_bf16((N, r), b_std, seed + 500)
    return A, B


def rms_gain(H: int, seed: int, std: float = 0.05) -> torch.Tensor:
    """RMSNorm gain ~ 1 + N(0, 0.05), bf16."""
    return normal_bf16((H,), std, seed, mean=1.0)


def aqn_noise(H: int, sigma: float, seed: int) -> torch.Tensor:
    """Noise vector Z ~ N(0, sigma^2 I), fp32; sigma is supplied by the caller."""
    return normal_f32((H,), float(sigma), seed)
