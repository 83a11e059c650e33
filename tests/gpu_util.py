"""Helpers for the GPU parity tests: move seeded inputs to the device, call the
C ABI through the binding, and compare with the oracle under the two gates."""
import numpy as np
import torch

import paper_2510_11696_amd as qerl
from oracle import nvfp4_oracle as oracle


def to_gpu_bf16(a_f32: np.ndarray) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(a_f32)).to(torch.bfloat16)
    assert np.array_equal(t.float().numpy(), a_f32), "input must be bf16-exact"
    return t.cuda()


def check_linear(y_gpu: torch.Tensor, y_ref: np.ndarray, what="", slack=1e-3):
    """Official gate: per row max|err| <= 2e-2 * max|y_ref row|.
    Tight gate (bf16 output rounding + fp32 summation order):
        |err| <= 2^-8 |y_ref| + slack * max|y_ref row|,  slack = 1e-3 for one linear on exact inputs.
    For a composition of operators (norm -> linear -> SiLU-mul -> linear) the device rounds each intermediate
    from an fp32 sum where the oracle rounds an fp64 one, so a few per cent of the intermediate activations are
    one bf16 unit (<= 2^-8 relative) apart; over a sum of K terms that adds about sqrt(0.02) * 2^-8 / 4 ~ 1.4e-4 of
    the row maximum in rms, 6e-4 at the 4.5 sigma of ~1e5 outputs; and a single one-unit difference on an outlier
    activation (|x| ~ 4) against an outlier weight is by itself up to ~1e-3 of the row maximum of the next operator at
    small K.  The feed-forward block chains two operators: its tests pass slack = 4e-3."""
    y = y_gpu.float().cpu().numpy().astype(np.float64)
    assert y.shape == y_ref.shape, (y.shape, y_ref.shape)
    assert np.all(np.isfinite(y)), what
    err = np.abs(y - y_ref)
    row_inf = np.abs(y_ref).max(axis=1, keepdims=True) if y_ref.size else np.zeros((y_ref.shape[0], 1))
    assert np.all(err.max(axis=1, keepdims=True) <= 2e-2 * row_inf + 1e-30), (
        what, float((err.max(axis=1, keepdims=True) / (row_inf + 1e-30)).max()))
    tight = 2.0 ** -8 * np.abs(y_ref) + slack * row_inf + 1e-30
    bad = err > tight
    assert not bad.any(), (what, int(bad.sum()), float((err / tight).max()))


def bf16_ulp_distance(y_gpu: torch.Tensor, y_ref64: np.ndarray) -> np.ndarray:
    """Distance in bf16 units between the GPU result and the correctly rounded oracle value."""
    ref = torch.from_numpy(y_ref64).to(torch.float32).to(torch.bfloat16)
    a = y_gpu.cpu().view(torch.int16).to(torch.int32).numpy()
    b = ref.view(torch.int16).to(torch.int32).numpy()
    # map sign-magnitude bit patterns to a monotone integer line
    a = np.where(a < 0, -(a & 0x7FFF), a)
    b = np.where(b < 0, -(b & 0x7FFF), b)
    return np.abs(a - b)


def quantize_both(W_f32: np.ndarray):
    """Quantise on the GPU and with the oracle; return both triples."""
    Wg = to_gpu_bf16(W_f32)
    codes, scales, ts = qerl.nvfp4_quantize(Wg)
    torch.cuda.synchronize()
    ref = oracle.nvfp4_quantize(W_f32)
    return (codes, scales, ts), ref
