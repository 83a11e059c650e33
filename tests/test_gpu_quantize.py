"""GPU parity: nvfp4_quantize / nvfp4_dequantize are bit-exact against the oracle."""
import numpy as np
import pytest
import torch

import paper_2510_11696_amd as qerl
from oracle import nvfp4_oracle as oracle
from tests import cases
from tests.gpu_util import quantize_both, to_gpu_bf16

pytestmark = pytest.mark.gpu


def _assert_same(gpu, ref, what):
    codes, scales, ts = gpu
    rcodes, rscales, rts = ref
    assert np.float32(ts.item()) == rts, (what, ts.item(), rts)
    assert np.array_equal(scales.cpu().numpy(), rscales), what
    assert np.array_equal(codes.cpu().numpy(), rcodes), what


@pytest.mark.parametrize("N,K", [(8, 128), (3, 32), (33, 272), (1, 16)])
def test_quantize_adversarial_cases_bit_exact(N, K):
    for name, W in cases.quantizer_cases(N, K, seed=100 + N).items():
        print("case", name, N, K, flush=True)
        gpu, ref = quantize_both(W)
        _assert_same(gpu, ref, name)
        # Eq. 6 on the GPU reproduces the oracle's fp32 dequantisation bit for bit
        Wh = qerl.nvfp4_dequantize(*gpu).cpu().numpy()
        assert np.array_equal(Wh.view(np.uint32), oracle.nvfp4_dequantize(*ref).view(np.uint32)), name


@pytest.mark.parametrize("N,K", [(512, 3584), (2048, 2048), (100, 18944)])
def test_quantize_model_shapes_bit_exact(N, K):
    W = cases.gaussian(N, K, seed=N + K)
    gpu, ref = quantize_both(W)
    _assert_same(gpu, ref, (N, K))


def test_quantize_order_sensitive_scale_chain():
    from tests.test_oracle_quantize import ORDER_SENSITIVE
    for amax, bamax in ORDER_SENSITIVE:
        W = np.zeros((1, 32), dtype=np.float32)
        W[0, 5] = -amax
        W[0, 20] = bamax
        gpu, ref = quantize_both(W)
        _assert_same(gpu, ref, (amax, bamax))


def test_quantize_strided_rows_and_empty():
    W = cases.gaussian(16, 256, seed=5)
    big = torch.zeros((16, 512), dtype=torch.bfloat16, device="cuda")
    big[:, :256] = to_gpu_bf16(W)
    big[:, 256:] = 99.0                      # must not be read as part of the tensor
    codes, scales, ts = qerl.nvfp4_quantize(big[:, :256])
    _assert_same((codes, scales, ts), oracle.nvfp4_quantize(W), "strided")
    codes, scales, ts = qerl.nvfp4_quantize(torch.empty((0, 64), dtype=torch.bfloat16, device="cuda"))
    assert ts.item() == 1.0 and codes.numel() == 0


def test_quantize_is_deterministic():
    W = to_gpu_bf16(cases.gaussian(256, 1024, seed=77))
    a = qerl.nvfp4_quantize(W)
    for _ in range(5):
        b = qerl.nvfp4_quantize(W)
        assert all(torch.equal(p, q) for p, q in zip(a, b))
