"""GPU parity: aqn_rmsnorm against the fp64 oracle, within 1 bf16 unit."""
import numpy as np
import pytest
import torch

import paper_2510_11696_amd as qerl
import qerl_synth as qs
from oracle import nvfp4_oracle as oracle
from tests.gpu_util import bf16_ulp_distance

pytestmark = pytest.mark.gpu


def _run(M, H, sigma, seed, scale=1.0):
    x = (qs.activations(M, H, seed).float() * scale).to(torch.bfloat16)
    g = qs.rms_gain(H, seed + 1)
    Z = qs.aqn_noise(H, sigma, seed + 2) if sigma is not None else None
    y = qerl.aqn_rmsnorm(x.cuda(), g.cuda(), Z.cuda() if Z is not None else None, eps=1e-6)
    torch.cuda.synchronize()
    ref = oracle.aqn_rmsnorm(x.float().numpy(), g.float().numpy(), Z.numpy() if Z is not None else None, 1e-6)
    d = bf16_ulp_distance(y, ref)
    assert d.max() <= 1, (M, H, sigma, int(d.max()))
    assert (d > 0).mean() < 0.01          # almost every element is the correctly rounded value
    return y


@pytest.mark.parametrize("M,H", [(1, 3584), (8, 3584), (128, 5120), (3, 2048), (5, 8192), (2, 16384), (4, 72)])
def test_rmsnorm_vector_path(M, H):
    for sigma in (None, 1e-2, 5e-4):
        _run(M, H, sigma, seed=M * 1000 + H)


@pytest.mark.parametrize("M,H", [(3, 100), (2, 3583), (1, 7)])
def test_rmsnorm_general_path(M, H):
    _run(M, H, 1e-2, seed=9)
    _run(M, H, None, seed=10)


def test_rmsnorm_stage0_equals_zero_noise_and_scales():
    M, H = 4, 3584
    x = qs.activations(M, H, 1).cuda()
    g = qs.rms_gain(H, 2).cuda()
    y0 = qerl.aqn_rmsnorm(x, g, None)
    yz = qerl.aqn_rmsnorm(x, g, torch.zeros(H, device="cuda"))
    assert torch.equal(y0, yz)
    _run(4, 3584, 1e-2, seed=3, scale=1e-3)     # small activations: eps matters
    _run(4, 3584, 1e-2, seed=4, scale=300.0)
    z = qerl.aqn_rmsnorm(torch.zeros((2, H), dtype=torch.bfloat16, device="cuda"), g, None)
    assert not z.any()


def test_rmsnorm_strided_io_and_schedule():
    M, H = 6, 512
    xb = torch.zeros((M, 1024), dtype=torch.bfloat16, device="cuda")
    x = qs.activations(M, H, 5)
    xb[:, :H] = x.cuda()
    out = torch.full((M, 768), 7.0, dtype=torch.bfloat16, device="cuda")
    g = qs.rms_gain(H, 6)
    for k in range(0, 11):
        sigma = qerl.aqn_sigma(k, 10, 1e-2, 5e-4)
        assert abs(sigma - oracle.aqn_sigma(k, 10, 1e-2, 5e-4)) <= 1e-18
        Z = qs.aqn_noise(H, sigma, 20 + k) if k else None
        qerl.aqn_rmsnorm(xb[:, :H], g.cuda(), Z.cuda() if k else None, out=out[:, :H])
        ref = oracle.aqn_rmsnorm(x.float().numpy(), g.float().numpy(), Z.numpy() if k else None)
        assert bf16_ulp_distance(out[:, :H].contiguous(), ref).max() <= 1
        assert torch.all(out[:, H:] == 7.0)
