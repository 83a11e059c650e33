"""On-device noise vector against the oracle's counter-based construction (GPU)."""
import math

import numpy as np
import pytest
import torch

import paper_2510_11696_amd as qerl
import qerl_synth as qs
from oracle import nvfp4_oracle as oracle
from tests.gpu_util import bf16_ulp_distance

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n", [1, 3, 4, 5, 3584, 2 * 28 * 3584 + 1])
@pytest.mark.parametrize("sigma,seed,sub", [(1e-2, 20251011, 0), (5e-4, 0xFEDCBA9876543210, 0x1_0000_0003), (1.0, 0, 7)])
def test_noise_fill_matches_the_oracle(n, sigma, seed, sub):
    """The integer part (generator, 24-bit uniforms) is identical by construction; the fp32 log, root,
    sine and cosine differ from the oracle's fp64 ones by a few units in the last place of z, whose
    magnitude is at most sqrt(48 ln 2) ~ 5.77: |z_gpu - z_ref| <= 4e-6 (about 6 ulp at the largest radius)."""
    print("noise case", n, sigma, seed, sub, flush=True)
    z = qerl.aqn_noise_fill(n, sigma, seed, sub)
    torch.cuda.synchronize()
    ref = oracle.aqn_noise_philox(n, sigma, seed, sub)
    got = z.cpu().numpy().astype(np.float64)
    assert got.shape == ref.shape
    assert np.all(np.abs(got - ref) <= 4e-6 * sigma), float(np.abs(got - ref).max() / sigma)
    # same call, same values; an unaligned destination takes the scalar stores and gives the same values
    again = qerl.aqn_noise_fill(n, sigma, seed, sub)
    assert torch.equal(z, again)
    buf = torch.full((n + 3,), 7.0, dtype=torch.float32, device="cuda")
    qerl.aqn_noise_fill(n, sigma, seed, sub, out=buf[1:])
    assert torch.equal(buf[1:n + 1], z) and buf[0].item() == 7.0 and buf[n + 1].item() == 7.0


def test_noise_fill_edge_cases():
    assert qerl.aqn_noise_fill(0, 1e-2, 1, 1).numel() == 0
    z = qerl.aqn_noise_fill(64, 0.0, 1, 1)
    assert torch.count_nonzero(z).item() == 0                      # sigma = 0: stage 0
    with pytest.raises(qerl.QerlError):
        qerl.aqn_noise_fill(8, -1.0, 1, 1)
    with pytest.raises(qerl.QerlError):
        qerl.aqn_noise_fill(8, float("nan"), 1, 1)


def test_generated_noise_through_the_rmsnorm():
    """Noise generated on the device feeds aqn_rmsnorm: within one bf16 unit of the oracle fed with the
    oracle's own noise vector (the 4e-6 sigma difference in Z is far below the rounding step)."""
    M, H, sigma = 8, 3584, oracle.aqn_sigma(1, 10, 1e-2, 5e-4)
    x = qs.activations(M, H, 5001)
    gain = qs.rms_gain(H, 5002)
    z = qerl.aqn_noise_fill(H, sigma, 99, 3)
    y = qerl.aqn_rmsnorm(x.cuda(), gain.cuda(), z, 1e-6)
    torch.cuda.synchronize()
    ref = oracle.aqn_rmsnorm(x.float().numpy(), gain.float().numpy(),
                             oracle.aqn_noise_philox(H, sigma, 99, 3).astype(np.float32), 1e-6)
    d = bf16_ulp_distance(y, ref)
    assert d.max() <= 1 and (d > 0).mean() < 0.01
