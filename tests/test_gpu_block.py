"""GPU parity of the fused decode launches against the oracle's composition of the same operators:
    aqn_rmsnorm -> (round to bf16) -> nvfp4_lora_linear for every member                      (norm + group)
    aqn_rmsnorm -> gate, up -> (round to bf16) -> silu_mul -> nvfp4_lora_linear(down)         (feed-forward block)
The device rounds the intermediate activations from fp32 sums, the oracle from fp64 ones, so a few of them differ by
one bf16 unit.  One such unit on an outlier activation (|x| ~ 4 after the norm) against an outlier weight moves an
output of the NEXT operator by 2^-8 |x w|, up to ~1e-3 of the row maximum per operator at these sizes, and the feed-forward
block chains two: the tight gate is therefore taken with 4e-3 of the row maximum (slack) for the feed-forward block; the
official gate (2e-2 of the row maximum) is unchanged."""
import numpy as np
import pytest
import torch

import paper_2510_11696_amd as qerl
import qerl_synth as qs
from oracle import nvfp4_oracle as oracle
from tests import cases
from tests.gpu_util import check_linear

pytestmark = pytest.mark.gpu


def _bf16(a64):
    """fp64 -> bf16 values (nearest even) held in float32, as the next operator of a bf16 model sees them."""
    return oracle.round_to_bf16(a64).astype(np.float32)


def _member(N, K, r, seed, bias=False):
    W = cases.gaussian(N, K, seed)
    codes, scales, ts = oracle.nvfp4_quantize(W)
    g = lambda a: torch.from_numpy(a).cuda()
    pw = qerl.nvfp4_prepack(g(codes), g(scales), torch.tensor([ts], device="cuda"))
    A = B = None
    if r:
        A, B = qs.lora_pair(N, K, r, seed + 1)
    b = None
    if bias:
        b = (torch.randn(N, generator=torch.Generator().manual_seed(seed + 2)) * 0.5).to(torch.bfloat16)
    return dict(codes=codes, scales=scales, ts=ts, pw=pw, A=A, B=B, bias=b, r=r, N=N,
                Ad=A.cuda() if r else None, Bd=B.cuda() if r else None, bd=b.cuda() if bias else None)


def _ref(m, x_f32, lora_scale):
    return oracle.nvfp4_lora_linear(x_f32, m["codes"], m["scales"], m["ts"],
                                    m["A"].float().numpy() if m["r"] else None,
                                    m["B"].float().numpy() if m["r"] else None, lora_scale,
                                    bias=m["bias"].float().numpy() if m["bias"] is not None else None)


def _norm_inputs(M, H, seed, sigma):
    xin = qs.activations(M, H, seed)
    gain = qs.rms_gain(H, seed + 1)
    Z = qs.aqn_noise(H, sigma, seed + 2) if sigma is not None else None
    xn = _bf16(oracle.aqn_rmsnorm(xin.float().numpy(), gain.float().numpy(), Z.numpy() if Z is not None else None, 1e-6))
    return xin, gain, Z, xn


@pytest.mark.parametrize("M", [1, 3, 8, 9, 16])
@pytest.mark.parametrize("H,Ns,rs,sigma,bias", [
    (3584, (3584, 512, 512), (32, 32, 32), 1e-2, True),     # q, k, v of the 7B block, with their biases
    (5120, (160, 64, 64), (64, 64, 64), 5e-4, False),       # three rank-64 adapters; rows longer than one K-range at 16 tokens
    (2048, (96, 40), (64, 16), None, False),                # stage 0 (no noise); ragged row tile; partial rank tile
    (4096, (64,), (8,), 1e-2, False),                       # a single small member: many K-ranges
    (3584, (1184, 1184), (32, 0), 1e-2, False),             # a member without adapter
    (1040, (72,), (0,), 5e-3, False),                       # K not a multiple of 128, no adapter at all: no producers
])
def test_norm_and_group_in_one_launch(M, H, Ns, rs, sigma, bias):
    print("norm+group case", M, H, Ns, rs, sigma, bias, flush=True)
    xin, gain, Z, xn = _norm_inputs(M, H, 400 + M, sigma)
    mem = [_member(N, H, r, 5000 + 10 * i + M, bias) for i, (N, r) in enumerate(zip(Ns, rs))]
    ws = qerl.Workspace(qerl.aqn_rmsnorm_nvfp4_lora_linear_group_workspace_bytes(M, H, list(Ns), list(rs)))
    call = lambda: qerl.aqn_rmsnorm_nvfp4_lora_linear_group(
        xin.cuda(), gain.cuda(), Z.cuda() if Z is not None else None, 1e-6, [m["pw"] for m in mem],
        [m["Ad"] for m in mem], [m["Bd"] for m in mem], [2.0] * len(mem), workspace=ws, biases=[m["bd"] for m in mem])
    outs = [o.clone() for o in call()]
    again = call()
    torch.cuda.synchronize()
    assert qerl.workspace_status(ws) == 0
    for i, (m, y) in enumerate(zip(mem, outs)):
        check_linear(y, _ref(m, xn, 2.0), ("norm+group", i, M, H, Ns, rs))
    assert all(torch.equal(p, q) for p, q in zip(outs, again)), "second run on the same workspace differs"


@pytest.mark.parametrize("M", [2, 16])
def test_group_without_norm_in_the_block_kernel(M):
    """gain = NULL: the stage input is used as it is (what o_proj and a stand-alone down_proj would be)."""
    K, Ns, rs = 18944, (96, 40), (32, 32)
    x = qs.activations(M, K, 700 + M)
    mem = [_member(N, K, r, 5200 + 10 * i + M) for i, (N, r) in enumerate(zip(Ns, rs))]
    outs = qerl.aqn_rmsnorm_nvfp4_lora_linear_group(x.cuda(), None, None, 0.0, [m["pw"] for m in mem],
                                                    [m["Ad"] for m in mem], [m["Bd"] for m in mem], [2.0] * len(mem))
    torch.cuda.synchronize()
    for i, (m, y) in enumerate(zip(mem, outs)):
        check_linear(y, _ref(m, x.float().numpy(), 2.0), ("group, no norm", i, M))


@pytest.mark.parametrize("M", [1, 5, 8, 13, 16])
@pytest.mark.parametrize("H,I,rs,sigma", [
    (512, 1024, (16, 16, 16), 1e-2),
    (3584, 2368, (32, 32, 32), 1e-2),        # 7B hidden size, 74 gate / up tile pairs; down's K = 2368 is not a multiple of 128
    (5120, 1728, (64, 64, 64), 5e-4),        # 32B hidden size and rank
    (2048, 4096, (0, 0, 0), None),           # no adapters, no noise
    (1024, 640, (8, 0, 64), 1e-2),           # mixed ranks
])
def test_feed_forward_block_in_one_launch(M, H, I, rs, sigma):
    print("mlp case", M, H, I, rs, sigma, flush=True)
    xin, gain, Z, xn = _norm_inputs(M, H, 800 + M, sigma)
    gate = _member(I, H, rs[0], 6000 + M)
    up = _member(I, H, rs[1], 6100 + M)
    down = _member(H, I, rs[2], 6200 + M)
    g_ref, u_ref = _bf16(_ref(gate, xn, 2.0)), _bf16(_ref(up, xn, 2.0))
    act = oracle.silu_mul(g_ref, u_ref).astype(np.float32)
    ref = _ref(down, act, 2.0)
    lib = qerl.load_library()
    ws = qerl.Workspace(lib.aqn_rmsnorm_nvfp4_lora_mlp_workspace_bytes(M, H, I, H, rs[0], rs[1], rs[2]))
    call = lambda: qerl.aqn_rmsnorm_nvfp4_lora_mlp(
        xin.cuda(), gain.cuda(), Z.cuda() if Z is not None else None, 1e-6, gate["pw"], up["pw"], down["pw"],
        (gate["Ad"], up["Ad"], down["Ad"]), (gate["Bd"], up["Bd"], down["Bd"]), (2.0, 2.0, 2.0), workspace=ws)
    y = call().clone()
    again = call()
    torch.cuda.synchronize()
    assert qerl.workspace_status(ws) == 0
    check_linear(y, ref, ("mlp", M, H, I, rs), slack=4e-3)
    assert torch.equal(y, again), "second run on the same workspace differs"
    # the same operators as separate launches agree with it to rounding
    xn_d = qerl.aqn_rmsnorm(xin.cuda(), gain.cuda(), Z.cuda() if Z is not None else None, 1e-6)
    gu = qerl.nvfp4_lora_linear_packed_group(xn_d, [gate["pw"], up["pw"]], [gate["Ad"], up["Ad"]], [gate["Bd"], up["Bd"]], [2.0, 2.0])
    sep = qerl.nvfp4_lora_linear_packed_swiglu(gu[0], gu[1], down["pw"], down["Ad"], down["Bd"], 2.0)
    check_linear(sep, ref, ("mlp as separate launches", M, H, I, rs), slack=4e-3)


@pytest.mark.parametrize("M", [17, 40])
def test_fused_entry_points_beyond_16_tokens_run_the_separate_launches(M):
    H, I, r = 1024, 768, 16
    xin, gain, Z, xn = _norm_inputs(M, H, 900 + M, 1e-2)
    gate, up, down = _member(I, H, r, 6300 + M), _member(I, H, r, 6310 + M), _member(H, I, r, 6320 + M)
    act = oracle.silu_mul(_bf16(_ref(gate, xn, 2.0)), _bf16(_ref(up, xn, 2.0))).astype(np.float32)
    y = qerl.aqn_rmsnorm_nvfp4_lora_mlp(xin.cuda(), gain.cuda(), Z.cuda(), 1e-6, gate["pw"], up["pw"], down["pw"],
                                        (gate["Ad"], up["Ad"], down["Ad"]), (gate["Bd"], up["Bd"], down["Bd"]), (2.0, 2.0, 2.0))
    outs = qerl.aqn_rmsnorm_nvfp4_lora_linear_group(xin.cuda(), gain.cuda(), Z.cuda(), 1e-6, [gate["pw"], up["pw"]],
                                                    [gate["Ad"], up["Ad"]], [gate["Bd"], up["Bd"]], [2.0, 2.0])
    torch.cuda.synchronize()
    check_linear(y, _ref(down, act, 2.0), ("mlp, separate launches", M), slack=4e-3)
    check_linear(outs[0], _ref(gate, xn, 2.0), ("group, separate launches", M))
    check_linear(outs[1], _ref(up, xn, 2.0), ("group, separate launches", M))


def test_a_wait_that_gives_up_is_reported_until_the_workspace_is_initialised_again():
    """The error path end to end, forced from the host: one wave runs the kernels' bounded wait (cut to a few polls) on
    a hand-over word that nobody raises, gives up, sets the sticky word and exits normally."""
    lib = qerl.load_library()
    M, H = 4, 512
    ws = qerl.Workspace(qerl.aqn_rmsnorm_nvfp4_lora_linear_group_workspace_bytes(M, H, [64], [16]))
    st = torch.cuda.current_stream().cuda_stream
    assert qerl.workspace_status(ws) == 0
    assert lib.qerl_selftest_wait_gives_up(ws.ptr, ws.nbytes, 8, st) == 0
    assert qerl.workspace_status(ws) == -6
    assert qerl.workspace_status(ws) == -6                      # sticky
    assert lib.qerl_workspace_init(ws.ptr, ws.nbytes, st) == 0
    assert qerl.workspace_status(ws) == 0
    # and the workspace serves a call again
    xin, gain, Z, xn = _norm_inputs(M, H, 990, 1e-2)
    m = _member(64, H, 16, 6400)
    y = qerl.aqn_rmsnorm_nvfp4_lora_linear_group(xin.cuda(), gain.cuda(), Z.cuda(), 1e-6, [m["pw"]], [m["Ad"]], [m["Bd"]], [2.0],
                                                 workspace=ws)[0]
    torch.cuda.synchronize()
    assert qerl.workspace_status(ws) == 0
    check_linear(y, _ref(m, xn, 2.0), ("after re-initialisation",))


@pytest.mark.timeout(600)
@pytest.mark.parametrize("rs", [(0, 0, 0), (16, 16, 16)])
def test_feed_forward_block_whose_stages_need_different_lds_areas(rs):
    """Hidden size 8192 at 16 tokens: the gate / up stage cannot hold its input in one piece (K-split pairs or phases with
    parked accumulators), while down's K = 3584 wants a large x slice: the stages' LDS areas are planned as a union."""
    M, H, I = 16, 8192, 3584
    print("mlp case with a wide hidden size", M, H, I, rs, flush=True)
    xin, gain, Z, xn = _norm_inputs(M, H, 850, 5e-3)
    gate, up, down = _member(I, H, rs[0], 6500), _member(I, H, rs[1], 6510), _member(H, I, rs[2], 6520)
    act = oracle.silu_mul(_bf16(_ref(gate, xn, 2.0)), _bf16(_ref(up, xn, 2.0))).astype(np.float32)
    lib = qerl.load_library()
    ws = qerl.Workspace(lib.aqn_rmsnorm_nvfp4_lora_mlp_workspace_bytes(M, H, I, H, *rs))
    call = lambda: qerl.aqn_rmsnorm_nvfp4_lora_mlp(
        xin.cuda(), gain.cuda(), Z.cuda(), 1e-6, gate["pw"], up["pw"], down["pw"], (gate["Ad"], up["Ad"], down["Ad"]),
        (gate["Bd"], up["Bd"], down["Bd"]), (2.0, 2.0, 2.0), workspace=ws)
    y = call().clone()
    again = call()
    torch.cuda.synchronize()
    assert qerl.workspace_status(ws) == 0
    check_linear(y, _ref(down, act, 2.0), ("mlp, wide hidden", M, H, I, rs), slack=4e-3)
    assert torch.equal(y, again)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("seed", [11, 12])
def test_random_shapes_through_the_fused_entry_points(seed):
    """Seeded random shapes (token counts, hidden and intermediate sizes that are not multiples of a tile, ranks from 0 to
    64 including partial rank tiles, with and without noise, norm and bias): every plan the host logic makes for them
    is checked against the oracle, twice on one workspace."""
    rng = np.random.default_rng(seed)
    lib = qerl.load_library()
    ranks = [0, 8, 16, 24, 32, 40, 64]
    for it in range(16):
        M = int(rng.integers(1, 17))
        H = int(rng.integers(4, 140)) * 16
        sigma = [None, 1e-2, 5e-4][int(rng.integers(0, 3))]
        if it % 2 == 0:
            I = int(rng.integers(1, 150)) * 16
            rs = tuple(int(ranks[rng.integers(0, len(ranks))]) for _ in range(3))
            print("random mlp case", seed, it, M, H, I, rs, sigma, flush=True)
            xin, gain, Z, xn = _norm_inputs(M, H, 100 * seed + it, sigma)
            gate, up, down = (_member(I, H, rs[0], 9000 + 10 * it + seed), _member(I, H, rs[1], 9001 + 10 * it + seed),
                              _member(H, I, rs[2], 9002 + 10 * it + seed))
            act = oracle.silu_mul(_bf16(_ref(gate, xn, 2.0)), _bf16(_ref(up, xn, 2.0))).astype(np.float32)
            ws = qerl.Workspace(lib.aqn_rmsnorm_nvfp4_lora_mlp_workspace_bytes(M, H, I, H, *rs))
            call = lambda: qerl.aqn_rmsnorm_nvfp4_lora_mlp(
                xin.cuda(), gain.cuda(), Z.cuda() if Z is not None else None, 1e-6, gate["pw"], up["pw"], down["pw"],
                (gate["Ad"], up["Ad"], down["Ad"]), (gate["Bd"], up["Bd"], down["Bd"]), (2.0, 2.0, 2.0), workspace=ws)
            y = call().clone()
            again = call()
            torch.cuda.synchronize()
            assert qerl.workspace_status(ws) == 0
            check_linear(y, _ref(down, act, 2.0), ("random mlp", seed, it, M, H, I, rs), slack=4e-3)
            assert torch.equal(y, again)
        else:
            n = int(rng.integers(1, 5))
            Ns = [int(rng.integers(1, 700)) for _ in range(n)]
            rs = [int(ranks[rng.integers(0, len(ranks))]) for _ in range(n)]
            use_norm, bias = bool(rng.random() < 0.7), bool(rng.integers(0, 2))
            print("random group case", seed, it, M, H, Ns, rs, sigma, use_norm, bias, flush=True)
            xin, gain, Z, xn = _norm_inputs(M, H, 100 * seed + it, sigma)
            mem = [_member(N, H, r, 9500 + 10 * it + i + seed, bias) for i, (N, r) in enumerate(zip(Ns, rs))]
            ws = qerl.Workspace(qerl.aqn_rmsnorm_nvfp4_lora_linear_group_workspace_bytes(M, H, Ns, rs))
            call = lambda: qerl.aqn_rmsnorm_nvfp4_lora_linear_group(
                xin.cuda(), gain.cuda() if use_norm else None, Z.cuda() if (Z is not None and use_norm) else None, 1e-6,
                [m["pw"] for m in mem], [m["Ad"] for m in mem], [m["Bd"] for m in mem], [2.0] * n, workspace=ws,
                biases=[m["bd"] for m in mem])
            outs = [o.clone() for o in call()]
            again = call()
            torch.cuda.synchronize()
            assert qerl.workspace_status(ws) == 0
            xr = xn if use_norm else xin.float().numpy()
            for i, (m, y) in enumerate(zip(mem, outs)):
                check_linear(y, _ref(m, xr, 2.0), ("random group", seed, it, i, M, H, Ns, rs), slack=2e-3)
            assert all(torch.equal(p, q) for p, q in zip(outs, again))
