"""GPU parity: nvfp4_lora_linear against the oracle (fp64 accumulation)."""
import numpy as np
import pytest
import torch

import paper_2510_11696_amd as qerl
import qerl_synth as qs
from oracle import nvfp4_oracle as oracle
from tests import cases
from tests.gpu_util import bf16_ulp_distance, check_linear, to_gpu_bf16

pytestmark = pytest.mark.gpu


def _problem(M, N, K, r, seed, w_std=0.02, W=None):
    if W is None:
        W = cases.gaussian(N, K, seed, w_std)
    x = qs.activations(M, K, seed + 1)
    A = B = None
    if r > 0:
        A, B = qs.lora_pair(N, K, r, seed + 2)
    return W, x, A, B


def _run(M, N, K, r, seed, alpha_over_r=2.0, W=None, label="", packed=False):
    print("linear case", label, M, N, K, r, seed, "packed" if packed else "canonical", flush=True)
    W, x, A, B = _problem(M, N, K, r, seed, W=W)
    codes, scales, ts = oracle.nvfp4_quantize(W)
    g = lambda a: torch.from_numpy(a).cuda()
    ts_gpu = torch.tensor([ts], dtype=torch.float32, device="cuda")
    if packed:
        pw = qerl.nvfp4_prepack(g(codes), g(scales), ts_gpu)
        y = qerl.nvfp4_lora_linear_packed(x.cuda(), pw, A.cuda() if r else None, B.cuda() if r else None,
                                          alpha_over_r)
    else:
        y = qerl.nvfp4_lora_linear(x.cuda(), g(codes), g(scales), ts_gpu,
                                   A.cuda() if r else None, B.cuda() if r else None, alpha_over_r)
    torch.cuda.synchronize()
    ref = oracle.nvfp4_lora_linear(x.float().numpy(), codes, scales, ts,
                                   A.float().numpy() if r else None, B.float().numpy() if r else None,
                                   alpha_over_r)
    check_linear(y, ref, (label, M, N, K, r))
    return y, ref


PATHS = [False, True]   # canonical layout, tile-packed layout


@pytest.mark.parametrize("packed", PATHS)
def test_config1_single_linear(packed):
    """K = N = 2048, one token, LoRA r = 16, alpha = 32."""
    _run(1, 2048, 2048, 16, seed=qs.seed_for(1, 0), alpha_over_r=32.0 / 16, packed=packed)


@pytest.mark.parametrize("packed", PATHS)
@pytest.mark.parametrize("M", [1, 2, 3, 8, 9, 15, 16])
@pytest.mark.parametrize("N,K,r", [(512, 3584, 32), (3584, 3584, 32), (96, 18944, 32), (1184, 3584, 0)])
def test_decode_shapes(M, N, K, r, packed):
    _run(M, N, K, r, seed=M * 7 + N + K, packed=packed)


@pytest.mark.parametrize("packed", PATHS)
@pytest.mark.parametrize("M,N,K,r", [
    (3, 40, 320, 8),       # ragged N tile, K not a multiple of 256
    (5, 17, 64, 3),        # single K chunk, odd rank
    (16, 1000, 2112, 16),  # ragged everything, several tiles
    (7, 16, 5120, 64),     # two workgroups along K
    (2, 33, 27648, 64),    # many workgroups along K
    (4, 70, 1024, 80),     # rank beyond the preloaded 64
    (8, 64, 48, 4),        # K smaller than one tile and not a multiple of 64
])
def test_ragged_shapes(M, N, K, r, packed):
    _run(M, N, K, r, seed=M + N + K, packed=packed)


@pytest.mark.parametrize("M,N,K,r", [(4, 24, 48, 4), (1, 8, 16, 0), (9, 130, 1040, 16)])
def test_general_kernel_k_not_multiple_of_64(M, N, K, r):
    _run(M, N, K, r, seed=3 * M + N)


@pytest.mark.parametrize("packed", PATHS)
@pytest.mark.parametrize("M", [17, 32, 100, 128])
def test_more_than_16_tokens(M, packed):
    _run(M, 512, 3584, 32, seed=M, packed=packed)


@pytest.mark.parametrize("M,N,K,r", [
    (17, 1000, 2112, 16),    # ragged N, K not a multiple of 128, one token past the decode kernels
    (32, 3584, 3584, 32),    # exactly one block of token rows
    (33, 96, 18944, 32),     # long K: split over workgroups, partial outputs added by the second kernel
    (64, 4736, 3584, 0),     # no adapter
    (65, 70, 1024, 64),      # ragged last tile, rank 64
    (100, 37, 48, 8),        # K smaller than one packed tile
    (128, 2048, 5120, 32),
    (128, 160, 27648, 8),    # longest K of the 32B shapes
])
def test_a_few_dozen_tokens_on_packed_weights(M, N, K, r):
    _run(M, N, K, r, seed=M + N + K + r, packed=True)


@pytest.mark.parametrize("packed", PATHS)
@pytest.mark.parametrize("M,N,K,r", [
    (129, 512, 3584, 32),    # one token past the 17..128-token kernel: two blocks of token rows in the GEMM
    (200, 1000, 2112, 16),   # ragged N and K
    (256, 96, 18944, 32),    # long K: the LoRA down-projection splits K over workgroups
    (300, 300, 1024, 0),     # no adapter
    (640, 130, 5120, 64),    # rank 64, ragged last column tile
])
def test_prefill_token_counts(M, N, K, r, packed):
    _run(M, N, K, r, seed=M + N + K + r, packed=packed)


@pytest.mark.parametrize("packed", PATHS)
def test_adversarial_weights_through_the_linear(packed):
    for name, W in cases.quantizer_cases(48, 512, seed=31).items():
        if name in ("scaled_up", "scaled_down"):
            continue
        _run(4, 48, 512, 8, seed=5, W=W, label=name, packed=packed)


def _pack_reference(codes, scales):
    """The tile-packed layout written out with numpy from its definition:
    tiles of 32 rows x 128 inputs, 2304 bytes each; lane l = (n = l % 32, kg = l // 32)
    owns, per 16-input step j, the 4 code bytes of inputs 16 j + 8 kg .. + 7."""
    N, K = codes.shape[0], codes.shape[1] * 2
    nt, kt = -(-N // 32), -(-K // 128)
    cp = np.zeros((nt * 32, kt * 64), dtype=np.uint8)
    cp[:N, :K // 2] = codes
    sp = np.zeros((nt * 32, kt * 8), dtype=np.uint8)
    sp[:N, :K // 16] = scales
    out = np.zeros((nt, kt, 2304), dtype=np.uint8)
    for a in range(nt):
        for b in range(kt):
            tile_c = cp[a * 32:(a + 1) * 32, b * 64:(b + 1) * 64]      # [n, 64 bytes]
            for plane in range(2):
                for lane in range(64):
                    n, kg = lane % 32, lane // 32
                    for dw in range(4):
                        j = 4 * plane + dw
                        src = tile_c[n, 8 * j + 4 * kg: 8 * j + 4 * kg + 4]
                        off = plane * 1024 + lane * 16 + dw * 4
                        out[a, b, off:off + 4] = src
            out[a, b, 2048:] = sp[a * 32:(a + 1) * 32, b * 8:(b + 1) * 8].reshape(-1)
    return out.reshape(-1)


@pytest.mark.parametrize("N,K", [(32, 128), (40, 320), (100, 48), (64, 1024)])
def test_prepack_is_the_documented_permutation(N, K):
    rng = np.random.default_rng(N + K)
    codes = rng.integers(0, 256, size=(N, K // 2)).astype(np.uint8)
    scales = rng.integers(0, 0x7F, size=(N, K // 16)).astype(np.uint8)
    pw = qerl.nvfp4_prepack(torch.from_numpy(codes).cuda(), torch.from_numpy(scales).cuda(),
                            torch.ones(1, device="cuda"))
    got = pw.packed.cpu().numpy()
    want = _pack_reference(codes, scales)
    assert got.size == want.size == -(-N // 32) * -(-K // 128) * 2304
    assert np.array_equal(got, want)


def test_one_hot_reads_exact_dequantised_column():
    N, K = 64, 512
    W = cases.gaussian(N, K, 3)
    codes, scales, ts = oracle.nvfp4_quantize(W)
    Wh = oracle.nvfp4_dequantize(codes, scales, ts)
    ks = [0, 15, 16, 255, 256, 300, 511]
    x = torch.zeros((len(ks), K), dtype=torch.bfloat16)
    for m, k in enumerate(ks):
        x[m, k] = 1.0
    g = lambda a: torch.from_numpy(a).cuda()
    y = qerl.nvfp4_lora_linear(x.cuda(), g(codes), g(scales), torch.tensor([ts], device="cuda"))
    want = torch.from_numpy(Wh[:, ks].T.copy()).to(torch.bfloat16)
    assert torch.equal(y.cpu(), want)
    pw = qerl.nvfp4_prepack(g(codes), g(scales), torch.tensor([ts], device="cuda"))
    assert torch.equal(qerl.nvfp4_lora_linear_packed(x.cuda(), pw).cpu(), want)


@pytest.mark.parametrize("packed", PATHS)
def test_deterministic_and_workspace_reuse(packed):
    M, N, K, r = 8, 3584, 18944, 32
    W, x, A, B = _problem(M, N, K, r, 11)
    cw, sw, tw = qerl.nvfp4_quantize(to_gpu_bf16(W))
    ws = qerl.Workspace(qerl.nvfp4_lora_linear_workspace_bytes(M, N, K, r))
    if packed:
        pw = qerl.nvfp4_prepack(cw, sw, tw)
        call = lambda x_, w_, A_, B_, **kw: qerl.nvfp4_lora_linear_packed(x_, w_, A_, B_, 2.0, **kw)
        w1 = pw
    else:
        call = lambda x_, w_, A_, B_, **kw: qerl.nvfp4_lora_linear(x_, *w_, A_, B_, 2.0, **kw)
        w1 = (cw, sw, tw)
    args = (x.cuda(), w1, A.cuda(), B.cuda())
    y0 = call(*args, workspace=ws).clone()
    for _ in range(10):
        assert torch.equal(call(*args, workspace=ws), y0)
    # a different, smaller problem on the same workspace, then the first again
    W2, x2, A2, B2 = _problem(3, 96, 18944, 32, 12)
    c2, s2, t2 = qerl.nvfp4_quantize(to_gpu_bf16(W2))
    w2 = qerl.nvfp4_prepack(c2, s2, t2) if packed else (c2, s2, t2)
    y2 = call(x2.cuda(), w2, A2.cuda(), B2.cuda(), workspace=ws)
    y2b = call(x2.cuda(), w2, A2.cuda(), B2.cuda())
    assert torch.equal(y2, y2b)
    assert torch.equal(call(*args, workspace=ws), y0)


def test_strided_x_and_y_and_canaries():
    M, N, K, r = 5, 200, 768, 16
    W, x, A, B = _problem(M, N, K, r, 21)
    codes, scales, ts = oracle.nvfp4_quantize(W)
    xb = torch.full((M, K + 64), 3.0, dtype=torch.bfloat16, device="cuda")
    xb[:, :K] = x.cuda()
    out = torch.full((M, N + 56), -5.0, dtype=torch.bfloat16, device="cuda")
    g = lambda a: torch.from_numpy(a).cuda()
    qerl.nvfp4_lora_linear(xb[:, :K], g(codes), g(scales), torch.tensor([ts], device="cuda"),
                           A.cuda(), B.cuda(), 2.0, out=out[:, :N])
    ref = oracle.nvfp4_lora_linear(x.float().numpy(), codes, scales, ts, A.float().numpy(), B.float().numpy(), 2.0)
    check_linear(out[:, :N].contiguous(), ref, "strided")
    assert torch.all(out[:, N:] == -5.0)


def test_rmsnorm_feeds_linear_end_to_end():
    """AQN RMSNorm -> NVFP4 linear equals the oracle's composition, and the
    noise acts like row-scaled weights (Appendix "Proof of Noise Sharing")."""
    M, H, N, r = 8, 3584, 512, 32
    xin = qs.activations(M, H, 50)
    gain = qs.rms_gain(H, 51)
    Z = qs.aqn_noise(H, 1e-2, 52)
    W = cases.gaussian(N, H, 53)
    A, B = qs.lora_pair(N, H, r, 54)
    codes, scales, ts = qerl.nvfp4_quantize(to_gpu_bf16(W))
    xn = qerl.aqn_rmsnorm(xin.cuda(), gain.cuda(), Z.cuda())
    y = qerl.nvfp4_lora_linear(xn, codes, scales, ts, A.cuda(), B.cuda(), 2.0)
    # oracle: the linear consumes the bf16 activations the norm produced
    ref = oracle.nvfp4_lora_linear(xn.float().cpu().numpy(), codes.cpu().numpy(), scales.cpu().numpy(),
                                   np.float32(ts.item()), A.float().numpy(), B.float().numpy(), 2.0)
    check_linear(y, ref, "norm->linear")


@pytest.mark.parametrize("M", [1, 8, 16, 17, 40, 128, 160, 300])   # the last two: the prefill kernel's grouped launch
@pytest.mark.parametrize("K,Ns,rs", [
    (3584, (3584, 512, 512), (32, 32, 32)),      # q, k, v of the 7B block
    (3584, (1184, 1184), (32, 32)),              # a slice of gate, up
    (5120, (1024, 96, 40), (64, 0, 16)),         # mixed ranks, ragged row tiles
    (18944, (64, 32), (32, 32)),                 # K split over several workgroups
])
def test_grouped_launch_equals_oracle(M, K, Ns, rs):
    """One launch for several linears that share x: each member within tolerance of the oracle (the
    single-linear call may split K differently, so the two agree to rounding, not bit for bit), and the
    grouped call repeats bit for bit."""
    print("group case", M, K, Ns, rs, flush=True)
    x = qs.activations(M, K, 900 + M)
    g = lambda a: torch.from_numpy(a).cuda()
    ws_, As, Bs, refs = [], [], [], []
    for i, (N, r) in enumerate(zip(Ns, rs)):
        W = cases.gaussian(N, K, 1000 + 10 * i + M)
        codes, scales, ts = oracle.nvfp4_quantize(W)
        A = B = None
        if r:
            A, B = qs.lora_pair(N, K, r, 2000 + i)
        ws_.append(qerl.nvfp4_prepack(g(codes), g(scales), torch.tensor([ts], device="cuda")))
        As.append(A.cuda() if r else None)
        Bs.append(B.cuda() if r else None)
        refs.append(oracle.nvfp4_lora_linear(x.float().numpy(), codes, scales, ts,
                                             A.float().numpy() if r else None, B.float().numpy() if r else None, 2.0))
    outs = qerl.nvfp4_lora_linear_packed_group(x.cuda(), ws_, As, Bs, [2.0] * len(Ns))
    torch.cuda.synchronize()
    for i, (y, ref) in enumerate(zip(outs, refs)):
        check_linear(y, ref, ("group", i, M, K, Ns, rs))
        single = qerl.nvfp4_lora_linear_packed(x.cuda(), ws_[i], As[i], Bs[i], 2.0)
        check_linear(single, ref, ("single", i, M, K, Ns, rs))
    again = qerl.nvfp4_lora_linear_packed_group(x.cuda(), ws_, As, Bs, [2.0] * len(Ns))
    assert all(torch.equal(p, q) for p, q in zip(outs, again))


@pytest.mark.parametrize("M", [1, 7, 8, 16])
@pytest.mark.parametrize("H,Ns,rs,sigma", [
    (3584, (3584, 512, 512), (32, 32, 32), 1e-2),   # q, k, v of the 7B block
    (3584, (1184, 1184), (32, 32), 5e-4),           # a slice of gate, up
    (2048, (96, 64), (64, 16), None),               # two rank tiles in one adapter; a partial rank tile; stage 0
    (4096, (64,), (8,), 1e-2),
    (5120, (1024, 96), (64, 64), 5e-3),             # rows longer than 4096: the wide variants; 14B / 32B hidden size
    (5120, (160, 64, 64), (64, 64, 64), 1e-2),      # q, k, v adapters of the 32B configuration: six rank tiles
])
def test_norm_with_lora_down_feeds_grouped_linear(M, H, Ns, rs, sigma):
    """aqn_rmsnorm_lora_down: y within one bf16 unit of the oracle (as aqn_rmsnorm), t = y A^T within fp32 summation error of
    the oracle's product, and the grouped linear fed with that t within tolerance of the oracle."""
    print("norm+down case", M, H, Ns, rs, sigma, flush=True)
    xin = qs.activations(M, H, 300 + M)
    gain = qs.rms_gain(H, 301)
    Z = qs.aqn_noise(H, sigma, 302) if sigma is not None else None
    g = lambda a: torch.from_numpy(a).cuda()
    ws_, As, Bs, W_q = [], [], [], []
    for i, (N, r) in enumerate(zip(Ns, rs)):
        W = cases.gaussian(N, H, 3000 + 10 * i + M)
        codes, scales, ts = oracle.nvfp4_quantize(W)
        A, B = qs.lora_pair(N, H, r, 4000 + i)
        ws_.append(qerl.nvfp4_prepack(g(codes), g(scales), torch.tensor([ts], device="cuda")))
        As.append(A.cuda()); Bs.append(B.cuda()); W_q.append((codes, scales, ts, A, B))
    y_plain = qerl.aqn_rmsnorm(xin.cuda(), gain.cuda(), Z.cuda() if Z is not None else None, 1e-6)
    y, ts_gpu = qerl.aqn_rmsnorm_lora_down(xin.cuda(), gain.cuda(), Z.cuda() if Z is not None else None, 1e-6, As)
    torch.cuda.synchronize()
    # same function as aqn_rmsnorm, other summation order of the mean: within one bf16 unit of the fp64 oracle
    ref_y = oracle.aqn_rmsnorm(xin.float().numpy(), gain.float().numpy(), Z.numpy() if Z is not None else None, 1e-6)
    d = bf16_ulp_distance(y, ref_y)
    assert d.max() <= 1 and (d > 0).mean() < 0.01
    assert bf16_ulp_distance(y_plain, ref_y).max() <= 1
    y64 = y.float().cpu().numpy().astype(np.float64)
    for (codes, scales, ts, A, B), t_gpu in zip(W_q, ts_gpu):
        t_ref = oracle.lora_down_projection(y.float().cpu().numpy(), A.float().numpy())   # Eq. 2's inner factor on the y the kernel wrote
        bound = 4 * H * 2.0 ** -24 * (np.abs(y64) @ np.abs(A.float().numpy().astype(np.float64)).T) + 1e-30
        assert tuple(t_gpu.shape) == (8, M, A.shape[0])
        assert (np.abs(t_gpu.cpu().numpy().astype(np.float64).sum(0) - t_ref) <= bound).all()
    outs = qerl.nvfp4_lora_linear_packed_group(y, ws_, As, Bs, [2.0] * len(Ns), ts=ts_gpu)
    outs_self = qerl.nvfp4_lora_linear_packed_group(y, ws_, As, Bs, [2.0] * len(Ns))
    torch.cuda.synchronize()
    for i, ((codes, scales, ts, A, B), out, out_self) in enumerate(zip(W_q, outs, outs_self)):
        ref = oracle.nvfp4_lora_linear(y.float().cpu().numpy(), codes, scales, ts, A.float().numpy(), B.float().numpy(), 2.0)
        check_linear(out, ref, ("norm+down -> group", i, M, H, Ns, rs))
        check_linear(out_self, ref, ("group computing t itself", i, M, H, Ns, rs))
    again = qerl.nvfp4_lora_linear_packed_group(y, ws_, As, Bs, [2.0] * len(Ns), ts=ts_gpu)
    assert all(torch.equal(p, q) for p, q in zip(outs, again))


def _sampled_rows(N, seed, n=192):
    rng = np.random.default_rng(seed)
    rows = np.unique(np.concatenate([np.arange(32), np.arange(N - 32, N), rng.integers(0, N, size=n)]))
    return rows


@pytest.mark.timeout(400)
def test_full_size_7b_mlp_block_as_the_benchmark_launches_it():
    """The 7B MLP linears at full size (gate, up: 18944 x 3584; down: 3584 x 18944; 8 tokens, r = 32) in the
    launch configuration the benchmark times -- fused norm + LoRA-down feeding one grouped gate+up launch,
    then down on its own (K split over workgroup ranges) -- checked on sampled output rows, which the oracle
    computes from the same quantised rows one by one (the layer is separable over output rows)."""
    M, H, I, r = 8, 3584, 18944, 32
    print("full-size case", M, H, I, r, flush=True)
    g = lambda a: torch.from_numpy(a).cuda()
    xin = qs.activations(M, H, 7001)
    gain = qs.rms_gain(H, 7002)
    Z = qs.aqn_noise(H, 1e-2, 7003)
    members = []
    for i, (N, K) in enumerate([(I, H), (I, H), (H, I)]):
        W = cases.gaussian(N, K, 7100 + i)
        codes, scales, ts = oracle.nvfp4_quantize(W)
        del W
        A, B = qs.lora_pair(N, K, r, 7200 + i)
        pw = qerl.nvfp4_prepack(g(codes), g(scales), torch.tensor([ts], device="cuda"))
        members.append((codes, scales, ts, A, B, pw))
        print("  quantised member", i, flush=True)
    y, ts_gpu = qerl.aqn_rmsnorm_lora_down(xin.cuda(), gain.cuda(), Z.cuda(), 1e-6, [m[3].cuda() for m in members[:2]])
    outs = qerl.nvfp4_lora_linear_packed_group(y, [m[5] for m in members[:2]], [m[3].cuda() for m in members[:2]],
                                               [m[4].cuda() for m in members[:2]], [2.0, 2.0], ts=ts_gpu)
    torch.cuda.synchronize()
    y_np = y.float().cpu().numpy()
    for i in range(2):
        codes, scales, ts, A, B, _ = members[i]
        rows = _sampled_rows(I, 7300 + i)
        ref = oracle.nvfp4_lora_linear(y_np, codes[rows], scales[rows], ts, A.float().numpy(), B.float().numpy()[rows], 2.0)
        check_linear(outs[i][:, torch.from_numpy(rows).cuda()], ref, ("full-size gate/up", i))
    # down reads the (synthetic) activation of the block: gate's output stands in for silu(gate) * up
    codes, scales, ts, A, B, pw = members[2]
    x_down = (outs[0].float() * 8.0).to(torch.bfloat16)   # rescaled to unit-ish magnitude, any bf16 values serve
    out = qerl.nvfp4_lora_linear_packed(x_down, pw, A.cuda(), B.cuda(), 2.0)
    torch.cuda.synchronize()
    rows = _sampled_rows(H, 7302)
    ref = oracle.nvfp4_lora_linear(x_down.float().cpu().numpy(), codes[rows], scales[rows], ts, A.float().numpy(),
                                   B.float().numpy()[rows], 2.0)
    check_linear(out[:, torch.from_numpy(rows).cuda()], ref, ("full-size down",))



@pytest.mark.timeout(400)
def test_full_size_14b_gate_at_prefill_as_the_benchmark_launches_it():
    """14B gate_proj (13824 x 5120), 2048 tokens, r = 64 -- the prefill configuration of the benchmark --
    checked on sampled output rows against the oracle."""
    M, K, N, r = 2048, 5120, 13824, 64
    print("full-size prefill case", M, N, K, r, flush=True)
    g = lambda a: torch.from_numpy(a).cuda()
    x = qs.activations(M, K, 8001)
    W = cases.gaussian(N, K, 8002)
    codes, scales, ts = oracle.nvfp4_quantize(W)
    del W
    A, B = qs.lora_pair(N, K, r, 8003)
    pw = qerl.nvfp4_prepack(g(codes), g(scales), torch.tensor([ts], device="cuda"))
    y = qerl.nvfp4_lora_linear_packed(x.cuda(), pw, A.cuda(), B.cuda(), 1.0)
    torch.cuda.synchronize()
    rows = _sampled_rows(N, 8004, n=96)
    ref = oracle.nvfp4_lora_linear(x.float().numpy(), codes[rows], scales[rows], ts, A.float().numpy(), B.float().numpy()[rows], 1.0)
    check_linear(y[:, torch.from_numpy(rows).cuda()], ref, ("full-size prefill gate",))


def test_grouped_prefill_with_many_token_blocks_and_rank_64():
    """33 token blocks, four adapters of rank 64 (eight rank tiles): the grouped down-projection and GEMM launches."""
    M, K, Ns, rs = 1056, 256, (64, 96, 32, 64), (64, 64, 64, 64)
    x = qs.activations(M, K, 9900)
    g = lambda a: torch.from_numpy(a).cuda()
    ws_, As, Bs, refs = [], [], [], []
    for i, (N, r) in enumerate(zip(Ns, rs)):
        W = cases.gaussian(N, K, 9910 + i)
        codes, scales, ts = oracle.nvfp4_quantize(W)
        A, B = qs.lora_pair(N, K, r, 9920 + i)
        ws_.append(qerl.nvfp4_prepack(g(codes), g(scales), torch.tensor([ts], device="cuda")))
        As.append(A.cuda()); Bs.append(B.cuda())
        refs.append(oracle.nvfp4_lora_linear(x.float().numpy(), codes, scales, ts, A.float().numpy(), B.float().numpy(), 2.0))
    outs = qerl.nvfp4_lora_linear_packed_group(x.cuda(), ws_, As, Bs, [2.0] * len(Ns))
    torch.cuda.synchronize()
    for i, (y, ref) in enumerate(zip(outs, refs)):
        check_linear(y, ref, ("many token blocks", i))


@pytest.mark.parametrize("M,K,Ns,rs", [
    (257, 992, (64, 40, 96), (64, 32, 8)),            # 4 rank tiles, one of them partial; K not a multiple of 64; ragged token block
    (300, 2048, (32, 32, 64, 32), (64, 64, 64, 64)),  # 8 rank tiles: four per wave
    (320, 64, (96,), (8,)),                           # one partial rank tile; a single slab, no K-parts
    (513, 4096, (64, 64, 32), (64, 32, 64)),          # 5 rank tiles (the sixth slot repeats the last); 8 K-parts
    (1030, 1536, (40,), (64,)),                       # one adapter, two tiles; 17 token blocks
])
def test_lora_down_projection_of_256_tokens_and_more(M, K, Ns, rs):
    """The 64-token down-projection kernel behind the prefill GEMM: odd and full rank-tile counts, partial tiles,
    K-parts with a ragged last slab, ragged token blocks.  Small N keeps the main product cheap; the adapters' share
    of the output is made large (lora_scale 8) so that a wrong t shows."""
    print("down-projection case", M, K, Ns, rs, flush=True)
    x = qs.activations(M, K, 9700 + M)
    g = lambda a: torch.from_numpy(a).cuda()
    ws_, As, Bs, refs = [], [], [], []
    for i, (N, r) in enumerate(zip(Ns, rs)):
        W = cases.gaussian(N, K, 9710 + 10 * i + M)
        codes, scales, ts = oracle.nvfp4_quantize(W)
        A, B = qs.lora_pair(N, K, r, 9720 + i)
        ws_.append(qerl.nvfp4_prepack(g(codes), g(scales), torch.tensor([ts], device="cuda")))
        As.append(A.cuda()); Bs.append(B.cuda())
        refs.append(oracle.nvfp4_lora_linear(x.float().numpy(), codes, scales, ts, A.float().numpy(), B.float().numpy(), 8.0))
    outs = qerl.nvfp4_lora_linear_packed_group(x.cuda(), ws_, As, Bs, [8.0] * len(Ns))
    torch.cuda.synchronize()
    for i, (y, ref) in enumerate(zip(outs, refs)):
        check_linear(y, ref, ("down-projection", i, M, K))
    again = qerl.nvfp4_lora_linear_packed_group(x.cuda(), ws_, As, Bs, [8.0] * len(Ns))
    assert all(torch.equal(p, q) for p, q in zip(outs, again))
    if len(Ns) == 1:
        single = qerl.nvfp4_lora_linear_packed(x.cuda(), ws_[0], As[0], Bs[0], 8.0)
        check_linear(single, refs[0], ("down-projection, single call", M, K))


@pytest.mark.timeout(600)
def test_full_size_14b_gate_and_up_at_prefill_as_the_benchmark_launches_them():
    """14B gate_proj and up_proj (13824 x 5120 each) in one grouped call at 2048 tokens, r = 64, with bias: 864
    workgroups of the largest tile shape, 3.4 rounds of the chip, which goes out as three whole rounds plus a launch
    of the remaining columns in a smaller shape, cut inside up_proj.  Checked on sampled output rows against the
    oracle, the rows on both sides of every multiple of 512 near the cut among them."""
    M, K, N, r = 2048, 5120, 13824, 64
    print("full-size grouped prefill case", M, N, K, r, flush=True)
    g = lambda a: torch.from_numpy(a).cuda()
    x = qs.activations(M, K, 8101)
    members = []
    for i in range(2):
        W = cases.gaussian(N, K, 8110 + i)
        codes, scales, ts = oracle.nvfp4_quantize(W)
        del W
        A, B = qs.lora_pair(N, K, r, 8120 + i)
        bias = (torch.randn(N, generator=torch.Generator().manual_seed(8130 + i)) * 0.5).to(torch.bfloat16)
        pw = qerl.nvfp4_prepack(g(codes), g(scales), torch.tensor([ts], device="cuda"))
        members.append((codes, scales, ts, A, B, bias, pw))
        print("  quantised member", i, flush=True)
    outs = qerl.nvfp4_lora_linear_packed_group(x.cuda(), [m[6] for m in members], [m[3].cuda() for m in members],
                                               [m[4].cuda() for m in members], [1.0, 1.0],
                                               biases=[m[5].cuda() for m in members])
    torch.cuda.synchronize()
    x_np = x.float().numpy()
    edges = np.concatenate([np.arange(c - 2, c + 2) for c in range(9216, N, 512)])
    for i, (codes, scales, ts, A, B, bias, _) in enumerate(members):
        rows = np.unique(np.concatenate([_sampled_rows(N, 8140 + i, n=64), edges]))
        ref = oracle.nvfp4_lora_linear(x_np, codes[rows], scales[rows], ts, A.float().numpy(), B.float().numpy()[rows], 1.0,
                                       bias=bias.float().numpy()[rows])
        check_linear(outs[i][:, torch.from_numpy(rows).cuda()], ref, ("full-size grouped prefill", i))


@pytest.mark.parametrize("M", [1, 8, 16, 40, 128, 200])
@pytest.mark.parametrize("K,Ns,rs", [
    (3584, (3584, 512, 512), (32, 32, 32)),      # q, k, v of the 7B block: the three projections that carry a bias
    (18944, (96, 40), (32, 0)),                  # K split over workgroup ranges; a member without adapter; ragged tile
])
def test_bias_in_grouped_and_single_launches(M, K, Ns, rs):
    print("bias case", M, K, Ns, rs, flush=True)
    x = qs.activations(M, K, 9100 + M)
    g = lambda a: torch.from_numpy(a).cuda()
    ws_, As, Bs, biases, refs = [], [], [], [], []
    for i, (N, r) in enumerate(zip(Ns, rs)):
        W = cases.gaussian(N, K, 9200 + 10 * i + M)
        codes, scales, ts = oracle.nvfp4_quantize(W)
        A = B = None
        if r:
            A, B = qs.lora_pair(N, K, r, 9300 + i)
        bias = (torch.randn(N, generator=torch.Generator().manual_seed(9400 + i)) * 0.5).to(torch.bfloat16)
        ws_.append(qerl.nvfp4_prepack(g(codes), g(scales), torch.tensor([ts], device="cuda")))
        As.append(A.cuda() if r else None)
        Bs.append(B.cuda() if r else None)
        biases.append(bias.cuda())
        refs.append(oracle.nvfp4_lora_linear(x.float().numpy(), codes, scales, ts, A.float().numpy() if r else None,
                                             B.float().numpy() if r else None, 2.0, bias=bias.float().numpy()))
    outs = qerl.nvfp4_lora_linear_packed_group(x.cuda(), ws_, As, Bs, [2.0] * len(Ns), biases=biases)
    torch.cuda.synchronize()
    for i, (y, ref) in enumerate(zip(outs, refs)):
        check_linear(y, ref, ("group with bias", i, M, K))
        single = qerl.nvfp4_lora_linear_packed_group(x.cuda(), ws_[i:i + 1], As[i:i + 1], Bs[i:i + 1], [2.0],
                                                     biases=biases[i:i + 1])[0]
        check_linear(single, ref, ("single with bias", i, M, K))
    # a member without bias next to members with one
    mixed = qerl.nvfp4_lora_linear_packed_group(x.cuda(), ws_, As, Bs, [2.0] * len(Ns), biases=[biases[0]] + [None] * (len(Ns) - 1))
    check_linear(mixed[0], refs[0], ("mixed", 0))
    assert not torch.equal(mixed[1], outs[1])



@pytest.mark.parametrize("M", [1, 8, 16, 17, 40, 200])
@pytest.mark.parametrize("K,N,r,fused_buffer", [
    (18944, 160, 32, True),      # the 7B down projection's K (several K-ranges), ragged row tile; gate | up side by side
    (2048, 96, 16, False),
    (3584, 64, 0, False),        # no adapter
])
def test_down_projection_on_the_gated_input(M, K, N, r, fused_buffer):
    """y = down(bf16(bf16(SiLU(gate)) * up)): within tolerance of the oracle, and nearly bit for bit what the
    plain packed linear gives when it is handed the oracle's gated tensor (the device evaluates SiLU in fp32
    with the hardware's exp2 and reciprocal, the oracle in fp64: a rounding to bf16 may fall the other way for a few
    elements in ten thousand)."""
    print("swiglu case", M, K, N, r, flush=True)
    gu = qs.activations(M, 2 * K, 7100 + M) * 2.0
    gate, up = gu[:, :K], gu[:, K:]
    W = cases.gaussian(N, K, 7200 + M)
    codes, scales, ts = oracle.nvfp4_quantize(W)
    A = B = None
    if r:
        A, B = qs.lora_pair(N, K, r, 7300)
    g = lambda a: torch.from_numpy(a).cuda()
    pw = qerl.nvfp4_prepack(g(codes), g(scales), torch.tensor([ts], device="cuda"))
    act = oracle.silu_mul(gate.float().numpy(), up.float().numpy())
    ref = oracle.nvfp4_lora_linear(act.astype(np.float32), codes, scales, ts, A.float().numpy() if r else None,
                                   B.float().numpy() if r else None, 2.0)
    if fused_buffer:
        dev = gu.cuda()
        gd, ud = dev[:, :K], dev[:, K:]
    else:
        gd, ud = gate.contiguous().cuda(), up.contiguous().cuda()
    Ad, Bd = (A.cuda(), B.cuda()) if r else (None, None)
    y = qerl.nvfp4_lora_linear_packed_swiglu(gd, ud, pw, Ad, Bd, 2.0)
    torch.cuda.synchronize()
    check_linear(y, ref, ("swiglu", M, K, N, r))
    act_dev = torch.from_numpy(act.astype(np.float32)).to(torch.bfloat16).cuda()
    assert np.array_equal(act_dev.float().cpu().numpy(), act.astype(np.float32))       # the oracle's tensor is bf16-exact
    plain = qerl.nvfp4_lora_linear_packed(act_dev, pw, Ad, Bd, 2.0)
    d = (y.float() - plain.float()).abs().cpu().numpy()
    scale = np.abs(ref).max(axis=1, keepdims=True)
    assert (d <= 2.0 ** -6 * scale).all(), d.max()
    assert (d == 0).mean() >= 0.9, (d == 0).mean()
    again = qerl.nvfp4_lora_linear_packed_swiglu(gd, ud, pw, Ad, Bd, 2.0)
    assert torch.equal(y, again)


@pytest.mark.parametrize("seed", [21, 22, 23])
def test_random_shapes_where_the_gemm_splits_k(seed):
    """Seeded random shapes from 96 tokens on with few output columns, where the GEMM splits K over workgroups, adds
    the parts by a second launch and carries the LoRA down-projections as its first workgroups: ragged token blocks,
    row tiles and K (any multiple of 16), ranks 0..64, one to three members, with and without bias; each call twice
    through one workspace (arrival counters and hand-over words are left at zero), bit-equal."""
    rng = np.random.default_rng(seed)
    g = lambda a: torch.from_numpy(a).cuda()
    for it in range(6):
        M = int(rng.integers(96, 700))
        K = 16 * int(rng.integers(40, 500))
        n = int(rng.integers(1, 4))
        Ns = [8 * int(rng.integers(4, 260)) for _ in range(n)]
        rs = [int(rng.choice([0, 8, 16, 24, 32, 64])) for _ in range(n)]
        with_bias = bool(rng.integers(0, 2))
        print("random split-K case", seed, it, M, K, Ns, rs, with_bias, flush=True)
        x = qs.activations(M, K, 9500 + seed * 10 + it)
        ws_, As, Bs, biases, refs = [], [], [], [], []
        for i, (N, r) in enumerate(zip(Ns, rs)):
            W = cases.gaussian(N, K, 9600 + seed * 100 + it * 10 + i)
            codes, scales, ts = oracle.nvfp4_quantize(W)
            A = B = None
            if r:
                A, B = qs.lora_pair(N, K, r, 9700 + seed * 100 + it * 10 + i)
            bias = (torch.randn(N, generator=torch.Generator().manual_seed(9800 + i)) * 0.5).to(torch.bfloat16) if with_bias else None
            ws_.append(qerl.nvfp4_prepack(g(codes), g(scales), torch.tensor([ts], device="cuda")))
            As.append(A.cuda() if r else None)
            Bs.append(B.cuda() if r else None)
            biases.append(bias.cuda() if with_bias else None)
            refs.append(oracle.nvfp4_lora_linear(x.float().numpy(), codes, scales, ts, A.float().numpy() if r else None,
                                                 B.float().numpy() if r else None, 2.0,
                                                 bias=bias.float().numpy() if with_bias else None))
        need = qerl.nvfp4_lora_linear_workspace_bytes(M, sum(Ns), K, sum(rs))
        ws = qerl.Workspace(need)
        outs = qerl.nvfp4_lora_linear_packed_group(x.cuda(), ws_, As, Bs, [2.0] * n, workspace=ws, biases=biases)
        outs = [o.clone() for o in outs]
        again = qerl.nvfp4_lora_linear_packed_group(x.cuda(), ws_, As, Bs, [2.0] * n, workspace=ws, biases=biases)
        torch.cuda.synchronize()
        assert qerl.workspace_status(ws) == 0
        for i, (y, ref) in enumerate(zip(outs, refs)):
            check_linear(y, ref, ("random split-K", seed, it, i, M, K, Ns, rs))
            assert torch.equal(y, again[i])
