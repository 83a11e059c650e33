"""GPU parity of the backward pass (dX through the frozen NVFP4 weights, dA, dB) against the oracle."""
import numpy as np
import pytest
import torch

import paper_2510_11696_amd as qerl
import qerl_synth as qs
from oracle import nvfp4_oracle as oracle
from tests import cases
from tests.gpu_util import check_linear

pytestmark = pytest.mark.gpu


def _pack_t_reference(codes, scales):
    """Tiles of 32 inputs x 128 rows, 2304 bytes, tiles of one input tile consecutive along the rows: plane p
    (rows 64 p ..), lane l = (c = l % 32, g = l // 32): dword j at p * 1024 + 16 l + 4 j holds the codes of rows
    64 p + 16 j + 8 g + i (nibble i) at input 32 kt + c; scale bytes at 2048 + p * 128 + kb * 64 + row."""
    N, K = codes.shape[0], codes.shape[1] * 2
    kt_n, nt_n = -(-K // 32), -(-N // 128)
    nib = np.zeros((nt_n * 128, kt_n * 32), dtype=np.uint8)
    nib[:N, 0:K:2] = codes & 15
    nib[:N, 1:K:2] = codes >> 4
    sp = np.zeros((nt_n * 128, kt_n * 2), dtype=np.uint8)
    sp[:N, :K // 16] = scales
    out = np.zeros((kt_n, nt_n, 2304), dtype=np.uint8)
    for kt in range(kt_n):
        for nt in range(nt_n):
            for p in range(2):
                for lane in range(64):
                    c, g = lane % 32, lane // 32
                    for j in range(4):
                        w = 0
                        for i in range(8):
                            w |= int(nib[nt * 128 + 64 * p + 16 * j + 8 * g + i, kt * 32 + c]) << (4 * i)
                        off = p * 1024 + lane * 16 + 4 * j
                        out[kt, nt, off:off + 4] = np.frombuffer(np.uint32(w).tobytes(), dtype=np.uint8)
                for kb in range(2):
                    for row in range(64):
                        out[kt, nt, 2048 + p * 128 + kb * 64 + row] = sp[nt * 128 + 64 * p + row, kt * 2 + kb]
    return out.reshape(-1)


@pytest.mark.parametrize("N,K", [(128, 32), (40, 64), (200, 48), (256, 96)])
def test_prepack_t_is_the_documented_permutation(N, K):
    rng = np.random.default_rng(N * 7 + K)
    codes = rng.integers(0, 256, size=(N, K // 2)).astype(np.uint8)
    scales = rng.integers(0, 0x7F, size=(N, K // 16)).astype(np.uint8)
    pw = qerl.nvfp4_prepack_t(torch.from_numpy(codes).cuda(), torch.from_numpy(scales).cuda(), torch.tensor([1.0], device="cuda"))
    assert np.array_equal(pw.packed.cpu().numpy(), _pack_t_reference(codes, scales))


def _check_f32(got, ref, what):
    g = got.cpu().numpy().astype(np.float64)
    assert g.shape == ref.shape and np.all(np.isfinite(g)), what
    scale = np.abs(ref).max(axis=1, keepdims=True)
    err = np.abs(g - ref)
    # fp32 sums of bf16-exact products; x A^T and dY B enter as three bf16 terms (2^-24 relative)
    assert np.all(err <= 1e-4 * scale + 1e-30), (what, float((err / (scale + 1e-30)).max()))


@pytest.mark.parametrize("M,N,K,r", [
    (1, 64, 64, 8),
    (8, 96, 128, 16),            # fewer rows than one tile of 128; ragged input tiles
    (40, 160, 320, 16),
    (130, 1000, 2112, 32),       # two token blocks, ragged everywhere
    (200, 64, 3584, 64),         # the largest rank
    (300, 3584, 512, 32),        # the 7B k/v projection
    (520, 520, 1024, 64),        # 64-token down-projection kernel: nine token blocks (the last of 8 tokens), two rank tiles, a contraction (520) that ends inside a slab
    (64, 256, 256, 0),           # no adapter: dX only
    (16, 8, 256, 0), (16, 8, 256, 8),   # a contraction of eight rows
])
def test_backward_equals_oracle(M, N, K, r):
    print("backward case", M, N, K, r, flush=True)
    W = cases.gaussian(N, K, 8100 + M)
    codes, scales, ts = oracle.nvfp4_quantize(W)
    x = qs.activations(M, K, 8200 + M)
    dy = qs.activations(M, N, 8300 + M, std=0.5)
    A = B = None
    if r:
        A, B = qs.lora_pair(N, K, r, 8400 + M, b_std=0.05)
    g = lambda a: torch.from_numpy(a).cuda()
    pt = qerl.nvfp4_prepack_t(g(codes), g(scales), torch.tensor([ts], device="cuda"))
    dx_ref, dA_ref, dB_ref = oracle.nvfp4_lora_linear_backward(
        x.float().numpy(), dy.float().numpy(), codes, scales, ts,
        A.float().numpy() if r else None, B.float().numpy() if r else None, 2.0)
    dx, dA, dB = qerl.nvfp4_lora_linear_backward(x.cuda(), dy.cuda(), pt, A.cuda() if r else None, B.cuda() if r else None, 2.0)
    torch.cuda.synchronize()
    check_linear(dx, dx_ref, ("dx", M, N, K, r))
    if r:
        _check_f32(dA, dA_ref, ("dA", M, N, K, r))
        _check_f32(dB, dB_ref, ("dB", M, N, K, r))
    else:
        assert dA is None and dB is None
    again = qerl.nvfp4_lora_linear_backward(x.cuda(), dy.cuda(), pt, A.cuda() if r else None, B.cuda() if r else None, 2.0)
    assert torch.equal(dx, again[0]) and (not r or (torch.equal(dA, again[1]) and torch.equal(dB, again[2])))


def test_backward_of_one_hot_gradients_reads_dequantised_rows():
    """dy = rows of the identity: dx[m, :] is row n_m of W_hat rounded to bf16 (no adapter), for rows in both planes,
    several tiles and the padded tail."""
    N, K = 296, 96
    W = cases.gaussian(N, K, 8500)
    codes, scales, ts = oracle.nvfp4_quantize(W)
    rows = [0, 1, 7, 8, 15, 16, 63, 64, 127, 128, 200, 295]
    dy = torch.zeros((len(rows), 304), dtype=torch.bfloat16)[:, :N]      # a strided view: lddy = 304
    for m, n in enumerate(rows):
        dy[m, n] = 1.0
    g = lambda a: torch.from_numpy(a).cuda()
    pt = qerl.nvfp4_prepack_t(g(codes), g(scales), torch.tensor([ts], device="cuda"))
    dyd = torch.zeros((len(rows), 304), dtype=torch.bfloat16, device="cuda")
    dyd[:, :N] = dy.cuda()
    dx, _, _ = qerl.nvfp4_lora_linear_backward(None, dyd[:, :N], pt)
    What = oracle.nvfp4_dequantize(codes, scales, ts)
    want = torch.from_numpy(What[rows].astype(np.float32)).to(torch.bfloat16).float().numpy()
    assert np.array_equal(dx.float().cpu().numpy(), want)


@pytest.mark.parametrize("M,K,Ns,rs", [
    (1, 64, (64, 8), (8, 8)),
    (40, 320, (160, 96, 96), (16, 16, 0)),            # q / k / v shaped; one member without an adapter
    (130, 2112, (1000, 1000), (32, 32)),              # gate / up shaped, ragged everywhere
    (300, 512, (512, 128, 128), (32, 32, 32)),
    (520, 1024, (520, 264, 8, 1024), (64, 8, 0, 24)),  # four members, the 64-token down-projection kernel, a contraction of eight rows
    (2048, 3584, (3584, 512, 512), (32, 32, 32)),     # the 7B attention projections at a training batch
])
def test_group_backward_equals_oracle(M, K, Ns, rs):
    """dX summed over the members in one GEMM (members with different tensor scales), every member's dA and dB; one
    rounding of dX to bf16, so it is held to the linear's gate against the oracle's float64 sum."""
    print("backward group case", M, K, Ns, rs, flush=True)
    g = lambda a: torch.from_numpy(a).cuda()
    x = qs.activations(M, K, 9200 + M)
    members, weights, dys, As, Bs, scales_ = [], [], [], [], [], []
    for i, (N, r) in enumerate(zip(Ns, rs)):
        W = cases.gaussian(N, K, 9100 + M + i) * (1.0 + 3.0 * i)           # tensor scales differ from member to member
        codes, scales, ts = oracle.nvfp4_quantize(W)
        dy = qs.activations(M, N, 9300 + M + i, std=0.5)
        mem = {"dy": dy.float().numpy(), "codes": codes, "scales": scales, "tensor_scale": ts}
        A = B = None
        if r:
            A, B = qs.lora_pair(N, K, r, 9400 + M + i, b_std=0.05)
            mem.update(A=A.float().numpy(), B=B.float().numpy(), lora_scale=1.0 + 0.5 * i)
        members.append(mem)
        weights.append(qerl.nvfp4_prepack_t(g(codes), g(scales), torch.tensor([ts], device="cuda")))
        dys.append(dy.cuda()); As.append(A.cuda() if r else None); Bs.append(B.cuda() if r else None); scales_.append(1.0 + 0.5 * i)
    dx_ref, grads_ref = oracle.nvfp4_lora_linear_backward_group(x.float().numpy(), members)
    dx, grads = qerl.nvfp4_lora_linear_backward_group(x.cuda(), dys, weights, As, Bs, scales_)
    torch.cuda.synchronize()
    check_linear(dx, dx_ref, ("group dx", M, K, Ns, rs))
    for i, ((dA, dB), (dA_ref, dB_ref)) in enumerate(zip(grads, grads_ref)):
        if rs[i]:
            _check_f32(dA, dA_ref, ("group dA", i, M, K, Ns, rs))
            _check_f32(dB, dB_ref, ("group dB", i, M, K, Ns, rs))
        else:
            assert dA is None and dB is None
    again = qerl.nvfp4_lora_linear_backward_group(x.cuda(), dys, weights, As, Bs, scales_)
    assert torch.equal(dx, again[0])
    for (a0, b0), (a1, b1) in zip(grads, again[1]):
        assert (a0 is None and a1 is None) or (torch.equal(a0, a1) and torch.equal(b0, b1))
    # a group of one is the single call, bit for bit; dA_i depends on dY_i B_i alone, which both calls compute alike
    i = 0
    single = qerl.nvfp4_lora_linear_backward(x.cuda(), dys[i], weights[i], As[i], Bs[i], scales_[i])
    one = qerl.nvfp4_lora_linear_backward_group(x.cuda(), dys[:1], weights[:1], As[:1], Bs[:1], scales_[:1])
    assert torch.equal(one[0], single[0])
    if rs[i]:
        assert torch.equal(one[1][0][0], single[1]) and torch.equal(one[1][0][1], single[2])
        assert torch.equal(grads[i][0], single[1])
