"""Pins for the oracle's linear + LoRA and noisy RMSNorm (CPU only)."""
import math

import numpy as np
import pytest
import torch

import qerl_synth as qs
from oracle import nvfp4_oracle as o


def _tiny(N, K, M, r, seed):
    W = qs.weights(N, K, seed).float().numpy()
    x = qs.activations(M, K, seed + 1).float().numpy()
    A, B = qs.lora_pair(N, K, max(r, 1), seed + 2)
    A, B = A.float().numpy()[:r], B.float().numpy()[:, :r]
    return W, x, A, B


@pytest.mark.parametrize("N,K,M,r", [(5, 16, 1, 0), (8, 32, 3, 2), (3, 48, 2, 1)])
def test_linear_brute_force_python_loops(N, K, M, r):
    W, x, A, B = _tiny(N, K, M, r, seed=21)
    codes, scales, S32 = o.nvfp4_quantize(W)
    Wh = o.nvfp4_dequantize(codes, scales, S32)
    s = 2.0
    y = o.nvfp4_lora_linear(x, codes, scales, S32, A if r else None, B if r else None, s)
    assert y.shape == (M, N)
    for m in range(M):
        for n in range(N):
            acc = 0.0
            for k in range(K):
                acc += float(x[m, k]) * float(Wh[n, k])
            lo = 0.0
            for j in range(r):
                t = 0.0
                for k in range(K):
                    t += float(x[m, k]) * float(A[j, k])
                lo += t * float(B[n, j])
            want = acc + s * lo
            assert abs(y[m, n] - want) <= 1e-12 * (1 + abs(want))


def test_lora_down_projection_by_loops_one_hot_and_exact_integers():
    """t = x A^T, the inner factor of Eq. 2's low-rank branch: Python loops; a one-hot token reads out a
    column of A exactly; small-integer operands give exactly representable sums whatever the order."""
    W, x, A, B = _tiny(4, 48, 3, 3, seed=33)
    t = o.lora_down_projection(x, A)
    assert t.shape == (3, 3) and t.dtype == np.float64
    for m in range(3):
        for j in range(3):
            want = sum(float(x[m, k]) * float(A[j, k]) for k in range(48))
            assert abs(t[m, j] - want) <= 1e-13 * (1 + abs(want))
    x1 = np.zeros((1, 48), dtype=np.float32)
    x1[0, 17] = 1.0
    assert np.array_equal(o.lora_down_projection(x1, A)[0], A[:, 17].astype(np.float64))
    rng = np.random.default_rng(5)
    xi = rng.integers(-8, 9, size=(2, 32)).astype(np.float32)
    Ai = rng.integers(-8, 9, size=(5, 32)).astype(np.float32)
    assert np.array_equal(o.lora_down_projection(xi, Ai), (xi.astype(np.int64) @ Ai.astype(np.int64).T).astype(np.float64))
    # not transposed, not the outer factor: a [r, K] operand with r != M gives [M, r]
    assert o.lora_down_projection(xi, Ai).shape == (2, 5)


def test_one_hot_input_reads_out_a_weight_column():
    W, x, A, B = _tiny(6, 32, 1, 0, seed=5)
    codes, scales, S32 = o.nvfp4_quantize(W)
    Wh = o.nvfp4_dequantize(codes, scales, S32)
    for k in (0, 15, 16, 31):
        x1 = np.zeros((1, 32), dtype=np.float32)
        x1[0, k] = 1.0
        y = o.nvfp4_lora_linear(x1, codes, scales, S32)
        assert np.array_equal(y[0], Wh[:, k].astype(np.float64))


def test_dense_merge_equivalence_and_library_matmul():
    """x (W_hat + s B A)^T equals the two-branch form (Eq. 2); and with the
    weights dequantised the op is a textbook GEMM (torch.matmul, fp64)."""
    N, K, M, r = 24, 64, 5, 4
    W, x, A, B = _tiny(N, K, M, r, seed=8)
    codes, scales, S32 = o.nvfp4_quantize(W)
    y = o.nvfp4_lora_linear(x, codes, scales, S32, A, B, 2.0)
    Wh = torch.from_numpy(o.nvfp4_dequantize(codes, scales, S32)).double()
    merged = Wh + 2.0 * torch.from_numpy(B).double() @ torch.from_numpy(A).double()
    want = torch.from_numpy(x).double() @ merged.T
    assert np.allclose(y, want.numpy(), rtol=1e-12, atol=1e-13)
    y0 = o.nvfp4_lora_linear(x, codes, scales, S32)
    assert np.allclose(y0, (torch.from_numpy(x).double() @ Wh.T).numpy(), rtol=1e-13, atol=1e-14)
    # r = 0 and lora_scale = 0 both switch the branch off
    assert np.array_equal(y0, o.nvfp4_lora_linear(x, codes, scales, S32, A, B, 0.0))
    # fp32 accumulation variant stays within fp32 rounding of the fp64 one
    y32 = o.nvfp4_lora_linear(x, codes, scales, S32, A, B, 2.0, acc_dtype=np.float32)
    assert np.allclose(y32, y, rtol=1e-4, atol=1e-5)


def test_rmsnorm_plain_formula_and_library():
    M, H = 3, 96
    x = qs.activations(M, H, 31).float().numpy() * 3
    g = qs.rms_gain(H, 32).float().numpy()
    y = o.aqn_rmsnorm(x, g, None, eps=1e-6)
    for m in range(M):
        ms = sum(float(v) ** 2 for v in x[m]) / H
        for k in range(H):
            want = float(g[k]) * float(x[m, k]) / math.sqrt(ms + 1e-6)
            assert abs(y[m, k] - want) <= 1e-14 * (1 + abs(want))
    lib = torch.nn.functional.rms_norm(torch.from_numpy(x).double(), (H,),
                                       torch.from_numpy(g).double(), eps=1e-6)
    assert np.allclose(y, lib.numpy(), rtol=1e-13, atol=0)


def test_rmsnorm_noise_identities():
    """Appendix "Proof of Noise Sharing": RMSNorm_noise(x) = (Z/w + 1) (.) RMSNorm(x),
    and feeding it to a linear equals the clean norm times row-scaled weights."""
    M, H, N = 4, 64, 10
    x = qs.activations(M, H, 41).float().numpy()
    g = qs.rms_gain(H, 42).float().numpy()
    Z = qs.aqn_noise(H, 1e-2, 43).numpy()
    y_noise = o.aqn_rmsnorm(x, g, Z)
    y_clean = o.aqn_rmsnorm(x, g, None)
    factor = Z.astype(np.float64) / g.astype(np.float64) + 1.0
    assert np.allclose(y_noise, factor * y_clean, rtol=1e-13, atol=0)
    assert not np.allclose(y_noise, y_clean, rtol=1e-5, atol=0)
    W = qs.weights(N, H, 44).float().numpy()
    codes, scales, S32 = o.nvfp4_quantize(W)
    Wh = o.nvfp4_dequantize(codes, scales, S32).astype(np.float64)
    lhs = y_noise @ Wh.T
    rhs = y_clean @ (factor[None, :] * Wh).T
    assert np.allclose(lhs, rhs, rtol=1e-12, atol=1e-14)
    # eps sits inside the square root: an all-zero row maps to zero, not NaN
    z = o.aqn_rmsnorm(np.zeros((1, H), dtype=np.float32), g, Z)
    assert not z.any()
    # zero noise vector == no noise
    assert np.array_equal(o.aqn_rmsnorm(x, g, np.zeros(H, dtype=np.float32)), y_clean)


def test_bias_is_added_to_every_row_before_any_rounding():
    """A zero weight tensor leaves y = bias in every row; in general y(bias) - y(no bias) = bias to the
    last fp64 bit of the smaller term, LoRA or not."""
    W, x, A, B = _tiny(6, 32, 3, 2, 77)
    bias = np.array([0.5, -1.25, 3.0, 0.0, -0.0078125, 100.0], dtype=np.float32)
    codes0, scales0, ts0 = o.nvfp4_quantize(np.zeros_like(W))
    y0 = o.nvfp4_lora_linear(x, codes0, scales0, ts0, bias=bias)
    assert (y0 == bias[None, :].astype(np.float64)).all()
    codes, scales, ts = o.nvfp4_quantize(W)
    plain = o.nvfp4_lora_linear(x, codes, scales, ts, A, B, 2.0)
    with_bias = o.nvfp4_lora_linear(x, codes, scales, ts, A, B, 2.0, bias=bias)
    assert np.allclose(with_bias - plain, bias[None, :], rtol=0, atol=1e-12)
    assert with_bias.shape == plain.shape



# ---- SiLU(gate) (.) up, the input of the down projection -------------------------------------------------
def test_round_to_bf16_is_nearest_even_on_the_top_16_bits():
    r = o.round_to_bf16
    assert r(1.0) == 1.0 and r(-0.15625) == -0.15625                # representable values stay
    assert r(1.0 + 2.0 ** -8) == 1.0                                 # tie between 1 and 1 + 2^-7: even mantissa wins
    assert r(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6                 # tie between 1 + 2^-7 and 1 + 2^-6: even wins
    assert r(1.0 + 2.0 ** -8 + 2.0 ** -20) == 1.0 + 2.0 ** -7        # just above the tie
    v = np.array([0.1, -2.7, 1e-5, 123.456, 6.02e8])
    assert np.array_equal(r(r(v)), r(v))                             # idempotent
    assert np.all(np.abs(r(v) - v) <= np.abs(v) * 2.0 ** -8)         # half a unit in the last of 8 significant bits


def test_silu_mul_closed_forms_and_brute_force():
    import math
    z = np.zeros(4, dtype=np.float32)
    u = np.array([1.0, -2.0, 0.5, 3.0], dtype=np.float32)
    assert np.array_equal(o.silu_mul(z, u), np.zeros(4))                          # SiLU(0) = 0
    big = np.array([40.0, 64.0, 100.0], dtype=np.float32)
    one = np.ones(3, dtype=np.float32)
    assert np.array_equal(o.silu_mul(big, one), big.astype(np.float64))           # SiLU(g) -> g
    assert np.all(np.abs(o.silu_mul(-big, one)) < 1e-15)                               # SiLU(-g) -> -0
    # SiLU(g) - SiLU(-g) = g (sigma(g) + sigma(-g) = 1), up to the two bf16 roundings
    g = np.array([0.25, 0.5, 1.0, 2.0, 3.0, 5.0], dtype=np.float32)
    d = o.silu_mul(g, np.ones_like(g)) - o.silu_mul(-g, np.ones_like(g))
    assert np.all(np.abs(d - g) <= 2.0 ** -8 * g)
    # the minimum of SiLU is about -0.27846 at g = -1.27846
    assert abs(o.silu_mul(np.float32(-1.2784645), np.float32(1.0)) + 0.27846) < 2.0 ** -9
    # element by element against math.exp and an independent bf16 rounding through struct
    import struct

    def bf16(v):
        bits = struct.unpack("<I", struct.pack("<f", v))[0]
        bits = (bits + 0x7FFF + ((bits >> 16) & 1)) & 0xFFFF0000
        return struct.unpack("<f", struct.pack("<I", bits))[0]
    rng = np.random.default_rng(3)
    gs = [bf16(float(v)) for v in rng.standard_normal(200) * 3]
    us = [bf16(float(v)) for v in rng.standard_normal(200) * 2]
    got = o.silu_mul(np.array(gs, dtype=np.float32), np.array(us, dtype=np.float32))
    for gi, ui, yi in zip(gs, us, got):
        want = bf16(bf16(gi / (1.0 + math.exp(-gi))) * ui)
        assert yi == want, (gi, ui, yi, want)
    # the gate's sign decides the sign of SiLU; the product follows the usual sign rule
    assert o.silu_mul(np.float32(-1.0), np.float32(-1.0)) > 0 > o.silu_mul(np.float32(-1.0), np.float32(1.0))


# ---- backward pass ----------------------------------------------------------------------------------------
def _bwd_case(seed, M=3, N=20, K=32, r=8):
    rng = np.random.default_rng(seed)
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    codes, scales, ts = o.nvfp4_quantize(W)
    x = rng.standard_normal((M, K)).astype(np.float32)
    dy = rng.standard_normal((M, N)).astype(np.float32)
    A = (rng.standard_normal((r, K)) / r).astype(np.float32)
    B = (rng.standard_normal((N, r)) * 0.1).astype(np.float32)
    return x, dy, codes, scales, ts, A, B


def test_backward_is_the_adjoint_of_the_forward_map():
    """<dy, J v> = <J^T dy, v> for the three arguments the layer is (bi)linear in; the forward map is the pinned
    nvfp4_lora_linear.  y is linear in x, and linear in A (B fixed) and in B (A fixed): the directional
    derivatives are exact differences of forward values, no step size involved."""
    x, dy, codes, scales, ts, A, B = _bwd_case(1)
    s = 1.75
    f = lambda x_, A_, B_: o.nvfp4_lora_linear(x_, codes, scales, ts, A_, B_, s)
    dx, dA, dB = o.nvfp4_lora_linear_backward(x, dy, codes, scales, ts, A, B, s)
    rng = np.random.default_rng(2)
    vx = rng.standard_normal(x.shape).astype(np.float32)
    vA = rng.standard_normal(A.shape).astype(np.float32)
    vB = rng.standard_normal(B.shape).astype(np.float32)
    zero_x = np.zeros_like(x)
    assert np.isclose(np.sum(dy * (f(vx, A, B) - f(zero_x, A, B))), np.sum(dx * vx), rtol=1e-12)
    zA, zB = np.zeros_like(A), np.zeros_like(B)
    assert np.isclose(np.sum(dy * (f(x, vA, B) - f(x, zA, B))), np.sum(dA * vA), rtol=1e-11)
    assert np.isclose(np.sum(dy * (f(x, A, vB) - f(x, A, zB))), np.sum(dB * vB), rtol=1e-11)


def test_backward_entries_by_brute_force_and_special_cases():
    x, dy, codes, scales, ts, A, B = _bwd_case(3, M=2, N=5, K=16, r=3)
    s = 0.5
    W = o.nvfp4_dequantize(codes, scales, ts).astype(np.float64)
    dx, dA, dB = o.nvfp4_lora_linear_backward(x, dy, codes, scales, ts, A, B, s)
    M, K = x.shape
    N, r = B.shape
    for m in range(M):
        for k in range(K):
            want = sum(float(dy[m, n]) * (W[n, k] + s * sum(float(B[n, j]) * float(A[j, k]) for j in range(r))) for n in range(N))
            assert abs(dx[m, k] - want) <= 1e-12 * max(1.0, abs(want))
    for j in range(r):
        for k in range(K):
            want = s * sum(float(dy[m, n]) * float(B[n, j]) * float(x[m, k]) for m in range(M) for n in range(N))
            assert abs(dA[j, k] - want) <= 1e-12 * max(1.0, abs(want))
    for n in range(N):
        for j in range(r):
            want = s * sum(float(dy[m, n]) * sum(float(x[m, k]) * float(A[j, k]) for k in range(K)) for m in range(M))
            assert abs(dB[n, j] - want) <= 1e-12 * max(1.0, abs(want))
    # without an adapter: dx = dy W_hat, no LoRA gradients; with B = 0: dx has no LoRA term and dA = 0, dB != 0
    dx0, a0, b0 = o.nvfp4_lora_linear_backward(x, dy, codes, scales, ts)
    assert a0 is None and b0 is None and np.allclose(dx0, dy.astype(np.float64) @ W, rtol=1e-14)
    dx1, dA1, dB1 = o.nvfp4_lora_linear_backward(x, dy, codes, scales, ts, A, np.zeros_like(B), s)
    assert np.array_equal(dx1, dx0) and not dA1.any() and dB1.any()
    # finite differences of a quadratic loss L = |y|^2 / 2 (dL/dy = y): central differences are exact up to rounding
    y = o.nvfp4_lora_linear(x, codes, scales, ts, A, B, s)
    gx, gA, gB = o.nvfp4_lora_linear_backward(x, y.astype(np.float32), codes, scales, ts, A, B, s)
    L = lambda A_: 0.5 * np.sum(o.nvfp4_lora_linear(x, codes, scales, ts, A_, B, s) ** 2)
    h = np.float32(2.0 ** -6)
    E = np.zeros_like(A); E[1, 5] = h
    fd = (L(A + E) - L(A - E)) / (2 * float(h))
    yg = o.nvfp4_lora_linear_backward(x, y.astype(np.float32), codes, scales, ts, A, B, s)[1][1, 5]
    assert abs(fd - yg) <= 1e-4 * max(1.0, abs(fd))      # y was rounded to fp32 for the call: not bit-exact



def _bwd_group(seed, M=3, K=32, Ns=(20, 8, 12), rs=(8, 0, 4)):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((M, K)).astype(np.float32)
    members = []
    for N, r in zip(Ns, rs):
        W = (rng.standard_normal((N, K)) * rng.uniform(0.01, 0.1)).astype(np.float32)   # members with different tensor scales
        codes, scales, ts = o.nvfp4_quantize(W)
        mem = {"dy": rng.standard_normal((M, N)).astype(np.float32), "codes": codes, "scales": scales, "tensor_scale": ts}
        if r:
            mem.update(A=(rng.standard_normal((r, K)) / r).astype(np.float32), B=(rng.standard_normal((N, r)) * 0.1).astype(np.float32),
                       lora_scale=float(rng.uniform(0.5, 2.0)))
        members.append(mem)
    return x, members


def _group_forward(x, mem, A=None, B=None):
    A = mem.get("A") if A is None else A
    B = mem.get("B") if B is None else B
    return o.nvfp4_lora_linear(x, mem["codes"], mem["scales"], mem["tensor_scale"], A, B, mem.get("lora_scale", 0.0))


def test_group_backward_is_the_adjoint_of_the_stacked_forward_map():
    """The group's forward map x -> (y_1, .., y_n) is linear in x: <(dy_i), J v> = <dx, v> with the pinned forward
    linears, for several directions (a dropped member, a missing LoRA term or a wrong scale breaks it); each
    member's dA_i, dB_i are the adjoints of its own (bi)linear maps; a loss through one member only (the other
    dy_i zero) gives that member's single-linear dx."""
    x, members = _bwd_group(5)
    dx, grads = o.nvfp4_lora_linear_backward_group(x, members)
    rng = np.random.default_rng(6)
    for _ in range(3):
        v = rng.standard_normal(x.shape).astype(np.float32)
        lhs = sum(np.sum(m["dy"] * (_group_forward(v, m) - _group_forward(np.zeros_like(v), m))) for m in members)
        assert np.isclose(lhs, np.sum(dx * v), rtol=1e-11)
    for m, (dA, dB) in zip(members, grads):
        if "A" not in m:
            assert dA is None and dB is None
            continue
        vA = rng.standard_normal(m["A"].shape).astype(np.float32)
        vB = rng.standard_normal(m["B"].shape).astype(np.float32)
        dyi = m["dy"]
        assert np.isclose(np.sum(dyi * (_group_forward(x, m, A=vA) - _group_forward(x, m, A=np.zeros_like(vA)))), np.sum(dA * vA), rtol=1e-11)
        assert np.isclose(np.sum(dyi * (_group_forward(x, m, B=vB) - _group_forward(x, m, B=np.zeros_like(vB)))), np.sum(dB * vB), rtol=1e-11)
    # one member's loss alone
    for i, m in enumerate(members):
        only = [dict(mm, dy=(mm["dy"] if j == i else np.zeros_like(mm["dy"]))) for j, mm in enumerate(members)]
        dxi, gi = o.nvfp4_lora_linear_backward_group(x, only)
        single = o.nvfp4_lora_linear_backward(x, m["dy"], m["codes"], m["scales"], m["tensor_scale"], m.get("A"), m.get("B"), m.get("lora_scale", 0.0))
        assert np.allclose(dxi, single[0], rtol=1e-13, atol=1e-15)
        for j, (a, b) in enumerate(gi):
            if j != i and a is not None:
                assert not a.any() and not b.any()


def test_group_backward_entries_by_brute_force():
    x, members = _bwd_group(8, M=2, K=16, Ns=(5, 3), rs=(3, 2))
    dx, grads = o.nvfp4_lora_linear_backward_group(x, members)
    Ws = [o.nvfp4_dequantize(m["codes"], m["scales"], m["tensor_scale"]).astype(np.float64) for m in members]
    for mrow in range(x.shape[0]):
        for k in range(x.shape[1]):
            want = 0.0
            for m, W in zip(members, Ws):
                N, r = m["B"].shape
                want += sum(float(m["dy"][mrow, n]) * (W[n, k] + m["lora_scale"] * sum(float(m["B"][n, j]) * float(m["A"][j, k]) for j in range(r)))
                            for n in range(N))
            assert abs(dx[mrow, k] - want) <= 1e-12 * max(1.0, abs(want))
