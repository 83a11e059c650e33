"""CPU-side checks of the boundary: the library loads, exports every symbol the
header declares, and rejects misuse on the host before touching a GPU."""
import ctypes
import os
import re

import pytest

import paper_2510_11696_amd as qerl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(qerl.LIB_PATH):
        from paper_2510_11696_amd import build
        build.build(verbose=False)
    return qerl.load_library()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "qerl_nvfp4.h")).read()
    declared = re.findall(r"QERL_API\s+[\w\s\*]+?\b(\w+)\s*\(", header)
    assert len(declared) >= 10
    for name in declared:
        assert hasattr(lib, name), name
    assert set(declared) == set(qerl.EXPORTED_SYMBOLS)


def test_status_strings(lib):
    for code in range(0, -7, -1):
        assert lib.qerl_status_string(code)
        assert b"unknown" not in lib.qerl_status_string(code)
    assert b"unknown" in lib.qerl_status_string(-99)


def test_error_word_decoding_and_status_call_validation(lib):
    """The sticky word of the control region: zero is fine, any bit a kernel's abandoned wait sets (stage boundary,
    LoRA hand-over, another kernel's hand-over) reads as QERL_ERR_TIMEOUT; the host rejects bad arguments first."""
    assert lib.qerl_status_from_error_word(0) == 0
    for word in (1, 2, 4, 7, 0x80000000):
        assert lib.qerl_status_from_error_word(word) == -6
    assert b"wait" in lib.qerl_status_string(-6) or b"time" in lib.qerl_status_string(-6).lower()
    assert lib.qerl_workspace_status(None, None) == -1
    assert lib.qerl_workspace_status(0x10010, None) == -3
    assert lib.qerl_selftest_wait_gives_up(None, 1 << 20, 4, None) == -1
    assert lib.qerl_selftest_wait_gives_up(0x10000, 64, 4, None) == -4          # smaller than the control region
    assert lib.qerl_selftest_wait_gives_up(0x10000, 1 << 20, 0, None) == -2
    assert lib.qerl_selftest_wait_gives_up(0x10000, 1 << 20, 1 << 20, None) == -2  # no long spins on request


def test_sigma_schedule_host(lib):
    assert qerl.aqn_sigma(0, 10, 1e-2, 5e-4) == 0.0
    assert qerl.aqn_sigma(1, 10, 1e-2, 5e-4) == 1e-2
    assert abs(qerl.aqn_sigma(10, 10, 1e-2, 5e-4) - 5e-4) < 1e-18
    assert qerl.aqn_sigma(11, 10, 1e-2, 5e-4) != qerl.aqn_sigma(11, 10, 1e-2, 5e-4)   # NaN


def test_host_side_validation_needs_no_gpu(lib):
    p = ctypes.c_void_p
    fake = 0x10000   # aligned, never dereferenced: every call below fails validation first
    q = lib.nvfp4_quantize
    assert q(None, 4, 32, 32, fake, fake, None, fake, 1 << 20, None) == -1
    assert q(fake, 4, 24, 24, fake, fake, fake, fake, 1 << 20, None) == -2      # K % 16
    assert q(fake, 4, 32, 16, fake, fake, fake, fake, 1 << 20, None) == -2      # ldw < K
    assert q(fake, -1, 32, 32, fake, fake, fake, fake, 1 << 20, None) == -2
    assert q(None, 4, 32, 32, fake, fake, fake, fake, 1 << 20, None) == -1
    assert q(fake + 2, 4, 32, 32, fake, fake, fake, fake, 1 << 20, None) == -3
    assert q(fake, 4, 32, 36, fake, fake, fake, fake, 1 << 20, None) == -3      # ldw % 8
    assert q(fake, 4, 32, 32, fake, fake, fake, fake, 16, None) == -4
    assert q(fake, 4, 32, 32, fake, fake, fake, None, 1 << 20, None) == -4

    lin = lib.nvfp4_lora_linear
    ok = dict(x=fake, M=2, K=64, ldx=64, codes=fake, scales=fake, ts=fake, N=16, A=None, B=None, r=0,
              ls=0.0, y=fake, ldy=16, ws=fake, wsb=1 << 24, st=None)

    def call(**kw):
        a = dict(ok, **kw)
        return lin(a["x"], a["M"], a["K"], a["ldx"], a["codes"], a["scales"], a["ts"], a["N"], a["A"],
                   a["B"], a["r"], a["ls"], a["y"], a["ldy"], a["ws"], a["wsb"], a["st"])
    assert call(M=0) == 0                       # no-op, nothing launched
    assert call(K=40, ldx=40) == -2
    assert call(M=-1) == -2
    assert call(ldx=32) == -2
    assert call(ldy=8) == -2
    assert call(r=-1) == -2
    assert call(x=None) == -1
    assert call(codes=None) == -1
    assert call(r=8) == -1                      # A/B missing
    assert call(x=fake + 1) == -3
    assert call(r=8, A=fake + 1, B=fake) == -3
    assert call(ws=None) == -4
    assert call(wsb=64) == -4
    assert call(ws=fake + 16) == -4
    need = qerl.nvfp4_lora_linear_workspace_bytes(2, 16, 64, 0)
    assert call(wsb=need - 1) == -4

    rn = lib.aqn_rmsnorm
    assert rn(None, 1, 64, 64, fake, None, 1e-6, fake, 64, None) == -1
    assert rn(fake, 1, 0, 64, fake, None, 1e-6, fake, 64, None) == -2
    assert rn(fake, 1, 64, 32, fake, None, 1e-6, fake, 64, None) == -2
    assert rn(fake, 0, 64, 64, fake, None, 1e-6, fake, 64, None) == 0
    assert lib.qerl_workspace_init(None, 1024, None) == -1
    assert lib.qerl_workspace_init(fake + 4, 1024, None) == -3
    assert lib.nvfp4_dequantize(fake, fake, fake, 2, 24, fake, None) == -2


def test_host_side_validation_of_the_mx_linears(lib):
    fake = 0x10000
    f = ctypes.c_float(1.0)
    ok_ws = 1 << 30
    # plain variant
    assert lib.mxfp4_linear_native(fake, 4, 48, 48, fake, 8, fake, 8, fake, ok_ws, None) == -2      # K % 32
    assert lib.mxfp4_linear_native(fake, 4, 64, 64, None, 8, fake, 8, fake, ok_ws, None) == -1
    assert lib.mxfp4_linear_native(fake, 4, 64, 68, fake, 8, fake, 8, fake, ok_ws, None) == -3      # ldx % 8
    assert lib.mxfp4_linear_native(fake, 4, 64, 64, fake, 8, fake, 8, fake, 16, None) == -4
    assert lib.mxfp4_linear_native(fake, 0, 64, 64, fake, 8, fake, 8, None, 0, None) == 0
    # with the LoRA branch and bias
    call = lambda r, A=fake, B=fake, bias=None, ws=fake, wsb=ok_ws, K=64: lib.mxfp4_lora_linear_native(
        fake, 4, K, K, fake, 8, A, B, r, f, bias, fake, 8, ws, wsb, None)
    assert call(12) == -2 and call(136) == -2 and call(-8) == -2        # rank: a multiple of 8, at most 128
    assert call(8, K=48) == -2
    assert call(8, A=None) == -1 and call(8, B=None) == -1
    assert call(8, A=fake + 8) == -3 and call(8, B=fake + 2) == -3 and call(0, bias=fake + 1) == -3
    assert call(8, ws=None) == -4 and call(8, wsb=1024) == -4 and call(8, ws=fake + 64) == -4
    assert call(0, A=None, B=None, wsb=lib.mxfp4_lora_linear_native_workspace_bytes(4, 8, 64, 0) - 1) == -4
    for M in (1, 32, 33, 4096):
        for r in (0, 32, 128):
            assert lib.mxfp4_lora_linear_native_workspace_bytes(M, 5120, 5120, r) >= lib.mxfp4_linear_native_workspace_bytes(M, 5120, 5120)
    assert lib.mxfp4_lora_linear_native_workspace_bytes(8, 64, 128, 136) == 0
    assert lib.mxfp4_lora_linear_native_workspace_bytes(8, 64, 128, 32) < (32 << 20)


def test_binding_refuses_cpu_tensors():
    import torch
    with pytest.raises(TypeError):
        qerl.nvfp4_quantize(torch.zeros((2, 32), dtype=torch.bfloat16))
    with pytest.raises(TypeError):
        qerl.aqn_rmsnorm(torch.zeros((2, 32), dtype=torch.bfloat16), torch.ones(32, dtype=torch.bfloat16))


def test_workspace_size_is_monotone_enough(lib):
    f = qerl.nvfp4_lora_linear_workspace_bytes
    assert f(8, 3584, 18944, 32) >= f(8, 3584, 3584, 32)
    assert f(128, 3584, 3584, 32) >= f(8, 3584, 3584, 32)
    assert f(8, 3584, 18944, 32) < 64 << 20


def test_sigma_schedules_match_the_oracle():
    from oracle import nvfp4_oracle as oracle
    for kind in oracle.SCHEDULE_KINDS:
        for K in (1, 2, 10):
            for k in range(K + 1):
                got = qerl.aqn_sigma_schedule(kind, k, K, 1e-2, 5e-4)
                want = oracle.aqn_sigma_schedule(kind, k, K, 1e-2, 5e-4)
                assert abs(got - want) <= 1e-17, (kind, K, k, got, want)
        bad = qerl.aqn_sigma_schedule(kind, 11, 10, 1e-2, 5e-4)
        assert bad != bad   # NaN


def test_host_side_validation_of_the_fused_entry_points(lib):
    """Group linear, fused norm + LoRA-down, packed linear and noise fill: every call fails validation on the
    host (or is a no-op) before anything could be launched, so none of the fake pointers is ever dereferenced."""
    from paper_2510_11696_amd.binding import _LinearDesc
    fake = 0x10000
    grp = lib.nvfp4_lora_linear_packed_group
    d = (_LinearDesc * 5)()
    for i in range(5):
        d[i] = _LinearDesc(fake, fake, 32, None, None, 0, 0.0, fake, 32, None, None)
    dp = ctypes.cast(d, ctypes.c_void_p)
    big = 1 << 26
    assert grp(fake, 2, 64, 64, None, 1, fake, big, None) == -1            # no descriptors
    assert grp(fake, 2, 64, 64, dp, 0, fake, big, None) == -2               # 0 members
    assert grp(fake, 2, 64, 64, dp, 5, fake, big, None) == -2               # more than 4
    assert grp(fake, 0, 64, 64, dp, 2, fake, big, None) == 0                # no tokens: no-op
    assert grp(fake + 2, 2, 64, 64, dp, 2, fake, big, None) == -3           # x not 16-byte aligned
    assert grp(fake, 2, 64, 68, dp, 2, fake, big, None) == -3               # ldx % 8
    assert grp(fake, 2, 64, 64, dp, 2, None, big, None) == -4
    assert grp(fake, 2, 64, 64, dp, 2, fake, 64, None) == -4
    d[1].ldy = 16                                                            # ldy < N
    assert grp(fake, 2, 64, 64, dp, 2, fake, big, None) == -2
    d[1].ldy = 32
    d[1].r = 8                                                               # rank without A / B
    assert grp(fake, 2, 64, 64, dp, 2, fake, big, None) == -1
    d[1].A = fake; d[1].B = fake; d[1].t = fake + 4                          # precomputed t not 32-byte aligned
    assert grp(fake, 2, 64, 64, dp, 2, fake, big, None) == -3

    pk = lib.nvfp4_lora_linear_packed
    assert pk(fake, 0, 64, 64, fake, fake, 16, None, None, 0, 0.0, fake, 16, fake, big, None) == 0
    assert pk(fake, 2, 64, 64, fake + 8, fake, 16, None, None, 0, 0.0, fake, 16, fake, big, None) == -3
    assert pk(fake, 2, 0, 0, fake, fake, 16, None, None, 0, 0.0, fake, 16, fake, big, None) == -2
    assert lib.nvfp4_prepack(fake, fake, 4, 24, fake, None) == -2
    assert lib.nvfp4_prepack(fake, fake, 4, 32, fake + 4, None) == -3
    assert lib.nvfp4_prepack(None, fake, 4, 32, fake, None) == -1
    assert lib.nvfp4_prepack(fake, fake, 0, 32, fake, None) == 0
    assert lib.nvfp4_prepack_bytes(33, 130) == 2 * 2 * 2304 and lib.nvfp4_prepack_bytes(0, 64) == 0

    sw = lib.nvfp4_lora_linear_packed_swiglu
    assert sw(fake, fake, 0, 64, 64, 64, fake, fake, 16, None, None, 0, 0.0, fake, 16, fake, big, None) == 0
    assert sw(fake, None, 2, 64, 64, 64, fake, fake, 16, None, None, 0, 0.0, fake, 16, fake, big, None) == -1   # no up
    assert sw(fake, fake, 2, 64, 64, 32, fake, fake, 16, None, None, 0, 0.0, fake, 16, fake, big, None) == -2   # ldu < K
    assert sw(fake, fake + 2, 2, 64, 64, 64, fake, fake, 16, None, None, 0, 0.0, fake, 16, fake, big, None) == -3
    assert sw(fake, fake, 2, 64, 64, 68, fake, fake, 16, None, None, 0, 0.0, fake, 16, fake, big, None) == -3   # ldu % 8
    need = lib.nvfp4_lora_linear_swiglu_workspace_bytes(40, 16, 64, 0)
    assert need >= qerl.nvfp4_lora_linear_workspace_bytes(40, 16, 64, 0) + 40 * 64 * 2
    assert sw(fake, fake, 40, 64, 64, 64, fake, fake, 16, None, None, 0, 0.0, fake, 16, fake, need - 256, None) == -4

    bw = lib.nvfp4_lora_linear_backward
    okb = dict(x=fake, dy=fake, M=4, K=64, N=32, ldx=64, lddy=32, pt=fake, ts=fake, A=fake, B=fake, r=8, s=1.0,
               dx=fake, lddx=64, dA=fake, dB=fake, ws=fake, wsb=big)

    def callb(**kw):
        a = dict(okb, **kw)
        return bw(a["x"], a["dy"], a["M"], a["K"], a["N"], a["ldx"], a["lddy"], a["pt"], a["ts"], a["A"], a["B"], a["r"],
                  a["s"], a["dx"], a["lddx"], a["dA"], a["dB"], a["ws"], a["wsb"], None)
    assert callb(M=0) == 0
    assert callb(K=40, ldx=40, lddx=40) == -2            # K % 16
    assert callb(N=30, lddy=32) == -2                    # N % 8
    assert callb(r=72) == -2 and callb(r=12) == -2       # rank above 64 / not a multiple of 8
    assert callb(lddx=32) == -2 and callb(lddy=16) == -2
    assert callb(dy=None) == -1 and callb(dx=None) == -1 and callb(pt=None) == -1
    assert callb(dA=None) == -1 and callb(x=None) == -1
    assert callb(r=0, x=None, A=None, B=None, dA=None, dB=None, ws=None) == -4   # r = 0 needs no x / A / B, but a workspace
    assert callb(dy=fake + 2) == -3 and callb(lddy=36) == -3 and callb(A=fake + 8) == -3
    assert callb(wsb=64) == -4 and callb(ws=fake + 16) == -4
    assert lib.nvfp4_prepack_t_bytes(33, 130) == 5 * 1 * 2304 and lib.nvfp4_prepack_t_bytes(0, 64) == 0
    assert lib.nvfp4_prepack_t(fake, fake, 4, 24, fake, None) == -2
    assert lib.nvfp4_prepack_t(fake, fake, 4, 32, fake + 4, None) == -3
    assert lib.nvfp4_prepack_t(None, fake, 4, 32, fake, None) == -1
    assert lib.nvfp4_lora_linear_backward_workspace_bytes(2048, 13824, 5120, 64) < 64 << 20

    # the grouped form: a HOST array of descriptors
    from paper_2510_11696_amd.binding import _BackwardDesc
    bg = lib.nvfp4_lora_linear_backward_group

    def group(n=2, M=4, K=64, ldx=64, lddx=64, x=fake, dx=fake, ws=fake, wsb=big, edit=None):
        descs = (_BackwardDesc * max(n, 1))()
        for d in descs:
            d.dy, d.lddy, d.N, d.packed_t, d.tensor_scale = fake, 32, 32, fake, fake
            d.A, d.B, d.r, d.lora_scale, d.dA, d.dB = fake, fake, 8, 1.0, fake, fake
        if edit:
            edit(descs)
        return bg(x, M, K, ldx, ctypes.cast(descs, ctypes.c_void_p), n, dx, lddx, ws, wsb, None), descs
    assert group(M=0)[0] == 0
    assert group(n=0)[0] == -2 and group(n=5)[0] == -2
    assert bg(fake, 4, 64, 64, None, 2, fake, 64, fake, big, None) == -1
    assert group(K=40, ldx=40, lddx=40)[0] == -2 and group(lddx=32)[0] == -2
    assert group(edit=lambda d: setattr(d[1], "N", 30))[0] == -2           # N % 8 of the second member
    assert group(edit=lambda d: setattr(d[1], "r", 72))[0] == -2
    assert group(edit=lambda d: setattr(d[1], "dy", None))[0] == -1 and group(edit=lambda d: setattr(d[0], "dB", None))[0] == -1
    assert group(x=None)[0] == -1 and group(dx=None)[0] == -1
    assert group(edit=lambda d: setattr(d[1], "A", fake + 8))[0] == -3 and group(edit=lambda d: setattr(d[1], "lddy", 36))[0] == -3
    assert group(wsb=64)[0] == -4 and group(ws=fake + 16)[0] == -4

    def no_adapters(d):
        for e in d:
            e.A = e.B = e.dA = e.dB = None
            e.r = 0
    assert group(x=None, ws=None, edit=no_adapters)[0] == -4                  # no adapter anywhere: x is not read; a workspace still is
    _, descs = group()
    gb = lib.nvfp4_lora_linear_backward_group_workspace_bytes
    assert gb(4, 64, ctypes.cast(descs, ctypes.c_void_p), 0) == 0 and gb(4, 64, None, 2) == 0
    one = gb(2048, 5120, ctypes.cast(descs, ctypes.c_void_p), 1)
    assert one == lib.nvfp4_lora_linear_backward_workspace_bytes(2048, 32, 5120, 8)
    assert one < gb(2048, 5120, ctypes.cast(descs, ctypes.c_void_p), 2) < 2 * one

    nd = lib.aqn_rmsnorm_lora_down
    A = (ctypes.c_void_p * 5)(*([fake] * 5)); T = (ctypes.c_void_p * 5)(*([fake] * 5))
    R = (ctypes.c_int64 * 5)(32, 32, 32, 32, 32)
    ap, tp, rp = (ctypes.cast(v, ctypes.c_void_p) for v in (A, T, R))
    assert nd(fake, 17, 64, 64, fake, None, 1e-6, fake, 64, ap, rp, tp, 1, None) == -2     # more than 16 tokens
    assert nd(fake, 2, 72, 72, fake, None, 1e-6, fake, 72, ap, rp, tp, 1, None) == -2      # H % 16
    assert nd(fake, 2, 16384, 16384, fake, None, 1e-6, fake, 16384, ap, rp, tp, 1, None) == -2
    assert nd(fake, 2, 64, 64, fake, None, 1e-6, fake, 64, ap, rp, tp, 0, None) == -2
    assert nd(fake, 2, 64, 64, fake, None, 1e-6, fake, 64, ap, rp, tp, 5, None) == -2
    assert nd(fake, 2, 64, 64, None, None, 1e-6, fake, 64, ap, rp, tp, 1, None) == -1
    assert nd(fake, 2, 64, 64, fake, None, 1e-6, fake, 64, None, rp, tp, 1, None) == -1
    assert nd(fake + 2, 2, 64, 64, fake, None, 1e-6, fake, 64, ap, rp, tp, 1, None) == -3
    R[0] = 12                                                                              # rank not a multiple of 8
    assert nd(fake, 2, 64, 64, fake, None, 1e-6, fake, 64, ap, rp, tp, 1, None) == -2
    R[0] = 72
    assert nd(fake, 2, 64, 64, fake, None, 1e-6, fake, 64, ap, rp, tp, 1, None) == -2
    R[0] = 32
    assert nd(fake, 0, 64, 64, fake, None, 1e-6, fake, 64, ap, rp, tp, 1, None) == 0

    nf = lib.aqn_noise_fill
    assert nf(None, 0, 1e-2, 1, 1, None) == 0
    assert nf(None, 8, 1e-2, 1, 1, None) == -1
    assert nf(fake, -1, 1e-2, 1, 1, None) == -2
    assert nf(fake, 8, -1e-2, 1, 1, None) == -2
    assert nf(fake, 8, float("inf"), 1, 1, None) == -2
    assert nf(fake + 2, 8, 1e-2, 1, 1, None) == -3



def test_fused_launch_plans_exist_for_a_grid_of_shapes(lib):
    """Host logic of the persistent decode kernel: for every shape of a grid the planner (K-ranges, phases, LoRA
    producers, LDS layout of the union of the stages) finds a plan that also passes the launch's own validation --
    the sizing calls run both and return 0 otherwise.  No GPU is touched."""
    bad = []
    for M in (1, 2, 7, 8, 9, 15, 16):
        for H in (128, 512, 1040, 2048, 3584, 4096, 5120, 8192):
            for I in (64, 640, 2368, 4096, 13824, 18944, 27648):
                for r in (0, 8, 16, 64):
                    if lib.aqn_rmsnorm_nvfp4_lora_mlp_workspace_bytes(M, H, I, H, r, r, r) == 0:
                        bad.append(("mlp", M, H, I, r))
            for Ns in ((64,), (5120, 1024, 1024), (3584, 512, 512), (96, 40), (27648, 27648), (152064,)):
                for r in (0, 32, 64):
                    if qerl.aqn_rmsnorm_nvfp4_lora_linear_group_workspace_bytes(M, H, list(Ns), [r] * len(Ns)) == 0:
                        bad.append(("group", M, H, Ns, r))
    assert not bad, bad[:10]
    # what the kernel does not take is refused in the sizing call already
    assert lib.aqn_rmsnorm_nvfp4_lora_mlp_workspace_bytes(8, 512, 1024, 512, 12, 12, 12) == 0     # rank not a multiple of 8
    assert lib.aqn_rmsnorm_nvfp4_lora_mlp_workspace_bytes(8, 512, 1028, 512, 8, 8, 8) == 0        # gate rows not a multiple of 8
    assert lib.aqn_rmsnorm_nvfp4_lora_mlp_workspace_bytes(8, 520, 1024, 512, 8, 8, 8) == 0        # K not a multiple of 16
    # beyond 16 tokens the entry points compose the separate launches: their workspaces add up
    assert lib.aqn_rmsnorm_nvfp4_lora_mlp_workspace_bytes(64, 3584, 18944, 3584, 32, 32, 32) > 0
