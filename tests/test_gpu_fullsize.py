"""GPU parity at the benchmark's full sizes, in the launch plans the benchmark takes (7B shapes at 32 and 64
tokens; every 32B plan at 1, 16 and 128 tokens; 32B gate_proj at 4096 tokens), against the oracle on sampled
output rows.

The layer is separable over output rows, and a row's NVFP4 bytes depend on the rest of the tensor only through
the tensor scale (amax / 2688).  So the oracle quantises a sub-tensor made of the sampled rows plus the row that
holds the tensor maximum -- which gives exactly the bytes a whole-tensor quantisation gives those rows -- while the
GPU quantises and packs the whole tensor, and every plan (units per workgroup, K-ranges, in-launch LoRA
producers, the two-launch cut) is the one the full shape selects.  Every case runs twice on one workspace: the
second run must repeat the first bit for bit, which also shows that the control words were re-armed."""
import numpy as np
import pytest
import torch

import paper_2510_11696_amd as qerl
import qerl_synth as qs
from oracle import nvfp4_oracle as oracle
from tests import cases
from tests.gpu_util import bf16_ulp_distance, check_linear

pytestmark = pytest.mark.gpu


class FullMember:
    """One full-size linear: whole tensor quantised and packed on the GPU, sampled rows quantised by the oracle."""

    def __init__(self, name, N, K, r, seed, n_rows=160, keep_all=False):
        print("  building", name, N, K, r, flush=True)
        self.name, self.N, self.K, self.r = name, N, K, r
        W = cases.gaussian(N, K, seed)
        flat = int(np.abs(W).argmax())
        amax_row = flat // K
        rng = np.random.default_rng(seed + 1)
        self.rows = np.unique(np.concatenate([np.arange(32), np.arange(N - 32, N), rng.integers(0, N, size=n_rows)]))
        if keep_all:
            # the oracle quantises the whole tensor (half a minute for 27648 x 5120): needed where the oracle has to
            # produce every output of the layer, because the next operator of a composition reads them all
            self.codes_all, self.scales_all, ts = oracle.nvfp4_quantize(W)
            self.codes, self.scales, self.ts = self.codes_all[self.rows], self.scales_all[self.rows], ts
        else:
            sub = np.unique(np.concatenate([self.rows, [amax_row]]))
            codes, scales, ts = oracle.nvfp4_quantize(W[sub])
            keep = np.searchsorted(sub, self.rows)
            self.codes, self.scales, self.ts = codes[keep], scales[keep], ts
        Wg = torch.from_numpy(W).to(torch.bfloat16).cuda()
        del W
        gc, gs, gts = qerl.nvfp4_quantize(Wg)
        del Wg
        # the quantiser's own gate is bit-exactness; here the sampled rows must match the oracle's bytes as well
        rows_d = torch.from_numpy(self.rows).cuda()
        assert np.array_equal(gc[rows_d].cpu().numpy(), self.codes) and np.array_equal(gs[rows_d].cpu().numpy(), self.scales)
        assert np.float32(gts.item()) == self.ts
        self.pw = qerl.nvfp4_prepack(gc, gs, gts)
        del gc, gs
        self.A = self.B = None
        if r:
            self.A, self.B = qs.lora_pair(N, K, r, seed + 2)
            self.Ad, self.Bd = self.A.cuda(), self.B.cuda()
        else:
            self.Ad = self.Bd = None
        self.rows_d = rows_d

    def reference(self, x_f32, lora_scale, bias=None):
        return oracle.nvfp4_lora_linear(x_f32, self.codes, self.scales, self.ts,
                                        self.A.float().numpy() if self.r else None,
                                        self.B.float().numpy()[self.rows] if self.r else None, lora_scale,
                                        bias=None if bias is None else bias[self.rows])

    def reference_all(self, x_f32, lora_scale):
        """Every output row (keep_all members only)."""
        return oracle.nvfp4_lora_linear(x_f32, self.codes_all, self.scales_all, self.ts,
                                        self.A.float().numpy() if self.r else None,
                                        self.B.float().numpy() if self.r else None, lora_scale)

    def check(self, y, x_f32, lora_scale, what, slack=1e-3):
        check_linear(y[:, self.rows_d], self.reference(x_f32, lora_scale), what, slack=slack)


@pytest.fixture(scope="module")
def mlp_7b():
    H, I, r = 3584, 18944, 32
    return {"gate": FullMember("7b gate", I, H, r, 61001, keep_all=True), "up": FullMember("7b up", I, H, r, 61011, keep_all=True),
            "down": FullMember("7b down", H, I, r, 61021)}


@pytest.fixture(scope="module")
def block_32b():
    H, I, KV, r = 5120, 27648, 1024, 64
    return {"gate": FullMember("32b gate", I, H, r, 62001, keep_all=True), "up": FullMember("32b up", I, H, r, 62011, keep_all=True),
            "down": FullMember("32b down", H, I, r, 62021), "q": FullMember("32b q", H, H, r, 62031),
            "k": FullMember("32b k", KV, H, r, 62041), "v": FullMember("32b v", KV, H, r, 62051)}


def _normed_input(M, H, seed, fused, As):
    """The AQN RMSNorm in front of a group, as the benchmark launches it: fused with the adapters' down-projections up
    to 16 tokens, on its own beyond.  Returns (y on the device, y as float32 numpy, ts or None); y is held to one bf16
    unit of the oracle, t to fp32 summation error of the oracle's product of that y."""
    xin = qs.activations(M, H, seed)
    gain = qs.rms_gain(H, seed + 1)
    Z = qs.aqn_noise(H, 1e-2, seed + 2)
    ts = None
    if fused:
        y, ts = qerl.aqn_rmsnorm_lora_down(xin.cuda(), gain.cuda(), Z.cuda(), 1e-6, [A.cuda() for A in As])
    else:
        y = qerl.aqn_rmsnorm(xin.cuda(), gain.cuda(), Z.cuda(), 1e-6)
    torch.cuda.synchronize()
    ref_y = oracle.aqn_rmsnorm(xin.float().numpy(), gain.float().numpy(), Z.numpy(), 1e-6)
    assert bf16_ulp_distance(y, ref_y).max() <= 1
    y_np = y.float().cpu().numpy()
    if ts is not None:
        for A, t in zip(As, ts):
            a64 = A.float().numpy().astype(np.float64)
            t_ref = oracle.lora_down_projection(y_np, A.float().numpy())
            bound = 4 * H * 2.0 ** -24 * (np.abs(y_np.astype(np.float64)) @ np.abs(a64).T) + 1e-30
            assert (np.abs(t.cpu().numpy().astype(np.float64).sum(0) - t_ref) <= bound).all()
    return y, y_np, ts


def _group_twice(y, members, ts, lora_scale):
    M = y.shape[0]
    lib = qerl.load_library()
    ws = qerl.Workspace(lib.nvfp4_lora_linear_workspace_bytes(M, sum(m.N for m in members), members[0].K,
                                                             sum(m.r for m in members)))
    call = lambda: qerl.nvfp4_lora_linear_packed_group(y, [m.pw for m in members], [m.Ad for m in members],
                                                       [m.Bd for m in members], [lora_scale] * len(members),
                                                       workspace=ws, ts=ts)
    outs = [o.clone() for o in call()]
    again = call()
    torch.cuda.synchronize()
    assert all(torch.equal(p, q) for p, q in zip(outs, again)), "second run on the same workspace differs"
    return outs


def _single_twice(x, m, lora_scale):
    ws = qerl.Workspace(qerl.load_library().nvfp4_lora_linear_workspace_bytes(x.shape[0], m.N, m.K, m.r))
    out = qerl.nvfp4_lora_linear_packed(x, m.pw, m.Ad, m.Bd, lora_scale, workspace=ws).clone()
    again = qerl.nvfp4_lora_linear_packed(x, m.pw, m.Ad, m.Bd, lora_scale, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(out, again), "second run on the same workspace differs"
    return out


@pytest.mark.timeout(600)
@pytest.mark.parametrize("M", [32, 64, 128])
def test_7b_mlp_at_a_few_dozen_tokens_as_the_benchmark_launches_it(mlp_7b, M):
    """gate + up as one group (76 MB streamed: the adapters' down-projections run as the first workgroups of the
    launch) and down (K = 18944: K-splits and in-launch producers), r = 32, behind the stand-alone RMSNorm."""
    print("full-size 7B MLP,", M, "tokens", flush=True)
    g, u, d = mlp_7b["gate"], mlp_7b["up"], mlp_7b["down"]
    y, y_np, _ = _normed_input(M, 3584, 63000 + M, False, [])
    outs = _group_twice(y, [g, u], None, 2.0)
    g.check(outs[0], y_np, 2.0, ("7B gate", M))
    u.check(outs[1], y_np, 2.0, ("7B up", M))
    x_down = qs.activations(M, 18944, 63100 + M)
    out = _single_twice(x_down.cuda(), d, 2.0)
    d.check(out, x_down.float().numpy(), 2.0, ("7B down", M))


@pytest.mark.timeout(900)
@pytest.mark.parametrize("M", [1, 16, 128, 300])
def test_32b_mlp_as_the_benchmark_launches_it(block_32b, M):
    """32B gate + up (2 x 27648 x 5120: 1728 row tiles) as one group and down (5120 x 27648), r = 64.  From 96 tokens
    on the GEMM takes over: down's 40 column blocks split K over workgroups (partial sums added by a second launch)
    and carry the LoRA down-projection as the launch's first workgroups; 300 tokens: three token blocks, the last ragged."""
    print("full-size 32B MLP,", M, "tokens", flush=True)
    g, u, d = block_32b["gate"], block_32b["up"], block_32b["down"]
    y, y_np, ts = _normed_input(M, 5120, 64000 + M, M <= 16, [g.A, u.A])
    outs = _group_twice(y, [g, u], ts, 2.0)
    g.check(outs[0], y_np, 2.0, ("32B gate", M))
    u.check(outs[1], y_np, 2.0, ("32B up", M))
    x_down = qs.activations(M, 27648, 64100 + M)
    out = _single_twice(x_down.cuda(), d, 2.0)
    d.check(out, x_down.float().numpy(), 2.0, ("32B down", M))


@pytest.mark.timeout(600)
@pytest.mark.parametrize("M", [1, 16, 128, 300])
def test_32b_attention_projections_as_the_benchmark_launches_them(block_32b, M):
    """32B q + k + v (rank 64 each: six rank tiles for the fused norm) as one group, and a q-sized single
    linear standing in for o (same shape, its own input, in-launch LoRA producers)."""
    print("full-size 32B q+k+v,", M, "tokens", flush=True)
    q, k, v = block_32b["q"], block_32b["k"], block_32b["v"]
    y, y_np, ts = _normed_input(M, 5120, 65000 + M, M <= 16, [q.A, k.A, v.A])
    outs = _group_twice(y, [q, k, v], ts, 2.0)
    for m, o in zip((q, k, v), outs):
        m.check(o, y_np, 2.0, ("32B " + m.name, M))
    x_o = qs.activations(M, 5120, 65100 + M)
    out = _single_twice(x_o.cuda(), q, 2.0)
    q.check(out, x_o.float().numpy(), 2.0, ("32B o-shaped", M))


@pytest.mark.timeout(900)
def test_32b_gate_at_4096_tokens(block_32b):
    """The prefill GEMM at the largest token count of the benchmark: 32B gate_proj, 4096 tokens, r = 64."""
    M = 4096
    print("full-size 32B gate,", M, "tokens", flush=True)
    g = block_32b["gate"]
    x = qs.activations(M, 5120, 66001)
    out = _single_twice(x.cuda(), g, 2.0)
    g.check(out, x.float().numpy(), 2.0, ("32B gate", M))
    # gate + up grouped, as the benchmark's step launches them
    outs = _group_twice(x.cuda(), [g, block_32b["up"]], None, 2.0)
    g.check(outs[0], x.float().numpy(), 2.0, ("32B gate grouped", M))
    block_32b["up"].check(outs[1], x.float().numpy(), 2.0, ("32B up grouped", M))


def _bf16(a64):
    return oracle.round_to_bf16(a64).astype(np.float32)


def _fused_mlp_case(mem, M, H, seed):
    """The feed-forward block in ONE launch (norm, gate + up, SiLU-mul, down) on full-size weights, against the
    oracle's composition of the operators: the oracle computes every gate / up output (the down projection reads
    them all) and the sampled rows of down.  Twice on one workspace, second run bit-identical."""
    g, u, d = mem["gate"], mem["up"], mem["down"]
    xin = qs.activations(M, H, seed)
    gain = qs.rms_gain(H, seed + 1)
    Z = qs.aqn_noise(H, 1e-2, seed + 2)
    xn = _bf16(oracle.aqn_rmsnorm(xin.float().numpy(), gain.float().numpy(), Z.numpy(), 1e-6))
    act = oracle.silu_mul(_bf16(g.reference_all(xn, 2.0)), _bf16(u.reference_all(xn, 2.0))).astype(np.float32)
    ref = d.reference(act, 2.0)
    lib = qerl.load_library()
    ws = qerl.Workspace(lib.aqn_rmsnorm_nvfp4_lora_mlp_workspace_bytes(M, H, g.N, d.N, g.r, u.r, d.r))
    call = lambda: qerl.aqn_rmsnorm_nvfp4_lora_mlp(xin.cuda(), gain.cuda(), Z.cuda(), 1e-6, g.pw, u.pw, d.pw, (g.Ad, u.Ad, d.Ad),
                                                   (g.Bd, u.Bd, d.Bd), (2.0, 2.0, 2.0), workspace=ws)
    y = call().clone()
    again = call()
    torch.cuda.synchronize()
    assert qerl.workspace_status(ws) == 0
    assert torch.equal(y, again), "second run on the same workspace differs"
    # (composed operators: the device rounds the intermediate activations from fp32 sums, the oracle from fp64 ones)
    check_linear(y[:, d.rows_d], ref, ("fused MLP", M, H), slack=4e-3)


@pytest.mark.timeout(900)
@pytest.mark.parametrize("M", [1, 8, 16])
def test_32b_feed_forward_block_in_one_launch(block_32b, M):
    print("full-size 32B feed-forward block in one launch,", M, "tokens", flush=True)
    _fused_mlp_case(block_32b, M, 5120, 67000 + M)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("M", [8, 16])
def test_7b_feed_forward_block_in_one_launch(mlp_7b, M):
    print("full-size 7B feed-forward block in one launch,", M, "tokens", flush=True)
    _fused_mlp_case(mlp_7b, M, 3584, 67100 + M)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("M", [1, 16])
def test_32b_norm_and_attention_projections_in_one_launch(block_32b, M):
    """AQN RMSNorm + q + k + v of the 32B block as one launch of the block kernel."""
    print("full-size 32B norm + q + k + v in one launch,", M, "tokens", flush=True)
    q, k, v = block_32b["q"], block_32b["k"], block_32b["v"]
    H = 5120
    xin = qs.activations(M, H, 68000 + M)
    gain = qs.rms_gain(H, 68001 + M)
    Z = qs.aqn_noise(H, 1e-2, 68002 + M)
    xn = _bf16(oracle.aqn_rmsnorm(xin.float().numpy(), gain.float().numpy(), Z.numpy(), 1e-6))
    ws = qerl.Workspace(qerl.aqn_rmsnorm_nvfp4_lora_linear_group_workspace_bytes(M, H, [q.N, k.N, v.N], [q.r, k.r, v.r]))
    call = lambda: qerl.aqn_rmsnorm_nvfp4_lora_linear_group(xin.cuda(), gain.cuda(), Z.cuda(), 1e-6, [q.pw, k.pw, v.pw],
                                                            [q.Ad, k.Ad, v.Ad], [q.Bd, k.Bd, v.Bd], [2.0] * 3, workspace=ws)
    outs = [o.clone() for o in call()]
    again = call()
    torch.cuda.synchronize()
    assert qerl.workspace_status(ws) == 0
    assert all(torch.equal(p, q_) for p, q_ in zip(outs, again)), "second run on the same workspace differs"
    for m, o in zip((q, k, v), outs):
        m.check(o, xn, 2.0, ("32B fused " + m.name, M))
