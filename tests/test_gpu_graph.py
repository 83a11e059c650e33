"""Every launch sequence of the path recorded into a HIP graph and replayed: each replay, with eager work and
synchronisations between the replays, reproduces the eager result bit for bit. The eager results themselves are
held to the oracle by the other GPU tests; what is checked here is that the launches carry no state a replay
breaks (progress words, exchange counters and staging areas in the workspace are re-armed by the kernels)."""
import pytest
import torch

import paper_2510_11696_amd as qerl

pytestmark = pytest.mark.gpu

REPLAYS = 5


def _weights(N, K, r, gen, transposed=False):
    codes = torch.randint(0, 256, (N, K // 2), device="cuda", dtype=torch.uint8, generator=gen)
    scales = torch.randint(0x30, 0x48, (N, K // 16), device="cuda", dtype=torch.uint8, generator=gen)
    ts = torch.tensor([2e-4], device="cuda")
    A = (torch.randn((r, K), device="cuda", generator=gen) / r).to(torch.bfloat16)
    B = (torch.randn((N, r), device="cuda", generator=gen) * 0.02).to(torch.bfloat16)
    pack = qerl.nvfp4_prepack_t if transposed else qerl.nvfp4_prepack
    return pack(codes, scales, ts), A, B


def _replays_match(run, results):
    """run() launches on the current stream and returns nothing; results() lists the tensors it writes."""
    run()
    torch.cuda.synchronize()
    want = [t.clone() for t in results()]
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        run()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph):
            run()
    torch.cuda.synchronize()
    recorded = results()                        # what the recorded launches write (run() may allocate its outputs)
    for rep in range(REPLAYS):
        for t in recorded:
            t.fill_(float("nan")) if t.is_floating_point() else t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, (a, b) in enumerate(zip(want, recorded)):
            assert torch.equal(a, b), ("replay", rep, "tensor", i)
        run()                                   # the program's own eager work between the replays
        torch.cuda.synchronize()


# 8: the streaming kernel; 40: the mid kernel behind a launch of the LoRA down-projection; 128: the mid kernel with
# the down-projection's workgroups inside its own launch; 300: the grouped GEMM
@pytest.mark.parametrize("M", [8, 40, 128, 300])
def test_mlp_block_launches_replay_like_eager(M):
    print("graph case: mlp block, M =", M, flush=True)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(50 + M)
    H, I, r = 1024, 2816, 32
    gate, up, down = _weights(I, H, r, gen), _weights(I, H, r, gen), _weights(H, I, r, gen)
    x = torch.randn((M, H), device="cuda", generator=gen).to(torch.bfloat16)
    gain = (1.0 + 0.1 * torch.randn(H, device="cuda", generator=gen)).to(torch.bfloat16)
    noise = 0.01 * torch.randn(H, device="cuda", generator=gen)
    lib = qerl.load_library()
    ws = qerl.Workspace(max(qerl.nvfp4_lora_linear_workspace_bytes(M, 2 * I, H, 2 * r),
                            lib.nvfp4_lora_linear_swiglu_workspace_bytes(M, H, I, r)))
    xn = torch.empty_like(x)
    outs = [torch.empty((M, I), device="cuda", dtype=torch.bfloat16) for _ in range(2)]
    y = torch.empty((M, H), device="cuda", dtype=torch.bfloat16)

    def run():
        qerl.aqn_rmsnorm(x, gain, noise, 1e-6, out=xn)
        qerl.nvfp4_lora_linear_packed_group(xn, [gate[0], up[0]], [gate[1], up[1]], [gate[2], up[2]], [2.0, 2.0],
                                            workspace=ws, outs=outs)
        qerl.nvfp4_lora_linear_packed_swiglu(outs[0], outs[1], down[0], down[1], down[2], 2.0, workspace=ws, out=y)

    _replays_match(run, lambda: [xn, outs[0], outs[1], y])


# the persistent multi-stage kernel: its stage boundary, hand-over words and K-range counters live in the workspace
# and are re-armed by the launch itself
@pytest.mark.parametrize("M", [1, 8, 16])
def test_fused_block_launches_replay_like_eager(M):
    print("graph case: fused launches, M =", M, flush=True)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(70 + M)
    H, I, r = 2048, 2816, 32
    gate, up, down = _weights(I, H, r, gen), _weights(I, H, r, gen), _weights(H, I, r, gen)
    q, k = _weights(H, H, r, gen), _weights(256, H, r, gen)
    x = torch.randn((M, H), device="cuda", generator=gen).to(torch.bfloat16)
    gain = (1.0 + 0.1 * torch.randn(H, device="cuda", generator=gen)).to(torch.bfloat16)
    noise = 0.01 * torch.randn(H, device="cuda", generator=gen)
    lib = qerl.load_library()
    ws_g = qerl.Workspace(qerl.aqn_rmsnorm_nvfp4_lora_linear_group_workspace_bytes(M, H, [H, 256], [r, r]))
    ws_m = qerl.Workspace(lib.aqn_rmsnorm_nvfp4_lora_mlp_workspace_bytes(M, H, I, H, r, r, r))
    outs = [torch.empty((M, H), device="cuda", dtype=torch.bfloat16), torch.empty((M, 256), device="cuda", dtype=torch.bfloat16)]
    y = torch.empty((M, H), device="cuda", dtype=torch.bfloat16)

    def run():
        qerl.aqn_rmsnorm_nvfp4_lora_linear_group(x, gain, noise, 1e-6, [q[0], k[0]], [q[1], k[1]], [q[2], k[2]], [2.0, 2.0],
                                                 workspace=ws_g, outs=outs)
        qerl.aqn_rmsnorm_nvfp4_lora_mlp(x, gain, noise, 1e-6, gate[0], up[0], down[0], (gate[1], up[1], down[1]),
                                        (gate[2], up[2], down[2]), (2.0, 2.0, 2.0), workspace=ws_m, out=y)

    _replays_match(run, lambda: [outs[0], outs[1], y])
    assert qerl.workspace_status(ws_g) == 0 and qerl.workspace_status(ws_m) == 0


@pytest.mark.parametrize("M", [24, 300])
def test_backward_launches_replay_like_eager(M):
    print("graph case: backward, M =", M, flush=True)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(70 + M)
    N, K, r = 1536, 1024, 32
    wt, A, B = _weights(N, K, r, gen, transposed=True)
    x = torch.randn((M, K), device="cuda", generator=gen).to(torch.bfloat16)
    dy = torch.randn((M, N), device="cuda", generator=gen).to(torch.bfloat16)
    need = qerl.load_library().nvfp4_lora_linear_backward_workspace_bytes(M, N, K, r)
    ws = torch.empty((need + 256,), dtype=torch.uint8, device="cuda")
    held = {}

    def run():
        held["out"] = qerl.nvfp4_lora_linear_backward(x, dy, wt, A, B, 2.0, workspace=ws)

    _replays_match(run, lambda: list(held["out"]))


@pytest.mark.parametrize("M", [8, 200])
def test_mx_linear_launches_replay_like_eager(M):
    print("graph case: mx linear, M =", M, flush=True)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(90 + M)
    N, K = 1536, 2048
    codes = torch.randint(0, 256, (N, K // 2), device="cuda", dtype=torch.uint8, generator=gen)
    scales = torch.randint(118, 126, (N, K // 32), device="cuda", dtype=torch.uint8, generator=gen)
    pw = qerl.mxfp4_prepack(codes, scales)
    x = torch.randn((M, K), device="cuda", generator=gen).to(torch.bfloat16)
    held = {}

    def run():
        held["y"] = qerl.mxfp4_linear_native(x, pw)

    _replays_match(run, lambda: [held["y"]])


@pytest.mark.parametrize("M", [8, 200])
def test_mx_lora_linear_launches_replay_like_eager(M):
    """The down-projection's K-parts count their arrivals in the workspace and leave the counters at zero: replays and
    eager calls through the same workspace agree."""
    print("graph case: mx lora linear, M =", M, flush=True)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(95 + M)
    N, K, r = 1536, 2048, 32
    codes = torch.randint(0, 256, (N, K // 2), device="cuda", dtype=torch.uint8, generator=gen)
    scales = torch.randint(118, 126, (N, K // 32), device="cuda", dtype=torch.uint8, generator=gen)
    pw = qerl.mxfp4_prepack(codes, scales)
    x = torch.randn((M, K), device="cuda", generator=gen).to(torch.bfloat16)
    A = (torch.randn((r, K), device="cuda", generator=gen) / r).to(torch.bfloat16)
    B = (torch.randn((N, r), device="cuda", generator=gen) * 0.05).to(torch.bfloat16)
    bias = torch.randn((N,), device="cuda", generator=gen).to(torch.bfloat16)
    ws = qerl.Workspace(qerl.load_library().mxfp4_lora_linear_native_workspace_bytes(M, N, K, r))
    y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")

    def run():
        qerl.mxfp4_lora_linear_native(x, pw, A, B, 2.0, bias, workspace=ws, out=y)

    _replays_match(run, lambda: [y])


@pytest.mark.parametrize("M", [24, 300])
def test_group_backward_launches_replay_like_eager(M):
    print("graph case: backward group, M =", M, flush=True)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(75 + M)
    K, r = 1024, 32
    members = [_weights(N, K, r, gen, transposed=True) for N in (1024, 256, 256)]
    x = torch.randn((M, K), device="cuda", generator=gen).to(torch.bfloat16)
    dys = [torch.randn((M, N), device="cuda", generator=gen).to(torch.bfloat16) for N in (1024, 256, 256)]
    held = {}
    first = qerl.nvfp4_lora_linear_backward_group(x, dys, [m[0] for m in members], [m[1] for m in members], [m[2] for m in members], [2.0] * 3)
    need = 64 << 20
    ws = torch.empty((need,), dtype=torch.uint8, device="cuda")

    def run():
        held["out"] = qerl.nvfp4_lora_linear_backward_group(x, dys, [m[0] for m in members], [m[1] for m in members],
                                                            [m[2] for m in members], [2.0] * 3, workspace=ws)

    _replays_match(run, lambda: [held["out"][0]] + [t for pair in held["out"][1] for t in pair])
    assert torch.equal(first[0], held["out"][0])
