"""Benchmark of the NVFP4 + LoRA linear hot path on one MI355X.

Default workload: BASELINE configuration 5 -- the Qwen2.5-32B-shaped linear stack, all 64 layers' NVFP4
weights resident in HBM and distinct (17.55 GB packed, so nothing is served from a cache that a rollout would not
have), LoRA r = 64 on all seven projections, an AQN RMSNorm before q/k/v and before gate/up.  A step is one pass
of M tokens through every layer's linears:
    per layer  aqn_rmsnorm -> {q, k, v} -> o -> aqn_rmsnorm -> {gate, up} -> down
(linears in braces share their input and go out as one grouped call).  Attention is not part of this library; o
reads a fixed synthetic activation.  Up to 16 tokens down reads SiLU(gate) * up of the step's own gate / up
outputs, and {norm, q, k, v} and {norm, gate, up, SiLU-mul, down} each go out either as one persistent launch
or as separate launches (norm + LoRA down-projections, the group, down), whichever --launch-plan says; beyond
16 tokens down reads a fixed synthetic activation unless --swiglu is given.

Prints ONE JSON line.  `value` is the whole-step packed-weight GB/s of the headline leg (decode, M = 16);
`legs` carries the other token counts of the configuration (M = 1, 128: GB/s; M = 4096: TFLOP/s), each with the
roofline of its dominant kernel measured live with events on the launch stream; `achievable` holds what a
nothing-but-loads kernel and a nothing-but-MFMA kernel reach on this machine (--no-peaks skips them); `cpu_baseline`
is the oracle timed on a bounded sample on the host cores.  --config 2/3/4 and --M select the other
configurations (one leg).
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import paper_2510_11696_amd as qerl  # noqa: E402
import qerl_synth as qs              # noqa: E402

HBM_PEAK_GBS = 8000.0       # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0


class Layer:
    """NVFP4 weights + LoRA adapters + norm parameters of one decoder layer, on the GPU."""

    def __init__(self, cfg, index, gen, config_no):
        self.lin = {}
        hidden = cfg["hidden"]
        r = cfg["r"]
        for j, shp in enumerate(cfg["linears"]):
            W = (torch.randn((shp.N, shp.K), generator=gen, device="cuda", dtype=torch.float32) * 0.02
                 ).to(torch.bfloat16)
            codes, scales, ts = qerl.nvfp4_quantize(W)
            packed = qerl.nvfp4_prepack(codes, scales, ts)     # one-time re-layout of the frozen weights
            del W, codes, scales
            A = (torch.randn((r, shp.K), generator=gen, device="cuda") / r).to(torch.bfloat16)
            B = (torch.randn((shp.N, r), generator=gen, device="cuda") * 0.01).to(torch.bfloat16)
            self.lin[shp.name] = (packed, A, B)
        self.gain_in = (1 + 0.05 * torch.randn(hidden, generator=gen, device="cuda")).to(torch.bfloat16)
        self.gain_post = (1 + 0.05 * torch.randn(hidden, generator=gen, device="cuda")).to(torch.bfloat16)
        self.z_in = self.z_post = None     # views into the model's noise buffer, refilled on the device every step


class Weights:
    """Every layer's frozen tensors of a configuration, generated and quantised on the device, plus the noise
    buffer of all its RMSNorms.  Shared by the legs (token counts) of a run."""

    def __init__(self, config_no: int, layers: int | None = None):
        cfg = qs.CONFIGS[config_no]
        self.config_no, self.cfg = config_no, cfg
        self.n_layers = layers or cfg["layers"]
        self.gen = torch.Generator(device="cuda")
        self.gen.manual_seed(qs.seed_for(config_no, 0))
        t0 = time.perf_counter()
        self.layers = []
        for i in range(self.n_layers):
            self.layers.append(Layer(cfg, i, self.gen, config_no))
            if i % 16 == 15:
                torch.cuda.synchronize()
                print(f"bench.py: {i + 1} of {self.n_layers} layers quantised and packed "
                      f"({time.perf_counter() - t0:.0f} s)", file=sys.stderr, flush=True)
        hidden = cfg["hidden"]
        # the noise vectors of all RMSNorms in one buffer: one generator launch per forward pass, which draws
        # every vector anew (Section 3.3, "Adaptive Quantization Noise")
        self.sigma = qerl.aqn_sigma(1, 10, 1e-2, 5e-4)
        self.noise = torch.empty((2 * self.n_layers * hidden,), dtype=torch.float32, device="cuda")
        for i, L in enumerate(self.layers):
            L.z_in = self.noise[(2 * i) * hidden:(2 * i + 1) * hidden]
            L.z_post = self.noise[(2 * i + 1) * hidden:(2 * i + 2) * hidden]
        self.packed_bytes_per_layer = sum(s.packed_bytes for s in cfg["linears"])


class Stack:
    """Activations, outputs and workspace for M tokens on a model's weights, and the step over its layers."""

    def __init__(self, weights: Weights, M: int, swiglu: bool = False, eager: bool = False, plan: str = "auto"):
        cfg = weights.cfg
        self.w, self.cfg, self.M = weights, cfg, M
        self.swiglu, self.eager = swiglu, eager
        self.plan_request = plan
        self.n_layers, self.layers = weights.n_layers, weights.layers
        gen = weights.gen
        hidden = cfg["hidden"]
        inter = max(s.K for s in cfg["linears"])
        self.h = torch.randn((M, hidden), generator=gen, device="cuda").to(torch.bfloat16)
        self.attn = torch.randn((M, hidden), generator=gen, device="cuda").to(torch.bfloat16)
        self.act = torch.randn((M, inter), generator=gen, device="cuda").to(torch.bfloat16)
        self.xn = torch.empty((M, hidden), dtype=torch.bfloat16, device="cuda")
        self.out = {s.name: torch.empty((M, s.N), dtype=torch.bfloat16, device="cuda") for s in cfg["linears"]}
        self.t = {s.name: torch.empty((8, M, cfg["r"]), dtype=torch.float32, device="cuda") for s in cfg["linears"]}
        self.lora_scale = cfg["alpha"] / cfg["r"]
        self.passes = 0
        by = {s.name: s for s in cfg["linears"]}
        # a decoder block (q, k, v, o, gate, up, down), or any other list of linears run one after the other
        self.block = all(n in by for n in ("q", "k", "v", "o", "gate", "up", "down"))
        groups = (("q", "k", "v"), ("gate", "up")) if self.block else ()
        need = max([qerl.nvfp4_lora_linear_workspace_bytes(M, s.N, s.K, cfg["r"]) for s in cfg["linears"]]
                   + [qerl.nvfp4_lora_linear_workspace_bytes(M, sum(by[n].N for n in g), by[g[0]].K, cfg["r"] * len(g))
                      for g in groups])
        if swiglu and not self.block:
            raise SystemExit("--swiglu needs a configuration with gate, up and down projections")
        if swiglu:
            need = max(need, qerl.load_library().nvfp4_lora_linear_swiglu_workspace_bytes(M, by["down"].N, by["down"].K, cfg["r"]))
        self.ws = qerl.Workspace(need)
        self.packed_bytes_per_layer = weights.packed_bytes_per_layer
        self.flops_per_layer = sum(2 * M * s.N * s.K for s in cfg["linears"])
        # Decode (up to 16 tokens) of a decoder block: down reads SiLU(gate) * up of this step's gate / up outputs,
        # and each of {norm, q, k, v} and {norm, gate, up, SiLU-mul, down} can go out as ONE persistent launch
        # (block_kernel) or as the separate launches (norm + LoRA down-projections, the grouped stream_kernel,
        # stream_kernel with the SiLU-mul prologue).  Both compute the same thing; which is faster depends on the
        # shapes, so the stack times both over all layers when it is set up and keeps the faster ("auto").
        self.decode_block = self.block and M <= 16
        self.plan = {"qkv": "separate", "mlp": "separate"}
        self.plan_us = {}
        if self.decode_block:
            self.swiglu = True
            r = cfg["r"]
            lib = qerl.load_library()
            self.ws_qkv = qerl.Workspace(qerl.aqn_rmsnorm_nvfp4_lora_linear_group_workspace_bytes(
                M, hidden, [by[n].N for n in ("q", "k", "v")], [r] * 3))
            self.ws_mlp = qerl.Workspace(lib.aqn_rmsnorm_nvfp4_lora_mlp_workspace_bytes(
                M, hidden, by["gate"].N, by["down"].N, r, r, r))
            need = max(need, lib.nvfp4_lora_linear_swiglu_workspace_bytes(M, by["down"].N, by["down"].K, r))
            self.ws = qerl.Workspace(need)
            if plan in ("separate", "fused"):
                self.plan = {"qkv": plan, "mlp": plan}
            else:
                self.choose_plan()

    def qkv(self, L, variant):
        names = ("q", "k", "v")
        if variant == "fused":
            ws, As, Bs = zip(*(L.lin[n] for n in names))
            qerl.aqn_rmsnorm_nvfp4_lora_linear_group(self.h, L.gain_in, L.z_in, 1e-6, list(ws), list(As), list(Bs),
                                                     [self.lora_scale] * 3, workspace=self.ws_qkv,
                                                     outs=[self.out[n] for n in names])
        else:
            self.norm_group(L, names, L.gain_in, L.z_in)

    def mlp(self, L, variant):
        if variant == "fused":
            (wg, Ag, Bg), (wu, Au, Bu), (wd, Ad, Bd) = L.lin["gate"], L.lin["up"], L.lin["down"]
            qerl.aqn_rmsnorm_nvfp4_lora_mlp(self.h, L.gain_post, L.z_post, 1e-6, wg, wu, wd, (Ag, Au, Ad), (Bg, Bu, Bd),
                                            (self.lora_scale,) * 3, workspace=self.ws_mlp, out=self.out["down"])
            return
        self.norm_group(L, ("gate", "up"), L.gain_post, L.z_post)
        if self.swiglu:   # down reads SiLU(gate) (.) up straight from the two outputs above
            packed, A, B = L.lin["down"]
            qerl.nvfp4_lora_linear_packed_swiglu(self.out["gate"], self.out["up"], packed, A, B, self.lora_scale,
                                                 workspace=self.ws, out=self.out["down"])
        else:
            self.linear(L, "down", self.act)

    def choose_plan(self):
        """Time each part of the block both ways over every layer's distinct weights (graph replay, as the step
        runs) and keep the faster."""
        for part, fn in (("qkv", self.qkv), ("mlp", self.mlp)):
            best = None
            for variant in ("separate", "fused"):
                def sweep(fn=fn, variant=variant):
                    for L in self.layers:
                        fn(L, variant)
                run = sweep if self.eager else capture(sweep)
                run()
                us = timed(run, 5) / len(self.layers) * 1e3
                self.plan_us[f"{part}:{variant}"] = round(us, 2)
                if best is None or us < best[0]:
                    best = (us, variant)
            self.plan[part] = best[1]

    def linear(self, layer, name, x):
        packed, A, B = layer.lin[name]
        return qerl.nvfp4_lora_linear_packed(x, packed, A, B, self.lora_scale,
                                             workspace=self.ws, out=self.out[name])

    def norm_group(self, layer, names, gain, noise):
        """AQN RMSNorm of the hidden state, then the linears `names` that read it.  At decode sizes:
        one launch for the norm together with the LoRA down-projections, one for the group."""
        ws, As, Bs = zip(*(layer.lin[n] for n in names))
        ts = None
        if self.M <= 16:
            _, ts = qerl.aqn_rmsnorm_lora_down(self.h, gain, noise, 1e-6, list(As), out=self.xn,
                                               ts=[self.t[n] for n in names])
        else:
            qerl.aqn_rmsnorm(self.h, gain, noise, 1e-6, out=self.xn)
        return qerl.nvfp4_lora_linear_packed_group(self.xn, list(ws), list(As), list(Bs),
                                                   [self.lora_scale] * len(names), workspace=self.ws,
                                                   outs=[self.out[n] for n in names], ts=ts)

    def step(self):
        # (a captured step replays with the subsequence it was recorded with: same cost, same values)
        qerl.aqn_noise_fill(self.w.noise.numel(), self.w.sigma, qs.seed_for(0, 0), self.passes, out=self.w.noise)
        self.passes += 1
        if not self.block:
            for L in self.layers:
                for shp in self.cfg["linears"]:
                    if shp.K == self.cfg["hidden"]:
                        self.norm_group(L, (shp.name,), L.gain_in, L.z_in)
                    else:
                        self.linear(L, shp.name, self.act)
            return
        for L in self.layers:
            self.qkv(L, self.plan["qkv"])
            self.linear(L, "o", self.attn)
            self.mlp(L, self.plan["mlp"])


def capture(fn):
    """Record the launches of fn() into a HIP graph on a side stream (the
    library enqueues on torch's current stream, which is the capturing one).
    A rollout engine replays its decode step the same way; without it the
    Python/ctypes call path, not the GPU, sets the pace."""
    fn()                                  # warm: everything allocated and loaded before capture
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        fn()
    return g.replay


def timed(fn, iters):
    """Milliseconds per call, HIP events on the stream the work is launched on."""
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    start.record()
    for _ in range(iters):
        fn()
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop) / iters


def measured_traffic(kernel: str, config_no: int, shape_name: str, M: int):
    """HBM bytes per launch (fetched + written) from the committed rocprofv3 --pmc summaries
    (profiles/traffic.json: key -> {"bytes", "kernel_source", "source_sha256_16", "measured_at_commit"}), or None.
    A warning goes to stderr when the kernel's source file is not the one the table was measured with."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    if not os.path.exists(path):
        return None
    try:
        table = json.load(open(path))
    except Exception:
        return None
    e = table.get(f"{kernel}:config{config_no}:{shape_name}:M{M}")
    if not isinstance(e, dict):
        return None
    src = os.path.join(ROOT, "paper_2510_11696_amd", "csrc", e.get("kernel_source", ""))
    if os.path.isfile(src):
        import hashlib
        if hashlib.sha256(open(src, "rb").read()).hexdigest()[:16] != e.get("source_sha256_16"):
            print(f"bench.py: {e.get('kernel_source')} has changed since profiles/traffic.json was measured "
                  f"(commit {e.get('measured_at_commit')}): roofline.traffic may be stale", file=sys.stderr)
    return e.get("bytes")


def dominant_kernel_roofline(stack: Stack, reps: int):
    """Average duration of one launch of the kernel most of the step's bytes / flops go through, run back
    to back over every layer's distinct weights.  Decode (M <= 16): the feed-forward block's single launch of
    block_kernel where the step uses it, else the grouped gate_proj + up_proj launch of stream_kernel, fed
    with the LoRA down-projections the norm's launch left in memory, exactly as in the step.  M > 16: the grouped
    gate_proj + up_proj call of the step (the LoRA down-projection's launch belongs to it), or the largest linear
    where the configuration is not a decoder block; priced against HBM or MFMA, whichever binds it at the peaks."""
    by = {s.name: s for s in stack.cfg["linears"]}
    kernel = None
    if stack.decode_block and stack.plan["mlp"] == "fused":
        # the feed-forward block's persistent launch: norm, gate + up, SiLU-mul and down in block_kernel
        def sweep():
            for L in stack.layers:
                stack.mlp(L, "fused")
        shape = {"name": "norm+gate+up+silu_mul+down", "N": by["gate"].N, "K": by["gate"].K, "M": stack.M}
        bytes_per_launch = sum(by[n].packed_bytes for n in ("gate", "up", "down"))
        kernel = "block_kernel"
    elif stack.M <= 16:
        names = ("gate", "up") if stack.block else (stack.cfg["linears"][0].name,)
        for L in stack.layers[:1]:          # any valid t will do for timing: it only feeds the up-projection
            stack.norm_group(L, names, L.gain_post, L.z_post)
        ts = [stack.t[n] for n in names]

        def sweep():
            for L in stack.layers:
                ws, As, Bs = zip(*(L.lin[n] for n in names))
                qerl.nvfp4_lora_linear_packed_group(stack.xn, list(ws), list(As), list(Bs),
                                                    [stack.lora_scale] * len(names), workspace=stack.ws,
                                                    outs=[stack.out[n] for n in names], ts=ts)
        shape = {"name": "+".join(names), "N": sum(by[n].N for n in names), "K": by[names[0]].K, "M": stack.M}
        bytes_per_launch = sum(by[n].packed_bytes for n in names)
    elif stack.block:
        # the grouped gate_proj + up_proj call as the step makes it (its LoRA down-projection launch belongs to it)
        names = ("gate", "up")

        def sweep():
            for L in stack.layers:
                ws, As, Bs = zip(*(L.lin[n] for n in names))
                qerl.nvfp4_lora_linear_packed_group(stack.xn, list(ws), list(As), list(Bs), [stack.lora_scale] * 2,
                                                    workspace=stack.ws, outs=[stack.out[n] for n in names])
        shape = {"name": "gate+up", "N": sum(by[n].N for n in names), "K": by["gate"].K, "M": stack.M}
        bytes_per_launch = sum(by[n].packed_bytes for n in names)
    else:
        shp = max(stack.cfg["linears"], key=lambda s: (s.packed_bytes, s.name == "gate"))

        def sweep():
            for L in stack.layers:
                stack.linear(L, shp.name, stack.act if shp.name == "down" else stack.xn)
        shape = {"name": shp.name, "N": shp.N, "K": shp.K, "M": stack.M}
        bytes_per_launch = shp.packed_bytes
    run = sweep if stack.eager else capture(sweep)
    run()
    ms = timed(run, reps) / len(stack.layers)
    common = {"shape": shape, "us_per_launch": round(ms * 1e3, 2),
              "note": "one call per launch slot, back to back over the layers' distinct weights, launch gaps included"}
    # which roof binds the launch at the published peaks, and the kernel that runs it (17..64 tokens, and single
    # linears up to 128: the weight-streaming mid_kernel; wide groups from 65 tokens on: the GEMM)
    t_hbm = bytes_per_launch / (HBM_PEAK_GBS * 1e9)
    t_mfma = 2 * stack.M * shape["N"] * shape["K"] / (MFMA_BF16_PEAK_TFLOPS * 1e12)
    gemm = stack.M > 128 or (stack.M > 64 and shape["name"] == "gate+up" and shape["N"] >= 16384)
    if stack.M <= 16 or (not gemm) or (stack.M <= 128 and t_hbm >= t_mfma):
        kernel = kernel or ("stream_kernel" if stack.M <= 16 else ("gemm32_kernel" if gemm else "mid_kernel"))
        achieved = bytes_per_launch / (ms * 1e-3) / 1e9
        return {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": measured_traffic(kernel, stack.w.config_no, shape["name"], stack.M), "kernel": kernel,
                "algorithmic_bytes_per_launch": bytes_per_launch, **common}
    flops = 2 * stack.M * shape["N"] * shape["K"]
    achieved = flops / (ms * 1e-3) / 1e12
    return {"bound": "mfma", "achieved": round(achieved, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4),
            "traffic": measured_traffic("gemm32_kernel", stack.w.config_no, shape["name"], stack.M), "kernel": "gemm32_kernel",
            "algorithmic_flops_per_launch": flops, **common}


def cpu_baseline(config_no: int, M: int, budget_s: float = 20.0):
    """The numpy oracle's linear on the host cores, over the layer's seven
    shapes in turn (the three MLP matrices cut to 4096 output rows) until
    about half the budget is oracle time; the rest goes to preparing inputs."""
    from oracle import nvfp4_oracle as oracle
    cfg = qs.CONFIGS[config_no]
    r = cfg["r"]
    done_bytes, t_total, names = 0, 0.0, []
    t_wall = time.perf_counter()
    for j, shp in enumerate(cfg["linears"] * 4):
        if t_total > budget_s / 2 or time.perf_counter() - t_wall > 1.5 * budget_s:
            break
        N = shp.N
        if shp.packed_bytes > 20e6:           # big MLP matrices: a slice of output rows
            N = 4096
        if M > 128:                           # prefill: the matmul dominates, keep the sample small
            N = min(N, 1024)
        W = qs.weights(N, shp.K, qs.seed_for(config_no, 10 + j)).float().numpy()
        x = qs.activations(M, shp.K, qs.seed_for(config_no, 30 + j)).float().numpy()
        A, B = qs.lora_pair(N, shp.K, r, qs.seed_for(config_no, 50 + j))
        codes, scales, ts = oracle.nvfp4_quantize(W)
        t0 = time.perf_counter()
        oracle.nvfp4_lora_linear(x, codes, scales, ts, A.float().numpy(), B.float().numpy(), cfg["alpha"] / r)
        t_total += time.perf_counter() - t0
        done_bytes += N * shp.K * 9 // 16
        names.append(f"{shp.name}[{N}x{shp.K}]")
    try:
        cores = len(os.sched_getaffinity(0))
    except AttributeError:
        cores = os.cpu_count()
    threads = min(cores, torch.get_num_threads())
    flops_names = names
    counts = {}
    for n in names:
        counts[n] = counts.get(n, 0) + 1
    names = [n if c == 1 else f"{c} x {n}" for n, c in counts.items()]
    if M > 128:
        flops = sum(2 * M * int(n.split("[")[1].split("x")[0]) * int(n.split("x")[1].rstrip("]")) for n in flops_names)
        return {"value": round(flops / t_total / 1e12, 5), "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
                "sample": f"oracle nvfp4_lora_linear (dequantise + fp64 matmul + LoRA), M={M}, on "
                          + ", ".join(names) + f"; {t_total:.1f} s"}
    return {"value": round(done_bytes / t_total / 1e9, 4), "unit": "GB/s", "cores": threads,
            "kind": "oracle",
            "sample": f"oracle nvfp4_lora_linear (dequantise + fp64 matmul + LoRA), M={M}, on "
                      + ", ".join(names) + f"; {t_total:.1f} s"}


def backward_bench(args):
    """--backward: the backward pass (dX through the frozen weights, dA, dB) of every linear of a few layers at
    the configuration's prefill size; one JSON line in the same format, TFLOP/s on the dX flops."""
    cfg = qs.CONFIGS[args.config]
    M = args.M or max(cfg["M"])      # a training batch: the configuration's prefill size
    n_layers = args.layers or 2
    gen = torch.Generator(device="cuda")
    gen.manual_seed(qs.seed_for(args.config, 1))
    r = cfg["r"]
    lib = qerl.load_library()
    lin, need = [], 0
    for _ in range(n_layers):
        for shp in cfg["linears"]:
            W = (torch.randn((shp.N, shp.K), generator=gen, device="cuda", dtype=torch.float32) * 0.02).to(torch.bfloat16)
            codes, scales, ts = qerl.nvfp4_quantize(W)
            pt = qerl.nvfp4_prepack_t(codes, scales, ts)
            del W, codes, scales
            A = (torch.randn((r, shp.K), generator=gen, device="cuda") / r).to(torch.bfloat16)
            B = (torch.randn((shp.N, r), generator=gen, device="cuda") * 0.01).to(torch.bfloat16)
            lin.append((shp, pt, A, B))
            need = max(need, lib.nvfp4_lora_linear_backward_workspace_bytes(M, shp.N, shp.K, r))
    xs = {k: torch.randn((M, k), generator=gen, device="cuda").to(torch.bfloat16) for k in {s.K for s, *_ in lin}}
    dys = {n: torch.randn((M, n), generator=gen, device="cuda").to(torch.bfloat16) for n in {s.N for s, *_ in lin}}
    ws = torch.empty((need + 256,), dtype=torch.uint8, device="cuda")
    scale = cfg["alpha"] / r

    # linears that read the same x (q + k + v, gate + up) go through one grouped call: one GEMM forms their summed dX
    calls, run = [], []
    for e in lin + [None]:
        if run and (e is None or e[0].K != run[0][0].K or e[0].name in ("q", "o", "gate", "down") or len(run) == 4):
            calls.append(run)
            run = []
        if e is not None:
            run.append(e)
    for run in calls:
        if len(run) > 1:
            descs = (qerl.binding._BackwardDesc * len(run))()
            for d, (shp, *_) in zip(descs, run):
                d.N, d.r = shp.N, r
            need = max(need, lib.nvfp4_lora_linear_backward_group_workspace_bytes(M, run[0][0].K, ctypes.cast(descs, ctypes.c_void_p), len(run)))
    ws = torch.empty((need + 256,), dtype=torch.uint8, device="cuda")

    def step_separate():
        for shp, pt, A, B in lin:
            qerl.nvfp4_lora_linear_backward(xs[shp.K], dys[shp.N], pt, A, B, scale, workspace=ws)

    def step():
        for run in calls:
            if len(run) == 1:
                shp, pt, A, B = run[0]
                qerl.nvfp4_lora_linear_backward(xs[shp.K], dys[shp.N], pt, A, B, scale, workspace=ws)
            else:
                qerl.nvfp4_lora_linear_backward_group(xs[run[0][0].K], [dys[e[0].N] for e in run], [e[1] for e in run],
                                                      [e[2] for e in run], [e[3] for e in run], [scale] * len(run), workspace=ws)
    for _ in range(args.warmup):
        step()
        step_separate()
    ms_separate = timed(step_separate, args.steps)
    ms = timed(step, args.steps)
    flops = sum(2 * M * s.N * s.K for s, *_ in lin)
    tflops = flops / (ms * 1e-3) / 1e12
    # the dominant kernel: dX of the widest linear (gate: 13824 rows contracted), timed alone with its LoRA launches
    shp, pt, A, B = max(lin, key=lambda e: e[0].N * e[0].K)
    one = lambda: qerl.nvfp4_lora_linear_backward(None, dys[shp.N], pt, None, None, 0.0, workspace=ws)
    one()
    us = timed(one, max(3, args.steps)) * 1e3
    fl = 2 * M * shp.N * shp.K
    print(json.dumps({
        "metric": "NVFP4+LoRA linear backward: TFLOP/s (dX flops 2*M*N*K; dA, dB and LoRA flops not counted)",
        "value": round(tflops, 1), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 x fp4(e2m1)*fp8(e4m3) -> fp32 accumulate", "data": "synthetic",
        "config": {"workload": f"config {args.config}: backward of {cfg['model']}-shaped decoder linears, {n_layers} layers, "
                               f"M={M}, LoRA r={r} alpha={cfg['alpha']:g}; dX bf16, dA and dB fp32; eager launches; "
                               f"q+k+v and gate+up as grouped calls (summed dX)",
                   "ms_per_step_one_call_per_linear": round(ms_separate, 4)},
        "roofline": {"bound": "mfma", "achieved": round(fl / (us * 1e-6) / 1e12, 1), "peak": MFMA_BF16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(fl / (us * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": None,
                     "kernel": "gemm32_kernel<.., true> (transposed operand)", "algorithmic_flops_per_launch": fl,
                     "shape": {"name": shp.name, "N": shp.N, "K": shp.K, "M": M}, "us_per_launch": round(us, 2),
                     "note": "dX alone (no adapter): one launch"},
    }))


def mx_bench(args):
    """--mx: the MXFP4 variant's linear (x quantised to MXFP8, block-scaled matrix instruction) over the linears
    of a few layers of the configuration, no adapters; one JSON line in the same format."""
    cfg = qs.CONFIGS[args.config]
    M = args.M or cfg["M"][0]
    n_layers = args.layers or 2
    gen = torch.Generator(device="cuda")
    gen.manual_seed(qs.seed_for(args.config, 2))
    lib = qerl.load_library()
    lin, need = [], 0
    for _ in range(n_layers):
        for shp in cfg["linears"]:
            W = (torch.randn((shp.N, shp.K), generator=gen, device="cuda", dtype=torch.float32) * 0.02).to(torch.bfloat16)
            codes, scales = qerl.mxfp4_quantize(W)
            lin.append((shp, qerl.mxfp4_prepack(codes, scales)))
            del W, codes, scales
            need = max(need, lib.mxfp4_linear_native_workspace_bytes(M, shp.N, shp.K))
    xs = {k: torch.randn((M, k), generator=gen, device="cuda").to(torch.bfloat16) for k in {s.K for s, _ in lin}}
    ys = {n: torch.empty((M, n), dtype=torch.bfloat16, device="cuda") for n in {s.N for s, _ in lin}}
    ws = torch.empty((need + 256,), dtype=torch.uint8, device="cuda")

    def sweep():
        for shp, pw in lin:
            qerl.mxfp4_linear_native(xs[shp.K], pw, workspace=ws, out=ys[shp.N])
    step = sweep if args.eager else capture(sweep)
    for _ in range(args.warmup):
        step()
    ms = timed(step, args.steps)
    packed = sum(s.N * s.K * 17 // 32 for s, _ in lin)          # 4 bits per weight + one scale byte per 32
    flops = sum(2 * M * s.N * s.K for s, _ in lin)
    shp, pw = max(lin, key=lambda e: e[0].N * e[0].K)
    one = lambda: qerl.mxfp4_linear_native(xs[shp.K], pw, workspace=ws, out=ys[shp.N])
    one()
    us = timed(one, max(3, args.steps)) * 1e3
    if M <= 32:      # weight streaming: HBM bound
        value, unit, metric = packed / (ms * 1e-3) / 1e9, "GB/s", "MXFP4 linear (MXFP8 activations): packed-weight GB/s"
        ach = shp.N * shp.K * 17 // 32 / (us * 1e-6) / 1e9
        roof = {"bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBS, 4),
                "traffic": None, "kernel": "mx_native_kernel", "algorithmic_bytes_per_launch": shp.N * shp.K * 17 // 32}
    else:            # GEMM on the scaled FP8 x FP4 instruction; measured against the FP8 peak the instruction is listed under
        value, unit, metric = flops / (ms * 1e-3) / 1e12, "TFLOP/s", "MXFP4 linear (MXFP8 activations): TFLOP/s (2*M*N*K)"
        ach = 2 * M * shp.N * shp.K / (us * 1e-6) / 1e12
        roof = {"bound": "mfma", "achieved": round(ach, 1), "peak": 5000.0, "unit": "TFLOP/s", "frac": round(ach / 5000.0, 4),
                "traffic": None, "kernel": "mx_gemm_kernel (after mxfp8 quantisation of x)", "algorithmic_flops_per_launch": 2 * M * shp.N * shp.K}
    roof.update({"shape": {"name": shp.name, "N": shp.N, "K": shp.K, "M": M}, "us_per_launch": round(us, 2),
                 "note": "one call (activation quantisation + multiply), eager"})
    print(json.dumps({
        "metric": metric, "value": round(value, 1), "unit": unit, "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp8(e4m3)*e8m0 x fp4(e2m1)*e8m0 -> fp32 accumulate", "data": "synthetic",
        "config": {"workload": f"config {args.config}: MXFP4 variant of {cfg['model']}-shaped decoder linears, {n_layers} layers, "
                               f"M={M}, no adapters; " + ("eager launches" if args.eager else "one HIP graph replay per step")},
        "roofline": roof,
    }))


def quantize_bench(args):
    """--quantize: the offline step W bf16 -> NVFP4 (two-pass quantiser: tensor maximum, then scales and codes) plus
    the one-time re-layout into packed tiles, over the bf16 weights of one layer of the configuration; one JSON line
    in the same format.  Algorithmic bytes per weight: 2 x 2 B read (the tensor maximum is needed before any scale
    can be formed) + 0.5625 B written, and 0.5625 B read + 0.5625 B written by the re-layout."""
    cfg = qs.CONFIGS[args.config]
    gen = torch.Generator(device="cuda")
    gen.manual_seed(qs.seed_for(args.config, 3))
    Ws = [(shp, (torch.randn((shp.N, shp.K), generator=gen, device="cuda", dtype=torch.float32) * 0.02).to(torch.bfloat16))
          for shp in cfg["linears"]]
    n_weights = sum(s.N * s.K for s, _ in Ws)

    def quant():
        return [qerl.nvfp4_quantize(W) for _, W in Ws]

    def both():
        for c, sc, ts in quant():
            qerl.nvfp4_prepack(c, sc, ts)
    for _ in range(args.warmup):
        both()
    ms_q = timed(quant, args.steps)
    ms = timed(both, args.steps)
    bytes_q = n_weights * (4 + 0.5625)
    shp, W = max(Ws, key=lambda e: e[0].N * e[0].K)
    one = lambda: qerl.nvfp4_quantize(W)
    one()
    us = timed(one, max(3, args.steps)) * 1e3
    ach = shp.N * shp.K * (4 + 0.5625) / (us * 1e-6) / 1e9
    print(json.dumps({
        "metric": "NVFP4 quantiser + tile prepack: bf16 weight GB/s (2 B per weight over the wall time of both)",
        "value": round(n_weights * 2 / (ms * 1e-3) / 1e9, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 (scale arithmetic) on bf16 input -> fp4(e2m1) + fp8(e4m3) + f32", "data": "synthetic",
        "config": {"workload": f"config {args.config}: quantise and pack the seven linears of one {cfg['model']}-shaped layer "
                               f"({n_weights / 1e6:.1f} M weights); eager launches, torch allocates the outputs inside the timed region",
                   "ms_quantize_only": round(ms_q, 4), "algorithmic_GBps_quantize_only": round(bytes_q / (ms_q * 1e-3) / 1e9, 1)},
        "roofline": {"bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBS, 4),
                     "traffic": None, "kernel": "amax_partial_kernel + encode_kernel", "algorithmic_bytes_per_launch": int(shp.N * shp.K * (4 + 0.5625)),
                     "shape": {"name": shp.name, "N": shp.N, "K": shp.K}, "us_per_launch": round(us, 2),
                     "note": "one nvfp4_quantize call of the largest linear (three launches: partial maxima, final maximum, encode)"},
    }))


def measure_peaks():
    """What a kernel that does nothing else reaches on this machine: a streaming read of 4 GiB (far beyond the
    256 MiB memory-side cache) and a loop of nothing but v_mfma_f32_32x32x16_bf16.  Best of a few launch shapes."""
    lib = qerl.load_library()
    st = torch.cuda.current_stream().cuda_stream
    sink = torch.zeros(4, dtype=torch.float32, device="cuda")
    nbytes = 4 << 30
    buf = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    buf.view(torch.int32).random_(0, 1 << 30)
    best_read, shape_read = 0.0, None
    for wgs, kib in ((256, 8), (256, 16), (512, 8), (512, 16), (1024, 8), (1024, 4)):
        fn = lambda: lib.qerl_peak_stream_read(buf.data_ptr(), nbytes, wgs, kib, sink.data_ptr(), st)
        assert fn() == 0
        ms = timed(fn, 3)
        gbs = nbytes / (ms * 1e-3) / 1e9
        if gbs > best_read:
            best_read, shape_read = gbs, f"{wgs} workgroups x 8 waves, {kib} KiB in flight per wave"
    del buf
    ops = torch.randn(1024, device="cuda").to(torch.bfloat16)          # 2 KiB of real bf16 bit patterns
    best_mfma, shape_mfma = 0.0, None
    for wgs in (256, 512):
        iters = 20000
        fn = lambda: lib.qerl_peak_mfma_bf16(ops.data_ptr(), wgs, iters, sink.data_ptr(), st)
        assert fn() == 0
        ms = timed(fn, 3)
        tf = wgs * 4 * iters * 8 * 32768 / (ms * 1e-3) / 1e12
        if tf > best_mfma:
            best_mfma, shape_mfma = tf, f"{wgs} workgroups x 4 waves, 8 accumulators each, Gaussian bf16 operands"
    return {"hbm_read_GBps": round(best_read, 1), "hbm_read_shape": shape_read,
            "mfma_bf16_TFLOPs": round(best_mfma, 1), "mfma_shape": shape_mfma,
            "note": "measured in this run by qerl_peak_stream_read (4 GiB) / qerl_peak_mfma_bf16"}


def run_leg(weights: Weights, M: int, args, steps: int, warmup: int, peaks):
    """One token count on the model's resident weights: whole-step time and the dominant kernel's roofline."""
    cfg = weights.cfg
    stack = Stack(weights, M, swiglu=args.swiglu, eager=args.eager, plan=args.launch_plan)
    step = stack.step if args.eager else capture(stack.step)
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    ms = timed(step, steps)
    step_bytes = stack.packed_bytes_per_layer * stack.n_layers
    tflops = stack.flops_per_layer * stack.n_layers / (ms * 1e-3) / 1e12
    gbps = step_bytes / (ms * 1e-3) / 1e9
    decode = M <= 128
    value = gbps if decode else tflops
    roof = dominant_kernel_roofline(stack, max(3, steps // 2))
    peak = HBM_PEAK_GBS if decode else MFMA_BF16_PEAK_TFLOPS
    leg = {"M": M, "value": round(value, 1), "unit": "GB/s" if decode else "TFLOP/s", "steps": steps, "warmup": warmup,
           "ms_per_step": round(ms, 4), "weight_GBps": round(gbps, 1), "tflops": round(tflops, 2),
           "frac_of_peak_whole_step": round(value / peak, 4), "roofline": roof}
    if stack.decode_block:
        leg["launch_plan"] = dict(stack.plan)
        if stack.plan_us:
            leg["launch_plan_us_per_layer"] = stack.plan_us
    if decode:
        # at the published peaks the step cannot take less than the longer of its HBM time and its MFMA time
        t_hbm, t_mfma = step_bytes / (HBM_PEAK_GBS * 1e9), stack.flops_per_layer * stack.n_layers / (MFMA_BF16_PEAK_TFLOPS * 1e12)
        leg["binding_roof"] = "hbm" if t_hbm >= t_mfma else "mfma"
        leg["frac_of_binding_roof"] = round(max(t_hbm, t_mfma) / (ms * 1e-3), 4)
    if peaks:
        ach = peaks["hbm_read_GBps"] if decode else peaks["mfma_bf16_TFLOPs"]
        leg["frac_of_achievable_whole_step"] = round(value / ach, 4)
        roof["frac_of_achievable"] = round(roof["achieved"] / ach, 4)
    del stack
    torch.cuda.empty_cache()
    return leg


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=5, help="workload configuration number (1-based; see qerl_synth.CONFIGS)")
    ap.add_argument("--M", type=int, default=None, help="one token count instead of the configuration's legs")
    ap.add_argument("--layers", type=int, default=None)
    ap.add_argument("--backward", action="store_true",
                    help="time the backward pass (dX, dA, dB) of the configuration's linears at its prefill size instead of the forward step")
    ap.add_argument("--mx", action="store_true",
                    help="time the MXFP4 variant's linear (MXFP8 activations, block-scaled matrix instruction) over the configuration's linears")
    ap.add_argument("--quantize", action="store_true",
                    help="time the offline quantiser (bf16 -> NVFP4) and the tile prepack over the weights of one layer of the configuration")
    ap.add_argument("--swiglu", action="store_true",
                    help="the down projection reads SiLU(gate) (.) up from the gate/up outputs (fused into its launch at M <= 16) instead of a resident input")
    ap.add_argument("--launch-plan", choices=("auto", "separate", "fused"), default="auto",
                    help="decode (M <= 16): {norm,q,k,v} and {norm,gate,up,SiLU-mul,down} as one persistent launch each "
                         "(fused), as the separate launches, or whichever is faster per part when timed at set-up (auto)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-peaks", action="store_true", help="skip the achievable-ceiling microbenchmarks")
    ap.add_argument("--eager", action="store_true", help="launch from Python each step instead of replaying a HIP graph")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 256 MiB device copy five times (reference for the rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE counters) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_read": 256 << 20, "bytes_written": 256 << 20, "launches": 5}))
        return
    if args.backward:
        backward_bench(args)
        return
    if args.mx:
        mx_bench(args)
        return
    if args.quantize:
        quantize_bench(args)
        return
    cfg = qs.CONFIGS[args.config]
    # the headline leg first, then the configuration's other token counts
    if args.M is not None:
        Ms = [args.M]
    elif args.config == 5:
        Ms = [16, 1, 128, 4096]
    else:
        Ms = list(cfg["M"])
    if args.layers is None and args.config != 5 and min(Ms) > 128:
        args.layers = 4                     # compute bound: a few distinct layers are enough
    peaks = None if args.no_peaks else measure_peaks()
    weights = Weights(args.config, args.layers)
    legs = []
    for i, M in enumerate(Ms):
        # the headline leg is timed over exactly --steps steps after --warmup; a prefill step of the whole stack is
        # a quarter of a second, so further prefill legs take a quarter of the steps
        steps = args.steps if (i == 0 or M <= 128) else max(3, args.steps // 4)
        warmup = args.warmup if (i == 0 or M <= 128) else min(args.warmup, 1)
        legs.append(run_leg(weights, M, args, steps, warmup, peaks))
        print(f"bench.py: leg M={M}: {legs[-1]['ms_per_step']} ms per step, {legs[-1]['value']} {legs[-1]['unit']}",
              file=sys.stderr, flush=True)
    head = legs[0]
    M = head["M"]
    decode = M <= 128
    step_bytes = weights.packed_bytes_per_layer * weights.n_layers
    line = {
        "metric": "NVFP4+LoRA linear: packed-weight GB/s at decode" if decode
                  else "NVFP4+LoRA linear: TFLOP/s at prefill (2*M*N*K, LoRA flops not counted)",
        "value": head["value"], "unit": head["unit"],
        "n_gpus": 1, "steps": head["steps"], "warmup": head["warmup"],
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 x fp4(e2m1)*fp8(e4m3) -> fp32 accumulate", "data": "synthetic",
        "config": {"workload": f"config {args.config}: {cfg['model']}-shaped decoder linears, "
                               f"{weights.n_layers} layers resident ({step_bytes / 1e9:.2f} GB packed), "
                               f"{'decode' if decode else 'prefill'} M={M}, "
                               f"LoRA r={cfg['r']} alpha={cfg['alpha']:g}, "
                               "AQN RMSNorm before q/k/v and gate/up, noise vectors regenerated on the device every step; "
                               + ("down reads SiLU(gate)*up of the gate/up outputs; " if (args.swiglu or head.get("launch_plan")) else "")
                               + (f"launches per layer: q+k+v {head['launch_plan']['qkv']}, o 1, feed-forward {head['launch_plan']['mlp']}; "
                                  if head.get("launch_plan") else "")
                               + ("eager launches" if args.eager else "one HIP graph replay per step"),
                   "packed_weight_bytes_per_step": step_bytes,
                   "tflops": head["tflops"], "weight_GBps": head["weight_GBps"],
                   "frac_of_peak_whole_step": head["frac_of_peak_whole_step"]},
        "roofline": head["roofline"],
    }
    if "frac_of_achievable_whole_step" in head:
        line["config"]["frac_of_achievable_whole_step"] = head["frac_of_achievable_whole_step"]
    if len(legs) > 1:
        line["legs"] = legs[1:]
    if peaks:
        line["achievable"] = peaks
    if not args.no_cpu:
        line["cpu_baseline"] = cpu_baseline(args.config, M)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
