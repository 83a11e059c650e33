"""The entry point that allocates nothing (nvfp4_lora_linear_packed_noalloc), through the C ABI: its output equals
the ordinary packed linear's bit for bit and holds the oracle's tolerance, on calls in a row that share the
library's scratch array -- a larger shape first, smaller ones after it, every kernel family (streaming decode with
in-launch LoRA producers and K-ranges, the 17..128-token kernel, the prefill GEMM) -- and a call beyond the
array's size is refused on the host."""
import numpy as np
import pytest
import torch

import paper_2510_11696_amd as qerl
import qerl_synth as qs
from oracle import nvfp4_oracle as oracle
from tests import cases
from tests.gpu_util import check_linear

pytestmark = pytest.mark.gpu


def _case(M, N, K, r, seed):
    W = cases.gaussian(N, K, seed)
    codes, scales, ts = oracle.nvfp4_quantize(W)
    x = qs.activations(M, K, seed + 1)
    A = B = None
    if r:
        A, B = qs.lora_pair(N, K, r, seed + 2)
    g = lambda a: torch.from_numpy(a).cuda()
    pw = qerl.nvfp4_prepack(g(codes), g(scales), torch.tensor([ts], device="cuda"))
    ref = oracle.nvfp4_lora_linear(x.float().numpy(), codes, scales, ts, A.float().numpy() if r else None,
                                   B.float().numpy() if r else None, 2.0)
    return x.cuda(), pw, (A.cuda() if r else None), (B.cuda() if r else None), ref


def test_no_alloc_entry_point_equals_the_workspace_one_on_calls_in_a_row():
    shapes = [(16, 640, 18944, 32),    # decode, K split over workgroup ranges, in-launch LoRA producers
              (8, 96, 3584, 32),       # smaller, right behind it on the same scratch
              (100, 320, 2048, 16),    # the 17..128-token kernel
              (1, 64, 256, 0),         # one token, no adapter
              (300, 160, 1024, 64),    # prefill GEMM with its down-projection launch
              (3, 40, 320, 8)]         # ragged and tiny
    problems = [_case(M, N, K, r, 88000 + 10 * i) for i, (M, N, K, r) in enumerate(shapes)]
    want = [qerl.nvfp4_lora_linear_packed(x, pw, A, B, 2.0) for x, pw, A, B, _ in problems]
    outs = [torch.empty_like(w) for w in want]          # the caller's buffers: allocated before the calls
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    for (x, pw, A, B, _), out in zip(problems, outs):   # back to back on one stream, no host work between them
        qerl.nvfp4_lora_linear_packed_noalloc(x, pw, A, B, 2.0, out)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    for (x, pw, A, B, ref), out, w, shp in zip(problems, outs, want, shapes):
        print("no-alloc case", shp, flush=True)
        assert torch.equal(out, w), shp
        check_linear(out, ref, ("no-alloc", shp))
    # once more in reverse order (smaller before larger), results unchanged
    for (x, pw, A, B, _), out in list(zip(problems, outs))[::-1]:
        out.zero_()
        qerl.nvfp4_lora_linear_packed_noalloc(x, pw, A, B, 2.0, out)
    torch.cuda.synchronize()
    assert all(torch.equal(o, w) for o, w in zip(outs, want))


def test_no_alloc_entry_point_refuses_what_its_array_cannot_hold():
    lib = qerl.load_library()
    limit = lib.nvfp4_lora_linear_packed_noalloc_max_bytes()
    assert limit == 36 << 20
    M, N, K, r = 1, 65536, 27648, 0      # 31 K-ranges of 2048 row tiles: the partial tiles alone need 124 MiB
    assert lib.nvfp4_lora_linear_workspace_bytes(M, N, K, r) > limit
    fake = 0x10000
    assert lib.nvfp4_lora_linear_packed_noalloc(fake, M, K, K, fake, fake, N, None, None, r, 0.0, fake, N, None) == -4
