"""ctypes binding of libqerl_nvfp4.so: argument marshalling only.

Every function takes torch tensors living on the GPU, checks dtypes/devices,
and passes raw device pointers, sizes and the current HIP stream to the C ABI
declared in include/qerl_nvfp4.h.  No arithmetic of the method happens here and
there is no fallback: if the library is missing or a tensor is not on the GPU
the call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libqerl_nvfp4.so")

_c_i64 = ctypes.c_int64
_c_sz = ctypes.c_size_t
_c_p = ctypes.c_void_p

_SIGNATURES = {
    "qerl_status_string": (ctypes.c_char_p, [ctypes.c_int]),
    "qerl_last_hip_error": (ctypes.c_int, []),
    "nvfp4_quantize": (ctypes.c_int, [_c_p, _c_i64, _c_i64, _c_i64, _c_p, _c_p, _c_p, _c_p, _c_sz, _c_p]),
    "nvfp4_quantize_workspace_bytes": (_c_sz, [_c_i64, _c_i64]),
    "nvfp4_dequantize": (ctypes.c_int, [_c_p, _c_p, _c_p, _c_i64, _c_i64, _c_p, _c_p]),
    "nvfp4_lora_linear": (ctypes.c_int, [_c_p, _c_i64, _c_i64, _c_i64, _c_p, _c_p, _c_p, _c_i64,
                                         _c_p, _c_p, _c_i64, ctypes.c_float, _c_p, _c_i64,
                                         _c_p, _c_sz, _c_p]),
    "nvfp4_lora_linear_workspace_bytes": (_c_sz, [_c_i64, _c_i64, _c_i64, _c_i64]),
    "nvfp4_prepack_bytes": (_c_sz, [_c_i64, _c_i64]),
    "nvfp4_prepack": (ctypes.c_int, [_c_p, _c_p, _c_i64, _c_i64, _c_p, _c_p]),
    "nvfp4_lora_linear_packed": (ctypes.c_int, [_c_p, _c_i64, _c_i64, _c_i64, _c_p, _c_p, _c_i64,
                                                _c_p, _c_p, _c_i64, ctypes.c_float, _c_p, _c_i64,
                                                _c_p, _c_sz, _c_p]),
    "nvfp4_lora_linear_packed_noalloc_max_bytes": (_c_sz, []),
    "nvfp4_lora_linear_packed_noalloc": (ctypes.c_int, [_c_p, _c_i64, _c_i64, _c_i64, _c_p, _c_p, _c_i64,
                                                        _c_p, _c_p, _c_i64, ctypes.c_float, _c_p, _c_i64, _c_p]),
    "nvfp4_lora_linear_swiglu_workspace_bytes": (_c_sz, [_c_i64, _c_i64, _c_i64, _c_i64]),
    "nvfp4_lora_linear_packed_swiglu": (ctypes.c_int, [_c_p, _c_p, _c_i64, _c_i64, _c_i64, _c_i64, _c_p, _c_p, _c_i64,
                                                       _c_p, _c_p, _c_i64, ctypes.c_float, _c_p, _c_i64,
                                                       _c_p, _c_sz, _c_p]),
    "nvfp4_prepack_t_bytes": (_c_sz, [_c_i64, _c_i64]),
    "nvfp4_prepack_t": (ctypes.c_int, [_c_p, _c_p, _c_i64, _c_i64, _c_p, _c_p]),
    "nvfp4_lora_linear_backward_workspace_bytes": (_c_sz, [_c_i64, _c_i64, _c_i64, _c_i64]),
    "nvfp4_lora_linear_backward_group_workspace_bytes": (_c_sz, [_c_i64, _c_i64, _c_p, ctypes.c_int]),
    "nvfp4_lora_linear_backward_group": (ctypes.c_int, [_c_p, _c_i64, _c_i64, _c_i64, _c_p, ctypes.c_int, _c_p, _c_i64, _c_p, _c_sz, _c_p]),
    "nvfp4_lora_linear_backward": (ctypes.c_int, [_c_p, _c_p, _c_i64, _c_i64, _c_i64, _c_i64, _c_i64, _c_p, _c_p, _c_p, _c_p,
                                                  _c_i64, ctypes.c_float, _c_p, _c_i64, _c_p, _c_p, _c_p, _c_sz, _c_p]),
    "nvfp4_lora_linear_packed_group": (ctypes.c_int, [_c_p, _c_i64, _c_i64, _c_i64, _c_p, ctypes.c_int,
                                                      _c_p, _c_sz, _c_p]),
    "qerl_workspace_init": (ctypes.c_int, [_c_p, _c_sz, _c_p]),
    "aqn_rmsnorm": (ctypes.c_int, [_c_p, _c_i64, _c_i64, _c_i64, _c_p, _c_p, ctypes.c_float,
                                   _c_p, _c_i64, _c_p]),
    "aqn_rmsnorm_lora_down": (ctypes.c_int, [_c_p, _c_i64, _c_i64, _c_i64, _c_p, _c_p, ctypes.c_float,
                                             _c_p, _c_i64, _c_p, _c_p, _c_p, ctypes.c_int, _c_p]),
    "aqn_sigma": (ctypes.c_double, [ctypes.c_int, ctypes.c_int, ctypes.c_double, ctypes.c_double]),
    "aqn_sigma_schedule": (ctypes.c_double, [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double, ctypes.c_double]),
    "aqn_noise_fill": (ctypes.c_int, [_c_p, _c_i64, ctypes.c_float, ctypes.c_uint64, ctypes.c_uint64, _c_p]),
    "mxfp4_quantize": (ctypes.c_int, [_c_p, _c_i64, _c_i64, _c_i64, _c_p, _c_p, _c_p]),
    "mxfp4_dequantize": (ctypes.c_int, [_c_p, _c_p, _c_i64, _c_i64, _c_p, _c_p]),
    "mxfp8_quantize": (ctypes.c_int, [_c_p, _c_i64, _c_i64, _c_i64, _c_p, _c_p, _c_p]),
    "mxfp4_prepack_bytes": (_c_sz, [_c_i64, _c_i64]),
    "mxfp4_prepack": (ctypes.c_int, [_c_p, _c_p, _c_i64, _c_i64, _c_p, _c_p]),
    "mxfp4_linear_native_workspace_bytes": (_c_sz, [_c_i64, _c_i64, _c_i64]),
    "mxfp4_linear_native": (ctypes.c_int, [_c_p, _c_i64, _c_i64, _c_i64, _c_p, _c_i64, _c_p, _c_i64, _c_p, _c_sz, _c_p]),
    "mxfp4_lora_linear_native_workspace_bytes": (_c_sz, [_c_i64, _c_i64, _c_i64, _c_i64]),
    "mxfp4_lora_linear_native": (ctypes.c_int, [_c_p, _c_i64, _c_i64, _c_i64, _c_p, _c_i64, _c_p, _c_p, _c_i64, ctypes.c_float, _c_p,
                                                _c_p, _c_i64, _c_p, _c_sz, _c_p]),
    "aqn_rmsnorm_nvfp4_lora_linear_group_workspace_bytes": (_c_sz, [_c_i64, _c_i64, _c_p, _c_p, ctypes.c_int]),
    "aqn_rmsnorm_nvfp4_lora_linear_group": (ctypes.c_int, [_c_p, _c_i64, _c_i64, _c_i64, _c_p, _c_p, ctypes.c_float,
                                                           _c_p, ctypes.c_int, _c_p, _c_sz, _c_p]),
    "aqn_rmsnorm_nvfp4_lora_mlp_workspace_bytes": (_c_sz, [_c_i64] * 7),
    "aqn_rmsnorm_nvfp4_lora_mlp": (ctypes.c_int, [_c_p, _c_i64, _c_i64, _c_i64, _c_p, _c_p, ctypes.c_float,
                                                  _c_p, _c_p, _c_p, _c_p, _c_sz, _c_p]),
    "qerl_workspace_status": (ctypes.c_int, [_c_p, _c_p]),
    "qerl_status_from_error_word": (ctypes.c_int, [ctypes.c_uint32]),
    "qerl_selftest_wait_gives_up": (ctypes.c_int, [_c_p, ctypes.c_size_t, ctypes.c_uint32, _c_p]),
    "qerl_peak_stream_read": (ctypes.c_int, [_c_p, _c_sz, ctypes.c_int, ctypes.c_int, _c_p, _c_p]),
    "qerl_peak_mfma_bf16": (ctypes.c_int, [_c_p, ctypes.c_int, ctypes.c_int, _c_p, _c_p]),
}

EXPORTED_SYMBOLS = tuple(_SIGNATURES)

_lib = None


class QerlError(RuntimeError):
    def __init__(self, fn: str, status: int, detail: str):
        super().__init__(f"{fn} failed with status {status}: {detail}")
        self.status = status


def load_library() -> ctypes.CDLL:
    """Load the HIP library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} not found: build it with `python -m paper_2510_11696_amd.build`")
        lib = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def _check(fn: str, status: int) -> None:
    if status != 0:
        lib = load_library()
        detail = lib.qerl_status_string(status).decode()
        if status == -5:
            detail += f" (hipError_t {lib.qerl_last_hip_error()})"
        raise QerlError(fn, status, detail)


def _dev(t: torch.Tensor, dtype, name: str) -> int:
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a GPU tensor")
    if t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    return t.data_ptr()


def _rows(t: torch.Tensor, name: str):
    """(rows, cols, leading dimension) of a 2-D tensor with unit inner stride."""
    if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
        raise ValueError(f"{name} must be 2-D with contiguous rows")
    ld = t.stride(0) if t.shape[0] > 1 else max(t.shape[1], t.stride(0))
    return t.shape[0], t.shape[1], ld


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


class Workspace:
    """Device scratch for nvfp4_lora_linear, initialised once."""

    def __init__(self, nbytes: int, device="cuda"):
        self.buf = torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)
        assert self.buf.data_ptr() % 256 == 0
        _check("qerl_workspace_init",
               load_library().qerl_workspace_init(self.buf.data_ptr(), self.buf.numel(), _stream()))

    @property
    def ptr(self) -> int:
        return self.buf.data_ptr()

    @property
    def nbytes(self) -> int:
        return self.buf.numel()


def aqn_rmsnorm_lora_down(x, gain, noise, eps, As, out: Optional[torch.Tensor] = None, ts=None):
    """RMSNorm as aqn_rmsnorm plus t_i = y A_i^T of the adapters As that read y, one launch (M <= 16).
    Each t_i comes as T_PARTS partial sums over slices of H, fp32 [T_PARTS, M, r_i] (t_i.sum(0) is the
    product).  Returns (y, [t_i]); pass the t_i as `ts` to nvfp4_lora_linear_packed_group."""
    lib = load_library()
    M, H, ldx = _rows(x, "x")
    if gain.numel() != H or not gain.is_contiguous():
        raise ValueError("gain must be contiguous [H]")
    n_ptr = None
    if noise is not None:
        if noise.numel() != H or not noise.is_contiguous():
            raise ValueError("noise must be contiguous [H]")
        n_ptr = _dev(noise, torch.float32, "noise")
    if out is None:
        out = torch.empty((M, H), dtype=torch.bfloat16, device=x.device)
    _, _, ldy = _rows(out, "out")
    n = len(As)
    for A in As:
        if A.dim() != 2 or A.shape[1] != H or not A.is_contiguous():
            raise ValueError("every A must be contiguous [r, H]")
    if ts is None:
        ts = [torch.empty((T_PARTS, M, A.shape[0]), dtype=torch.float32, device=x.device) for A in As]
    a_arr = (ctypes.c_void_p * n)(*[_dev(A, torch.bfloat16, "A") for A in As])
    r_arr = (ctypes.c_int64 * n)(*[A.shape[0] for A in As])
    t_arr = (ctypes.c_void_p * n)(*[_dev(t, torch.float32, "t") for t in ts])
    _check("aqn_rmsnorm_lora_down", lib.aqn_rmsnorm_lora_down(
        _dev(x, torch.bfloat16, "x"), M, H, ldx, _dev(gain, torch.bfloat16, "gain"), n_ptr, float(eps),
        _dev(out, torch.bfloat16, "out"), ldy, ctypes.cast(a_arr, _c_p), ctypes.cast(r_arr, _c_p),
        ctypes.cast(t_arr, _c_p), n, _stream()))
    return out, ts


def aqn_sigma(stage: int, num_stages: int, sigma_start: float, sigma_end: float) -> float:
    return float(load_library().aqn_sigma(stage, num_stages, sigma_start, sigma_end))


SCHEDULE_KINDS = {"exponential": 0, "linear": 1, "cosine": 2, "logarithmic": 3}


def aqn_sigma_schedule(kind: str, stage: int, num_stages: int, sigma_start: float, sigma_end: float) -> float:
    return float(load_library().aqn_sigma_schedule(SCHEDULE_KINDS[kind], stage, num_stages, sigma_start, sigma_end))


def aqn_noise_fill(n: int, sigma: float, seed: int, subsequence: int, out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """fp32 [n] on the GPU: N(0, sigma^2) noise, a pure function of (seed, subsequence, n, sigma)."""
    if out is None:
        out = torch.empty((n,), dtype=torch.float32, device="cuda")
    if out.numel() < n:
        raise ValueError("out is too small")
    _check("aqn_noise_fill", load_library().aqn_noise_fill(
        _dev(out, torch.float32, "out"), n, float(sigma), seed & (2 ** 64 - 1), subsequence & (2 ** 64 - 1), _stream()))
    return out


def nvfp4_quantize_workspace_bytes(N: int, K: int) -> int:
    return int(load_library().nvfp4_quantize_workspace_bytes(N, K))


def nvfp4_lora_linear_workspace_bytes(M: int, N: int, K: int, r: int) -> int:
    return int(load_library().nvfp4_lora_linear_workspace_bytes(M, N, K, r))


def nvfp4_quantize(W: torch.Tensor):
    """W[N,K] bf16 -> (codes[N,K/2] u8, scales[N,K/16] u8, tensor_scale[1] f32)."""
    lib = load_library()
    N, K, ldw = _rows(W, "W")
    dev = W.device
    codes = torch.empty((N, K // 2), dtype=torch.uint8, device=dev)
    scales = torch.empty((N, K // 16), dtype=torch.uint8, device=dev)
    ts = torch.empty(1, dtype=torch.float32, device=dev)
    ws = torch.empty(lib.nvfp4_quantize_workspace_bytes(N, K), dtype=torch.uint8, device=dev)
    _check("nvfp4_quantize", lib.nvfp4_quantize(
        _dev(W, torch.bfloat16, "W"), N, K, ldw, codes.data_ptr(), scales.data_ptr(), ts.data_ptr(),
        ws.data_ptr(), ws.numel(), _stream()))
    return codes, scales, ts


def nvfp4_dequantize(codes: torch.Tensor, scales: torch.Tensor, tensor_scale: torch.Tensor):
    lib = load_library()
    N, K2 = codes.shape
    K = 2 * K2
    out = torch.empty((N, K), dtype=torch.float32, device=codes.device)
    _check("nvfp4_dequantize", lib.nvfp4_dequantize(
        _dev(codes, torch.uint8, "codes"), _dev(scales, torch.uint8, "scales"),
        _dev(tensor_scale, torch.float32, "tensor_scale"), N, K, out.data_ptr(), _stream()))
    return out


def nvfp4_lora_linear(x, codes, scales, tensor_scale, A: Optional[torch.Tensor] = None,
                      B: Optional[torch.Tensor] = None, lora_scale: float = 0.0,
                      workspace: Optional[Workspace] = None, out: Optional[torch.Tensor] = None):
    """y[M,N] = tensor_scale * x . dequant(codes, scales)^T + lora_scale * (x A^T) B^T, bf16."""
    lib = load_library()
    M, K, ldx = _rows(x, "x")
    N = codes.shape[0]
    if codes.shape[1] * 2 != K or tuple(scales.shape) != (N, K // 16):
        raise ValueError("codes must be [N, K/2] and scales [N, K/16]")
    if not codes.is_contiguous() or not scales.is_contiguous():
        raise ValueError("codes and scales must be contiguous")
    r = 0
    a_ptr = b_ptr = None
    if A is not None and B is not None and A.shape[0] > 0:
        r = A.shape[0]
        if tuple(A.shape) != (r, K) or tuple(B.shape) != (N, r) or not A.is_contiguous() or not B.is_contiguous():
            raise ValueError("A must be contiguous [r, K] and B contiguous [N, r]")
        a_ptr, b_ptr = _dev(A, torch.bfloat16, "A"), _dev(B, torch.bfloat16, "B")
    if out is None:
        out = torch.empty((M, N), dtype=torch.bfloat16, device=x.device)
    _, n_out, ldy = _rows(out, "out")
    if out.shape[0] != M or n_out != N:
        raise ValueError("out must be [M, N]")
    need = lib.nvfp4_lora_linear_workspace_bytes(M, N, K, r)
    if workspace is None:
        workspace = Workspace(need, x.device)
    _check("nvfp4_lora_linear", lib.nvfp4_lora_linear(
        _dev(x, torch.bfloat16, "x"), M, K, ldx, _dev(codes, torch.uint8, "codes"),
        _dev(scales, torch.uint8, "scales"), _dev(tensor_scale, torch.float32, "tensor_scale"), N,
        a_ptr, b_ptr, r, float(lora_scale), _dev(out, torch.bfloat16, "out"), ldy,
        workspace.ptr, workspace.nbytes, _stream()))
    return out


class PackedWeight:
    """Tile-packed NVFP4 weight (see nvfp4_prepack in the header) plus its shape."""

    def __init__(self, packed: torch.Tensor, tensor_scale: torch.Tensor, N: int, K: int):
        self.packed, self.tensor_scale, self.N, self.K = packed, tensor_scale, int(N), int(K)


def nvfp4_prepack(codes: torch.Tensor, scales: torch.Tensor, tensor_scale: torch.Tensor) -> PackedWeight:
    lib = load_library()
    N, K2 = codes.shape
    K = 2 * K2
    if tuple(scales.shape) != (N, K // 16) or not codes.is_contiguous() or not scales.is_contiguous():
        raise ValueError("codes must be contiguous [N, K/2] and scales contiguous [N, K/16]")
    packed = torch.empty(max(lib.nvfp4_prepack_bytes(N, K), 16), dtype=torch.uint8, device=codes.device)
    _check("nvfp4_prepack", lib.nvfp4_prepack(
        _dev(codes, torch.uint8, "codes"), _dev(scales, torch.uint8, "scales"), N, K,
        packed.data_ptr(), _stream()))
    return PackedWeight(packed, tensor_scale, N, K)


def nvfp4_lora_linear_packed(x, w: PackedWeight, A: Optional[torch.Tensor] = None,
                             B: Optional[torch.Tensor] = None, lora_scale: float = 0.0,
                             workspace: Optional[Workspace] = None, out: Optional[torch.Tensor] = None):
    """Same result as nvfp4_lora_linear, from tile-packed weights."""
    lib = load_library()
    M, K, ldx = _rows(x, "x")
    N = w.N
    if K != w.K:
        raise ValueError("x has the wrong number of columns")
    r = 0
    a_ptr = b_ptr = None
    if A is not None and B is not None and A.shape[0] > 0:
        r = A.shape[0]
        if tuple(A.shape) != (r, K) or tuple(B.shape) != (N, r) or not A.is_contiguous() or not B.is_contiguous():
            raise ValueError("A must be contiguous [r, K] and B contiguous [N, r]")
        a_ptr, b_ptr = _dev(A, torch.bfloat16, "A"), _dev(B, torch.bfloat16, "B")
    if out is None:
        out = torch.empty((M, N), dtype=torch.bfloat16, device=x.device)
    _, n_out, ldy = _rows(out, "out")
    if out.shape[0] != M or n_out != N:
        raise ValueError("out must be [M, N]")
    if workspace is None:
        workspace = Workspace(lib.nvfp4_lora_linear_workspace_bytes(M, N, K, r), x.device)
    _check("nvfp4_lora_linear_packed", lib.nvfp4_lora_linear_packed(
        _dev(x, torch.bfloat16, "x"), M, K, ldx, _dev(w.packed, torch.uint8, "packed"),
        _dev(w.tensor_scale, torch.float32, "tensor_scale"), N, a_ptr, b_ptr, r, float(lora_scale),
        _dev(out, torch.bfloat16, "out"), ldy, workspace.ptr, workspace.nbytes, _stream()))
    return out


def nvfp4_lora_linear_packed_noalloc(x, w: PackedWeight, A: Optional[torch.Tensor], B: Optional[torch.Tensor],
                                     lora_scale: float, out: torch.Tensor):
    """nvfp4_lora_linear_packed on the library's own per-GPU scratch array: no workspace, nothing allocated
    (the caller brings `out`).  Calls on one GPU share that array and must not overlap."""
    lib = load_library()
    M, K, ldx = _rows(x, "x")
    if K != w.K:
        raise ValueError("x has the wrong number of columns")
    r = 0
    a_ptr = b_ptr = None
    if A is not None and B is not None and A.shape[0] > 0:
        r = A.shape[0]
        if tuple(A.shape) != (r, K) or tuple(B.shape) != (w.N, r) or not A.is_contiguous() or not B.is_contiguous():
            raise ValueError("A must be contiguous [r, K] and B contiguous [N, r]")
        a_ptr, b_ptr = _dev(A, torch.bfloat16, "A"), _dev(B, torch.bfloat16, "B")
    _, n_out, ldy = _rows(out, "out")
    if out.shape[0] != M or n_out != w.N:
        raise ValueError("out must be [M, N]")
    _check("nvfp4_lora_linear_packed_noalloc", lib.nvfp4_lora_linear_packed_noalloc(
        _dev(x, torch.bfloat16, "x"), M, K, ldx, _dev(w.packed, torch.uint8, "packed"),
        _dev(w.tensor_scale, torch.float32, "tensor_scale"), w.N, a_ptr, b_ptr, r, float(lora_scale),
        _dev(out, torch.bfloat16, "out"), ldy, _stream()))
    return out


def nvfp4_lora_linear_packed_swiglu(gate, up, w: PackedWeight, A: Optional[torch.Tensor] = None,
                                    B: Optional[torch.Tensor] = None, lora_scale: float = 0.0,
                                    workspace: Optional[Workspace] = None, out: Optional[torch.Tensor] = None):
    """The down projection applied to bf16(bf16(SiLU(gate)) * up)."""
    lib = load_library()
    M, K, ldg = _rows(gate, "gate")
    M2, K2, ldu = _rows(up, "up")
    N = w.N
    if K != w.K or (M2, K2) != (M, K):
        raise ValueError("gate and up must both be [M, K]")
    r = 0
    a_ptr = b_ptr = None
    if A is not None and B is not None and A.shape[0] > 0:
        r = A.shape[0]
        if tuple(A.shape) != (r, K) or tuple(B.shape) != (N, r) or not A.is_contiguous() or not B.is_contiguous():
            raise ValueError("A must be contiguous [r, K] and B contiguous [N, r]")
        a_ptr, b_ptr = _dev(A, torch.bfloat16, "A"), _dev(B, torch.bfloat16, "B")
    if out is None:
        out = torch.empty((M, N), dtype=torch.bfloat16, device=gate.device)
    _, n_out, ldy = _rows(out, "out")
    if out.shape[0] != M or n_out != N:
        raise ValueError("out must be [M, N]")
    if workspace is None:
        workspace = Workspace(lib.nvfp4_lora_linear_swiglu_workspace_bytes(M, N, K, r), gate.device)
    _check("nvfp4_lora_linear_packed_swiglu", lib.nvfp4_lora_linear_packed_swiglu(
        _dev(gate, torch.bfloat16, "gate"), _dev(up, torch.bfloat16, "up"), M, K, ldg, ldu,
        _dev(w.packed, torch.uint8, "packed"), _dev(w.tensor_scale, torch.float32, "tensor_scale"), N, a_ptr, b_ptr, r,
        float(lora_scale), _dev(out, torch.bfloat16, "out"), ldy, workspace.ptr, workspace.nbytes, _stream()))
    return out


class PackedWeightT:
    """The transposed tile order of one NVFP4 weight (nvfp4_prepack_t), for the backward pass."""

    def __init__(self, packed, tensor_scale, N, K):
        self.packed, self.tensor_scale, self.N, self.K = packed, tensor_scale, N, K


def nvfp4_prepack_t(codes: torch.Tensor, scales: torch.Tensor, tensor_scale: torch.Tensor) -> PackedWeightT:
    lib = load_library()
    N, K = codes.shape[0], codes.shape[1] * 2
    if tuple(scales.shape) != (N, K // 16) or not codes.is_contiguous() or not scales.is_contiguous():
        raise ValueError("codes must be contiguous [N, K/2] and scales contiguous [N, K/16]")
    packed = torch.empty((lib.nvfp4_prepack_t_bytes(N, K),), dtype=torch.uint8, device=codes.device)
    _check("nvfp4_prepack_t", lib.nvfp4_prepack_t(_dev(codes, torch.uint8, "codes"), _dev(scales, torch.uint8, "scales"),
                                                  N, K, _dev(packed, torch.uint8, "packed"), _stream()))
    return PackedWeightT(packed, tensor_scale, N, K)


def nvfp4_lora_linear_backward(x, dy, w: PackedWeightT, A: Optional[torch.Tensor] = None,
                               B: Optional[torch.Tensor] = None, lora_scale: float = 0.0,
                               workspace: Optional[torch.Tensor] = None):
    """(dx bf16 [M, K], dA fp32 [r, K] or None, dB fp32 [N, r] or None)."""
    lib = load_library()
    M, N, lddy = _rows(dy, "dy")
    K = w.K
    if N != w.N:
        raise ValueError("dy has the wrong number of columns")
    r = 0
    x_ptr = a_ptr = b_ptr = da_ptr = db_ptr = None
    ldx = K
    dA = dB = None
    if A is not None and B is not None and A.shape[0] > 0:
        r = A.shape[0]
        if tuple(A.shape) != (r, K) or tuple(B.shape) != (N, r) or not A.is_contiguous() or not B.is_contiguous():
            raise ValueError("A must be contiguous [r, K] and B contiguous [N, r]")
        Mx, Kx, ldx = _rows(x, "x")
        if (Mx, Kx) != (M, K):
            raise ValueError("x must be [M, K]")
        x_ptr = _dev(x, torch.bfloat16, "x")
        a_ptr, b_ptr = _dev(A, torch.bfloat16, "A"), _dev(B, torch.bfloat16, "B")
        dA = torch.empty((r, K), dtype=torch.float32, device=dy.device)
        dB = torch.empty((N, r), dtype=torch.float32, device=dy.device)
        da_ptr, db_ptr = _dev(dA, torch.float32, "dA"), _dev(dB, torch.float32, "dB")
    dx = torch.empty((M, K), dtype=torch.bfloat16, device=dy.device)
    need = lib.nvfp4_lora_linear_backward_workspace_bytes(M, N, K, r)
    if workspace is None:
        workspace = torch.empty((need + 256,), dtype=torch.uint8, device=dy.device)
    base = workspace.data_ptr()
    ws_ptr = (base + 255) & ~255
    _check("nvfp4_lora_linear_backward", lib.nvfp4_lora_linear_backward(
        x_ptr, _dev(dy, torch.bfloat16, "dy"), M, K, N, ldx, lddy, _dev(w.packed, torch.uint8, "packed_t"),
        _dev(w.tensor_scale, torch.float32, "tensor_scale"), a_ptr, b_ptr, r, float(lora_scale),
        _dev(dx, torch.bfloat16, "dx"), K, da_ptr, db_ptr, ws_ptr, workspace.numel() - (ws_ptr - base), _stream()))
    return dx, dA, dB


class _BackwardDesc(ctypes.Structure):
    """Mirror of qerl_backward_desc in the header."""
    _fields_ = [("dy", _c_p), ("lddy", _c_i64), ("N", _c_i64), ("packed_t", _c_p), ("tensor_scale", _c_p), ("A", _c_p), ("B", _c_p),
                ("r", _c_i64), ("lora_scale", ctypes.c_float), ("dA", _c_p), ("dB", _c_p)]


def nvfp4_lora_linear_backward_group(x, dys, weights, As=None, Bs=None, lora_scales=None, workspace: Optional[torch.Tensor] = None):
    """Backward of several linears that read the same x: (dx bf16 [M, K] summed over the members, [(dA_i, dB_i)])."""
    lib = load_library()
    n = len(weights)
    As = As if As is not None else [None] * n
    Bs = Bs if Bs is not None else [None] * n
    lora_scales = lora_scales if lora_scales is not None else [0.0] * n
    M, K, ldx = _rows(x, "x")
    descs = (_BackwardDesc * n)()
    grads, keep = [], []
    for i, (dy, w) in enumerate(zip(dys, weights)):
        Mi, N, lddy = _rows(dy, "dy")
        if Mi != M or N != w.N or w.K != K:
            raise ValueError("every dy must be [M, N_i] and every member must have K columns")
        d = descs[i]
        d.dy, d.lddy, d.N = _dev(dy, torch.bfloat16, "dy"), lddy, N
        d.packed_t, d.tensor_scale = _dev(w.packed, torch.uint8, "packed_t"), _dev(w.tensor_scale, torch.float32, "tensor_scale")
        A, B = As[i], Bs[i]
        dA = dB = None
        if A is not None and B is not None and A.shape[0] > 0:
            r = A.shape[0]
            if tuple(A.shape) != (r, K) or tuple(B.shape) != (N, r) or not A.is_contiguous() or not B.is_contiguous():
                raise ValueError("A must be contiguous [r, K] and B contiguous [N, r]")
            dA = torch.empty((r, K), dtype=torch.float32, device=x.device)
            dB = torch.empty((N, r), dtype=torch.float32, device=x.device)
            d.A, d.B, d.r, d.lora_scale = _dev(A, torch.bfloat16, "A"), _dev(B, torch.bfloat16, "B"), r, float(lora_scales[i])
            d.dA, d.dB = _dev(dA, torch.float32, "dA"), _dev(dB, torch.float32, "dB")
        grads.append((dA, dB))
        keep.append((dy, A, B))
    dx = torch.empty((M, K), dtype=torch.bfloat16, device=x.device)
    need = lib.nvfp4_lora_linear_backward_group_workspace_bytes(M, K, ctypes.cast(descs, _c_p), n)
    if need == 0:
        raise ValueError("a backward group has 1..4 members")
    if workspace is None:
        workspace = torch.empty((need + 256,), dtype=torch.uint8, device=x.device)
    base = workspace.data_ptr()
    ws_ptr = (base + 255) & ~255
    _check("nvfp4_lora_linear_backward_group", lib.nvfp4_lora_linear_backward_group(
        _dev(x, torch.bfloat16, "x"), M, K, ldx, ctypes.cast(descs, _c_p), n, _dev(dx, torch.bfloat16, "dx"), K,
        ws_ptr, workspace.numel() - (ws_ptr - base), _stream()))
    return dx, grads


T_PARTS = 8   # QERL_T_PARTS in the header


class _LinearDesc(ctypes.Structure):
    """Mirror of qerl_linear_desc in the header."""
    _fields_ = [("packed", _c_p), ("tensor_scale", _c_p), ("N", _c_i64), ("A", _c_p), ("B", _c_p),
                ("r", _c_i64), ("lora_scale", ctypes.c_float), ("y", _c_p), ("ldy", _c_i64), ("t", _c_p),
                ("bias", _c_p)]


def nvfp4_lora_linear_packed_group(x, weights, As=None, Bs=None, lora_scales=None,
                                   workspace: Optional[Workspace] = None, outs=None, ts=None, biases=None):
    """Several packed linears that read the same x (q/k/v, gate/up) in one launch.
    weights: list of PackedWeight; As/Bs: lists of LoRA matrices (or None); ts: optional list of
    precomputed x A^T (fp32 [M, r], from aqn_rmsnorm_lora_down); biases: optional list of bf16 [N]
    vectors (or None); returns the list of outputs."""
    lib = load_library()
    M, K, ldx = _rows(x, "x")
    n = len(weights)
    As = As if As is not None else [None] * n
    Bs = Bs if Bs is not None else [None] * n
    lora_scales = lora_scales if lora_scales is not None else [0.0] * n
    if outs is None:
        outs = [torch.empty((M, w.N), dtype=torch.bfloat16, device=x.device) for w in weights]
    descs = (_LinearDesc * n)()
    n_sum = r_sum = 0
    for i, w in enumerate(weights):
        if w.K != K:
            raise ValueError("every member must have K columns")
        r = 0
        a_ptr = b_ptr = None
        if As[i] is not None and Bs[i] is not None and As[i].shape[0] > 0:
            r = As[i].shape[0]
            if tuple(As[i].shape) != (r, K) or tuple(Bs[i].shape) != (w.N, r) or not As[i].is_contiguous() \
                    or not Bs[i].is_contiguous():
                raise ValueError("A must be contiguous [r, K] and B contiguous [N, r]")
            a_ptr, b_ptr = _dev(As[i], torch.bfloat16, "A"), _dev(Bs[i], torch.bfloat16, "B")
        _, n_out, ldy = _rows(outs[i], "out")
        if outs[i].shape[0] != M or n_out != w.N:
            raise ValueError("out must be [M, N]")
        t_ptr = None
        if ts is not None and ts[i] is not None and r > 0:
            if tuple(ts[i].shape) != (T_PARTS, M, r) or not ts[i].is_contiguous():
                raise ValueError("t must be contiguous [T_PARTS, M, r] as aqn_rmsnorm_lora_down writes it")
            t_ptr = _dev(ts[i], torch.float32, "t")
        bias_ptr = None
        if biases is not None and biases[i] is not None:
            if tuple(biases[i].shape) != (w.N,) or not biases[i].is_contiguous():
                raise ValueError("bias must be contiguous [N]")
            bias_ptr = _dev(biases[i], torch.bfloat16, "bias")
        descs[i] = _LinearDesc(_dev(w.packed, torch.uint8, "packed"),
                               _dev(w.tensor_scale, torch.float32, "tensor_scale"), w.N, a_ptr, b_ptr, r,
                               float(lora_scales[i]), _dev(outs[i], torch.bfloat16, "out"), ldy, t_ptr, bias_ptr)
        n_sum += w.N
        r_sum += r
    if workspace is None:
        workspace = Workspace(lib.nvfp4_lora_linear_workspace_bytes(M, n_sum, K, r_sum), x.device)
    _check("nvfp4_lora_linear_packed_group", lib.nvfp4_lora_linear_packed_group(
        _dev(x, torch.bfloat16, "x"), M, K, ldx, ctypes.cast(descs, _c_p), n,
        workspace.ptr, workspace.nbytes, _stream()))
    return outs


def _make_desc(w: PackedWeight, A, B, lora_scale, out, bias, K):
    """One qerl_linear_desc from torch tensors (out may be None: y = NULL); returns (desc, r)."""
    if w.K != K:
        raise ValueError("every member must have K columns")
    r = 0
    a_ptr = b_ptr = None
    if A is not None and B is not None and A.shape[0] > 0:
        r = A.shape[0]
        if tuple(A.shape) != (r, K) or tuple(B.shape) != (w.N, r) or not A.is_contiguous() or not B.is_contiguous():
            raise ValueError("A must be contiguous [r, K] and B contiguous [N, r]")
        a_ptr, b_ptr = _dev(A, torch.bfloat16, "A"), _dev(B, torch.bfloat16, "B")
    y_ptr, ldy = None, 0
    if out is not None:
        _, n_out, ldy = _rows(out, "out")
        if n_out != w.N:
            raise ValueError("out must be [M, N]")
        y_ptr = _dev(out, torch.bfloat16, "out")
    bias_ptr = None
    if bias is not None:
        if tuple(bias.shape) != (w.N,) or not bias.is_contiguous():
            raise ValueError("bias must be contiguous [N]")
        bias_ptr = _dev(bias, torch.bfloat16, "bias")
    return _LinearDesc(_dev(w.packed, torch.uint8, "packed"), _dev(w.tensor_scale, torch.float32, "tensor_scale"),
                       w.N, a_ptr, b_ptr, r, float(lora_scale), y_ptr, ldy, None, bias_ptr), r


def _norm_args(x, gain, noise):
    M, H, ldx = _rows(x, "x")
    g_ptr = n_ptr = None
    if gain is not None:
        if gain.numel() != H or not gain.is_contiguous():
            raise ValueError("gain must be contiguous [H]")
        g_ptr = _dev(gain, torch.bfloat16, "gain")
        if noise is not None:
            if noise.numel() != H or not noise.is_contiguous():
                raise ValueError("noise must be contiguous [H]")
            n_ptr = _dev(noise, torch.float32, "noise")
    return M, H, ldx, g_ptr, n_ptr


def aqn_rmsnorm_nvfp4_lora_linear_group(x, gain, noise, eps, weights, As=None, Bs=None, lora_scales=None,
                                        workspace: Optional[Workspace] = None, outs=None, biases=None):
    """AQN RMSNorm of x (gain None: x as it is), then the packed linears `weights` on it; one launch up to
    16 tokens.  Returns the list of outputs."""
    lib = load_library()
    M, K, ldx, g_ptr, n_ptr = _norm_args(x, gain, noise)
    n = len(weights)
    As = As if As is not None else [None] * n
    Bs = Bs if Bs is not None else [None] * n
    lora_scales = lora_scales if lora_scales is not None else [0.0] * n
    biases = biases if biases is not None else [None] * n
    if outs is None:
        outs = [torch.empty((M, w.N), dtype=torch.bfloat16, device=x.device) for w in weights]
    descs = (_LinearDesc * n)()
    rs = []
    for i, w in enumerate(weights):
        if outs[i].shape[0] != M:
            raise ValueError("out must be [M, N]")
        descs[i], r = _make_desc(w, As[i], Bs[i], lora_scales[i], outs[i], biases[i], K)
        rs.append(r)
    if workspace is None:
        workspace = Workspace(aqn_rmsnorm_nvfp4_lora_linear_group_workspace_bytes(M, K, [w.N for w in weights], rs), x.device)
    _check("aqn_rmsnorm_nvfp4_lora_linear_group", lib.aqn_rmsnorm_nvfp4_lora_linear_group(
        _dev(x, torch.bfloat16, "x"), M, K, ldx, g_ptr, n_ptr, float(eps), ctypes.cast(descs, _c_p), n,
        workspace.ptr, workspace.nbytes, _stream()))
    return outs


def aqn_rmsnorm_nvfp4_lora_linear_group_workspace_bytes(M: int, K: int, Ns, rs) -> int:
    n = len(Ns)
    return int(load_library().aqn_rmsnorm_nvfp4_lora_linear_group_workspace_bytes(
        M, K, ctypes.cast((ctypes.c_int64 * n)(*Ns), _c_p), ctypes.cast((ctypes.c_int64 * n)(*rs), _c_p), n))


def aqn_rmsnorm_nvfp4_lora_mlp(x, gain, noise, eps, gate: PackedWeight, up: PackedWeight, down: PackedWeight,
                               As=(None, None, None), Bs=(None, None, None), lora_scales=(0.0, 0.0, 0.0),
                               workspace: Optional[Workspace] = None, out: Optional[torch.Tensor] = None):
    """Feed-forward block: AQN RMSNorm -> gate, up -> SiLU(gate) * up -> down; one launch up to 16 tokens.
    As / Bs / lora_scales are (gate, up, down) triples.  Returns down's output [M, down.N]."""
    lib = load_library()
    M, H, ldx, g_ptr, n_ptr = _norm_args(x, gain, noise)
    if gate.N != up.N or down.K != gate.N:
        raise ValueError("gate and up must have the same N, which is down's K")
    if out is None:
        out = torch.empty((M, down.N), dtype=torch.bfloat16, device=x.device)
    if out.shape[0] != M:
        raise ValueError("out must be [M, N]")
    dg, rg = _make_desc(gate, As[0], Bs[0], lora_scales[0], None, None, H)
    du, ru = _make_desc(up, As[1], Bs[1], lora_scales[1], None, None, H)
    dd, rd = _make_desc(down, As[2], Bs[2], lora_scales[2], out, None, gate.N)
    if workspace is None:
        workspace = Workspace(lib.aqn_rmsnorm_nvfp4_lora_mlp_workspace_bytes(M, H, gate.N, down.N, rg, ru, rd), x.device)
    _check("aqn_rmsnorm_nvfp4_lora_mlp", lib.aqn_rmsnorm_nvfp4_lora_mlp(
        _dev(x, torch.bfloat16, "x"), M, H, ldx, g_ptr, n_ptr, float(eps), ctypes.byref(dg), ctypes.byref(du),
        ctypes.byref(dd), workspace.ptr, workspace.nbytes, _stream()))
    return out


def workspace_status(workspace: Workspace) -> int:
    """0, or the negative status a kernel's abandoned wait left in the workspace (synchronises)."""
    return int(load_library().qerl_workspace_status(workspace.ptr, _stream()))


def aqn_rmsnorm(x, gain, noise: Optional[torch.Tensor] = None, eps: float = 1e-6,
                out: Optional[torch.Tensor] = None):
    """y = (gain + noise) * x / sqrt(mean(x^2) + eps), bf16; noise=None is the noise-free stage."""
    lib = load_library()
    M, H, ldx = _rows(x, "x")
    if gain.numel() != H or not gain.is_contiguous():
        raise ValueError("gain must be contiguous [H]")
    n_ptr = None
    if noise is not None:
        if noise.numel() != H or not noise.is_contiguous():
            raise ValueError("noise must be contiguous [H]")
        n_ptr = _dev(noise, torch.float32, "noise")
    if out is None:
        out = torch.empty((M, H), dtype=torch.bfloat16, device=x.device)
    _, _, ldy = _rows(out, "out")
    _check("aqn_rmsnorm", lib.aqn_rmsnorm(
        _dev(x, torch.bfloat16, "x"), M, H, ldx, _dev(gain, torch.bfloat16, "gain"), n_ptr,
        float(eps), _dev(out, torch.bfloat16, "out"), ldy, _stream()))
    return out


# ---- MXFP4 variant ---------------------------------------------------------------------------------
def mxfp4_quantize(W: torch.Tensor):
    """W [N, K] bf16 (rows may be strided) -> (codes [N, K/2] u8, scales [N, K/32] u8 E8M0)."""
    N, K, ldw = _rows(W, "W")
    codes = torch.empty((N, K // 2), dtype=torch.uint8, device=W.device)
    scales = torch.empty((N, K // 32), dtype=torch.uint8, device=W.device)
    _check("mxfp4_quantize", load_library().mxfp4_quantize(
        _dev(W, torch.bfloat16, "W"), N, K, ldw, _dev(codes, torch.uint8, "codes"), _dev(scales, torch.uint8, "scales"), _stream()))
    return codes, scales


def mxfp4_dequantize(codes: torch.Tensor, scales: torch.Tensor) -> torch.Tensor:
    N, K = codes.shape[0], codes.shape[1] * 2
    W = torch.empty((N, K), dtype=torch.float32, device=codes.device)
    _check("mxfp4_dequantize", load_library().mxfp4_dequantize(
        _dev(codes, torch.uint8, "codes"), _dev(scales, torch.uint8, "scales"), N, K, _dev(W, torch.float32, "W"), _stream()))
    return W


def mxfp8_quantize(x: torch.Tensor):
    """x [M, K] bf16 -> (codes [M, K] u8 E4M3, scales [M, K/32] u8 E8M0)."""
    M, K, ldx = _rows(x, "x")
    codes = torch.empty((M, K), dtype=torch.uint8, device=x.device)
    scales = torch.empty((M, K // 32), dtype=torch.uint8, device=x.device)
    _check("mxfp8_quantize", load_library().mxfp8_quantize(
        _dev(x, torch.bfloat16, "x"), M, K, ldx, _dev(codes, torch.uint8, "codes"), _dev(scales, torch.uint8, "scales"), _stream()))
    return codes, scales


class MxPackedWeight:
    """MXFP4 weights in the tile order of the scaled matrix instruction."""

    def __init__(self, packed: torch.Tensor, N: int, K: int):
        self.packed, self.N, self.K = packed, N, K


def mxfp4_prepack(codes: torch.Tensor, scales: torch.Tensor) -> MxPackedWeight:
    lib = load_library()
    N, K = codes.shape[0], codes.shape[1] * 2
    if not codes.is_contiguous() or not scales.is_contiguous() or tuple(scales.shape) != (N, K // 32):
        raise ValueError("codes [N, K/2] and scales [N, K/32] must be contiguous")
    packed = torch.empty((lib.mxfp4_prepack_bytes(N, K),), dtype=torch.uint8, device=codes.device)
    _check("mxfp4_prepack", lib.mxfp4_prepack(_dev(codes, torch.uint8, "codes"), _dev(scales, torch.uint8, "scales"), N, K,
                                              _dev(packed, torch.uint8, "packed"), _stream()))
    return MxPackedWeight(packed, N, K)


def mxfp4_linear_native(x: torch.Tensor, w: MxPackedWeight, workspace: Optional[torch.Tensor] = None,
                        out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """y = MXFP8(x) . MXFP4(W)^T on the block-scaled matrix instruction (any number of tokens)."""
    lib = load_library()
    M, K, ldx = _rows(x, "x")
    if K != w.K:
        raise ValueError("x must have K columns")
    if out is None:
        out = torch.empty((M, w.N), dtype=torch.bfloat16, device=x.device)
    _, n_out, ldy = _rows(out, "out")
    if out.shape[0] != M or n_out != w.N:
        raise ValueError("out must be [M, N]")
    need = lib.mxfp4_linear_native_workspace_bytes(M, w.N, K)
    if workspace is None:
        workspace = torch.empty((need + 256,), dtype=torch.uint8, device=x.device)
    base = workspace.data_ptr()
    ptr = (base + 255) & ~255
    _check("mxfp4_linear_native", lib.mxfp4_linear_native(
        _dev(x, torch.bfloat16, "x"), M, K, ldx, _dev(w.packed, torch.uint8, "packed"), w.N,
        _dev(out, torch.bfloat16, "out"), ldy, ptr, workspace.numel() - (ptr - base), _stream()))
    return out


def mxfp4_lora_linear_native(x: torch.Tensor, w: MxPackedWeight, A: Optional[torch.Tensor] = None,
                             B: Optional[torch.Tensor] = None, lora_scale: float = 0.0,
                             bias: Optional[torch.Tensor] = None, workspace: Optional[Workspace] = None,
                             out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """y = MXFP8(x) . MXFP4(W)^T + lora_scale * (x A^T) B^T + bias (Eq. 2 on the native product)."""
    lib = load_library()
    M, K, ldx = _rows(x, "x")
    if K != w.K:
        raise ValueError("x must have K columns")
    r = 0
    a_ptr = b_ptr = None
    if A is not None and B is not None and A.shape[0] > 0:
        r = A.shape[0]
        if tuple(A.shape) != (r, K) or tuple(B.shape) != (w.N, r) or not A.is_contiguous() or not B.is_contiguous():
            raise ValueError("A must be contiguous [r, K] and B contiguous [N, r]")
        a_ptr, b_ptr = _dev(A, torch.bfloat16, "A"), _dev(B, torch.bfloat16, "B")
    bias_ptr = None
    if bias is not None:
        if tuple(bias.shape) != (w.N,) or not bias.is_contiguous():
            raise ValueError("bias must be contiguous [N]")
        bias_ptr = _dev(bias, torch.bfloat16, "bias")
    if out is None:
        out = torch.empty((M, w.N), dtype=torch.bfloat16, device=x.device)
    _, n_out, ldy = _rows(out, "out")
    if out.shape[0] != M or n_out != w.N:
        raise ValueError("out must be [M, N]")
    if workspace is None:
        need = lib.mxfp4_lora_linear_native_workspace_bytes(M, w.N, K, r)
        if need == 0:
            raise ValueError("rank not supported by mxfp4_lora_linear_native")
        workspace = Workspace(need, x.device)
    _check("mxfp4_lora_linear_native", lib.mxfp4_lora_linear_native(
        _dev(x, torch.bfloat16, "x"), M, K, ldx, _dev(w.packed, torch.uint8, "packed"), w.N, a_ptr, b_ptr, r,
        float(lora_scale), bias_ptr, _dev(out, torch.bfloat16, "out"), ldy, workspace.ptr, workspace.nbytes, _stream()))
    return out
