"""CPU oracle for the NVFP4 + LoRA linear layer fed by a noisy RMSNorm (QeRL).

THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  It is a plain, slow, numpy
restatement of what the hot path computes, written from the paper's
definitions.  Only the test-suite, the smoke check and the benchmark's
`cpu_baseline` leg may import it.  It shares no code, table or constant
generator with the HIP library and never imports it.

What each function follows
--------------------------
* FP4 E2M1 element (1 sign, 2 exponent, 1 mantissa bit, largest magnitude 6):
  "Model Quantization" paragraph of the Preliminary section.
* NVFP4 tensor = E2M1 codes + one FP8 E4M3 scale per 16 elements + one FP32
  per-tensor scale, and the dequantisation  W_hat = S_FP32 * (S_E4M3 (.) W~):
  Section 3.3, "NVFP4 Quantization", Eq. (6).
* LoRA branch  W + B A  with B in R^{d x r}, A in R^{r x k}: Preliminary,
  "Low-rank Adaptation", Eq. (2); the alpha/r factor is Algorithm 1's
  "LoRA rank, LoRA alpha" inputs.
* Noisy RMSNorm  (Z + w) (.) x / sqrt(mean(x^2) + delta): Section 3.3,
  "Noise Merging", Eq. (10); Appendix "Proof of Noise Sharing".
* Exponential sigma schedule: Section 3.3, Eq. (8); stage 0 is noise-free
  (Algorithm 1, "Set noise level").  Linear, cosine and logarithmic decay are
  named in the scheduler ablation without formulas; the readings are stated
  at aqn_sigma_schedule.
* Backward pass of the layer (the paper optimises A and B only and
  backpropagates through the frozen quantised weights: Preliminary,
  "Low-rank Adaptation"): nvfp4_lora_linear_backward.
* Gated input of the down projection, SiLU(gate) (.) up: the feed-forward
  block of the architectures the paper adapts (Preliminary, "Low-rank
  Adaptation" names W_gate, W_up, W_down); reading stated at silu_mul.
* Noise vector Z ~ N(0, sigma^2 I), drawn anew per forward pass: Section
  3.3, "Adaptive Quantization Noise".  The paper fixes the distribution, not
  the generator; aqn_noise_philox states the counter-based construction both
  sides of this build implement.

The paper states only the *de*quantisation.  The quantisation rule used here
is the round-to-nearest scale chain this build was asked to follow:
    S_FP32 = amax / (6 * 448)
    S_E4M3 = E4M3( block_amax / 6 / S_FP32 )        (per 16 along K)
    code   = E2M1( w / (S_FP32 * S_E4M3) )
evaluated in IEEE fp32, each operation correctly rounded, in exactly that
order, with round-to-nearest-even onto both grids and saturation at the
largest finite value.  Every reading taken where the paper is silent is
listed next to the function that takes it.

Conventions: W is [N, K] (out x in), K contiguous, blocks of 16 run along K.
bf16 tensors are passed as float32 numpy arrays whose values are
bf16-representable.  Parity status: every function here is pinned by
tests that run without a GPU (tests/test_oracle_*.py); none is "parity
unpinned".
"""
from __future__ import annotations

import math

import numpy as np

BLOCK = 16  # elements sharing one E4M3 scale (Section 3.3 / Preliminary)

# --- E2M1: sign(1) exponent(2) mantissa(1), bias 1, no Inf/NaN ---------------
# magnitude index i = (exponent << 1) | mantissa, i = 0..7
#   exponent 0 (subnormal): mantissa * 0.5          -> 0, 0.5
#   exponent e >= 1       : (1 + mantissa/2) * 2^(e-1) -> 1, 1.5, 2, 3, 4, 6
E2M1_GRID = np.array(
    [(m * 0.5) if e == 0 else (1.0 + m / 2.0) * 2.0 ** (e - 1)
     for e in range(4) for m in range(2)],
    dtype=np.float64,
)

# --- E4M3 (OCP FP8, "FN" flavour): sign(1) exponent(4) mantissa(3), bias 7 ---
# exponent 0: (m/8) * 2^-6 ; else (1 + m/8) * 2^(e-7); 0x7F is NaN, 0x7E = 448.
E4M3_GRID = np.array(
    [((b & 7) / 8.0) * 2.0 ** -6 if (b >> 3) == 0
     else (1.0 + (b & 7) / 8.0) * 2.0 ** ((b >> 3) - 7)
     for b in range(0x7F)],
    dtype=np.float64,
)  # index = byte value 0x00..0x7E, strictly increasing, last = 448


def e2m1_decode(code):
    """4-bit code -> value (float32).  Bit 3 is the sign."""
    code = np.asarray(code, dtype=np.uint8)
    mag = E2M1_GRID[code & 7].astype(np.float32)
    return np.where((code >> 3) & 1, -mag, mag).astype(np.float32)


def e4m3_decode(byte):
    """E4M3 byte (sign bit clear, not NaN) -> value (float32)."""
    byte = np.asarray(byte, dtype=np.uint8)
    if np.any(byte > 0x7E):
        raise ValueError("scale bytes are non-negative finite E4M3 (0x00..0x7E)")
    return E4M3_GRID[byte].astype(np.float32)


def round_to_grid_rne(v, grid):
    """Index of the grid point nearest to v >= 0; ties go to the even index;
    v beyond the last point saturates to it.

    `grid` is increasing and starts at 0.  For both formats above the index
    parity equals the parity of the mantissa's last bit, so "even index" is
    round-half-to-even.  Distances are taken in float64, where they are exact
    for every float32 v between two neighbouring grid points.
    """
    v = np.asarray(v, dtype=np.float64)
    if np.any(~np.isfinite(v)) or np.any(v < 0):
        raise ValueError("round_to_grid_rne expects finite non-negative input")
    last = len(grid) - 1
    hi = np.clip(np.searchsorted(grid, v, side="left"), 0, last)  # grid[hi] >= v (or last)
    lo = np.clip(hi - 1, 0, last)
    d_lo = v - grid[lo]
    d_hi = grid[hi] - v
    take_hi = (d_hi < d_lo) | ((d_hi == d_lo) & (hi % 2 == 0))
    idx = np.where(take_hi, hi, lo)
    idx = np.where(v >= grid[last], last, idx)
    return idx.astype(np.uint8)


def e4m3_encode(v):
    """float32 v >= 0 -> E4M3 byte, round-to-nearest-even incl. subnormals,
    saturating at 448 (0x7E)."""
    return round_to_grid_rne(v, E4M3_GRID)


def e2m1_encode_magnitude(a):
    """|q| -> 3-bit magnitude index, round-to-nearest-even, saturating at 6."""
    return round_to_grid_rne(a, E2M1_GRID)


def nvfp4_quantize(W):
    """W[N,K] (bf16 values held in float32) -> (codes[N,K/2] u8,
    scales[N,K/16] u8, tensor_scale float32).

    Readings where the paper is silent:
      * all arithmetic is fp32 and follows the chain in the module header
        left to right (6*448 is the constant 2688);
      * amax == 0  ->  tensor_scale = 1, every byte 0 except sign bits;
      * a block whose scale byte is 0 encodes magnitude 0 everywhere;
      * the code's sign bit is the input's sign bit (also for zeros);
      * low nibble = even k, high nibble = odd k; scales row-major.
    """
    W = np.ascontiguousarray(W, dtype=np.float32)
    if W.ndim != 2 or W.shape[1] % BLOCK != 0:
        raise ValueError("W must be [N, K] with K a multiple of 16")
    if not np.all(np.isfinite(W)):
        raise ValueError("non-finite weights are not supported")
    N, K = W.shape
    f32 = np.float32
    absW = np.abs(W)
    amax = f32(absW.max()) if W.size else f32(0)
    tensor_scale = f32(1.0) if amax == 0 else f32(amax / f32(2688.0))

    blocks = absW.reshape(N, K // BLOCK, BLOCK)
    bamax = blocks.max(axis=2).astype(f32)                     # [N, K/16]
    v = ((bamax / f32(6.0)).astype(f32) / tensor_scale).astype(f32)
    scales = e4m3_encode(v)                                    # u8 [N, K/16]

    d = (tensor_scale * e4m3_decode(scales)).astype(f32)       # [N, K/16]
    d_full = np.repeat(d, BLOCK, axis=1)                       # [N, K]
    with np.errstate(divide="ignore", invalid="ignore"):
        q = (absW / d_full).astype(f32)
    q = np.where(d_full == 0, f32(0), q)
    if not np.all(np.isfinite(q)):
        raise ValueError("w / (tensor_scale * block_scale) overflowed fp32")
    mag = e2m1_encode_magnitude(q)
    sign = np.signbit(W).astype(np.uint8)
    code = (mag | (sign << 3)).astype(np.uint8)                # [N, K]
    codes = (code[:, 0::2] | (code[:, 1::2] << 4)).astype(np.uint8)
    return codes, scales, tensor_scale


def nvfp4_dequantize(codes, scales, tensor_scale):
    """Eq. (6): W_hat = S_FP32 * (S_E4M3 (.) W~), evaluated in fp32.
    The inner product of an E4M3 and an E2M1 value is exact in fp32."""
    codes = np.asarray(codes, dtype=np.uint8)
    scales = np.asarray(scales, dtype=np.uint8)
    N, K2 = codes.shape
    K = 2 * K2
    if scales.shape != (N, K // BLOCK):
        raise ValueError("scales must be [N, K/16]")
    code = np.empty((N, K), dtype=np.uint8)
    code[:, 0::2] = codes & 0x0F
    code[:, 1::2] = codes >> 4
    inner = (np.repeat(e4m3_decode(scales), BLOCK, axis=1) * e2m1_decode(code)).astype(np.float32)
    return (np.float32(tensor_scale) * inner).astype(np.float32)


def lora_down_projection(x, A, acc_dtype=np.float64):
    """t[M,r] = x . A^T: the inner factor of the low-rank branch B A x (Eq. 2), in
    `acc_dtype`, not rounded.  x[M,K], A[r,K] hold bf16 values in float32."""
    x = np.asarray(x, dtype=np.float32).astype(acc_dtype)
    A = np.asarray(A, dtype=np.float32).astype(acc_dtype)
    return x @ A.T


def nvfp4_lora_linear(x, codes, scales, tensor_scale, A=None, B=None,
                      lora_scale=0.0, acc_dtype=np.float64, bias=None):
    """y[M,N] = x . W_hat^T + lora_scale * (x . A^T) . B^T (+ bias[N])     (Eq. 2 + Eq. 6)

    bias: the additive vector the q/k/v projections of the Qwen2.5 blocks carry (the paper's
    equations show none; a linear layer's bias is added to every output row, before any
    rounding).

    x[M,K], A[r,K], B[N,r] hold bf16 values in float32.  W_hat is the fp32
    dequantisation; products and sums run in `acc_dtype` (float64 by default;
    float32 gives the paper-precision variant).  t = x A^T is not rounded
    between the two LoRA products, and the result is not rounded to bf16:
    the caller compares against it with the stated tolerance.
    """
    x = np.asarray(x, dtype=np.float32).astype(acc_dtype)
    W_hat = nvfp4_dequantize(codes, scales, tensor_scale).astype(acc_dtype)
    y = x @ W_hat.T
    if A is not None and B is not None and np.asarray(A).shape[0] > 0:
        B = np.asarray(B, dtype=np.float32).astype(acc_dtype)
        t = lora_down_projection(x, A, acc_dtype)
        y = y + acc_dtype(lora_scale) * (t @ B.T)
    if bias is not None:
        y = y + np.asarray(bias, dtype=np.float32).astype(acc_dtype)[None, :]
    return y


def nvfp4_lora_linear_backward(x, dy, codes, scales, tensor_scale, A=None, B=None, lora_scale=0.0):
    """Gradients of  y = x W_hat^T + s (x A^T) B^T  (Eq. 2 + Eq. 6, s = lora_scale) for an upstream dL/dy = dy:

        dx = dy W_hat + s (dy B) A          [M, K]     (W_hat is frozen: it gets no gradient)
        dA = s (dy B)^T x                   [r, K]
        dB = s dy^T (x A^T)                 [N, r]

    The paper trains only the LoRA matrices and backpropagates through the quantised weights
    (Preliminary, "Low-rank Adaptation": W frozen, A and B optimised; Section 3.1: gradient
    backpropagation through the LoRA layers); it prints no formulas for the gradients, these are the plain
    matrix-calculus ones.  float64 throughout, nothing rounded.  Returns (dx, dA, dB); dA and dB are None
    without an adapter.
    """
    x = np.asarray(x, dtype=np.float32).astype(np.float64)
    dy = np.asarray(dy, dtype=np.float32).astype(np.float64)
    W_hat = nvfp4_dequantize(codes, scales, tensor_scale).astype(np.float64)
    dx = dy @ W_hat
    if A is None or B is None or np.asarray(A).shape[0] == 0:
        return dx, None, None
    A = np.asarray(A, dtype=np.float32).astype(np.float64)
    B = np.asarray(B, dtype=np.float32).astype(np.float64)
    s = np.float64(lora_scale)
    u = dy @ B                      # [M, r]
    t = x @ A.T                     # [M, r]
    return dx + s * (u @ A), s * (u.T @ x), s * (dy.T @ t)


def nvfp4_lora_linear_backward_group(x, members):
    """Backward of several linears that read the same x (the q / k / v or gate / up projections of a block:
    Section 3.3; Preliminary, "Low-rank Adaptation"): the loss sees x through every member, so

        dx = sum_i [ dy_i W_hat_i + s_i (dy_i B_i) A_i ]        [M, K]

    while each member's adapter gradients depend on its own dy_i only.  members: dicts with dy, codes, scales,
    tensor_scale and optionally A, B, lora_scale.  float64, nothing rounded.  Returns (dx, [(dA_i, dB_i)]).
    """
    x64 = np.asarray(x, dtype=np.float32).astype(np.float64)
    dx = np.zeros_like(x64)
    grads = []
    for mem in members:
        dy = np.asarray(mem["dy"], dtype=np.float32).astype(np.float64)
        dx += dy @ nvfp4_dequantize(mem["codes"], mem["scales"], mem["tensor_scale"]).astype(np.float64)
        A, B = mem.get("A"), mem.get("B")
        if A is None or B is None or np.asarray(A).shape[0] == 0:
            grads.append((None, None))
            continue
        A = np.asarray(A, dtype=np.float32).astype(np.float64)
        B = np.asarray(B, dtype=np.float32).astype(np.float64)
        s = np.float64(mem.get("lora_scale", 0.0))
        u = dy @ B
        dx += s * (u @ A)
        grads.append((s * (u.T @ x64), s * (dy.T @ (x64 @ A.T))))
    return dx, grads


def round_to_bf16(v):
    """fp64 -> nearest bf16 value (ties to even), returned as float64.  bf16 keeps the top 16 bits of an
    IEEE fp32; the inputs met here are far inside the fp32 range, so rounding the fp32 bit pattern is exact
    double rounding-free only if v is first representable in fp32 -- callers pass fp32-exact values or accept
    the (documented) one-ulp ambiguity at bf16 ties."""
    f = np.asarray(v, dtype=np.float64).astype(np.float32)
    b = f.view(np.uint32).astype(np.uint64)
    b = (b + 0x7FFF + ((b >> 16) & 1)) & 0xFFFF0000
    return b.astype(np.uint32).view(np.float32).astype(np.float64).reshape(np.shape(v))


def silu_mul(gate, up):
    """Input of the feed-forward block's down projection: act = SiLU(gate) (.) up, SiLU(g) = g / (1 + e^-g).

    The paper adapts W_gate, W_up and W_down of each block (Preliminary, "Low-rank Adaptation") of the
    Qwen2.5 / LLaMA architectures it cites, whose feed-forward block is down(SiLU(gate(x)) (.) up(x)); it
    does not restate the gating.  Reading: the roundings of a bf16 model evaluated operator by operator --
    gate and up arrive as bf16 values, SiLU(gate) is rounded to bf16, the product is rounded to bf16 -- with
    the function itself evaluated exactly (float64 here).  Returns bf16 values in float64.
    """
    g = np.asarray(gate, dtype=np.float32).astype(np.float64)
    u = np.asarray(up, dtype=np.float32).astype(np.float64)
    s = round_to_bf16(g / (1.0 + np.exp(-g)))
    return round_to_bf16(s * u)


def aqn_rmsnorm(x, gain, noise=None, eps=1e-6):
    """Eq. (10): y = (gain + noise) (.) x / sqrt(mean_k(x^2) + eps), float64.

    Readings: eps sits inside the square root; gain + noise is formed in
    full precision (it is not re-rounded to bf16); noise=None is stage 0
    (sigma = 0) and gives the plain RMSNorm; no intermediate rounding.
    """
    x = np.asarray(x, dtype=np.float32).astype(np.float64)
    g = np.asarray(gain, dtype=np.float32).astype(np.float64)
    if noise is not None:
        g = g + np.asarray(noise, dtype=np.float32).astype(np.float64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return g * x / np.sqrt(ms + np.float64(eps))


def aqn_sigma(stage, num_stages, sigma_start, sigma_end):
    """Eq. (8): sigma(k) = s0 * (s1/s0)^((k-1)/(K-1)) for k = 1..K;
    stage 0 returns 0 (Algorithm 1: only quantisation noise acts there)."""
    if stage < 0 or stage > num_stages or num_stages < 1:
        raise ValueError("stage must be in 0..num_stages")
    if stage == 0:
        return 0.0
    if num_stages == 1:
        return float(sigma_start)
    return float(sigma_start) * (float(sigma_end) / float(sigma_start)) ** (
        (stage - 1) / (num_stages - 1))


# --- scheduler ablation (Section 4 "Noise Scheduler", Appendix on schedulers) --------------
SCHEDULE_KINDS = ("exponential", "linear", "cosine", "logarithmic")


def aqn_sigma_schedule(kind, stage, num_stages, sigma_start, sigma_end):
    """sigma at stage k = 1..K for the four decay curves the paper compares; k = 0 -> 0.

    Only the exponential curve has a formula in the paper (Eq. 8).  Readings for the
    other three, each running from sigma_start at k = 1 to sigma_end at k = K with
    u = (k - 1) / (K - 1):
      linear       s0 + (s1 - s0) u
      cosine       s1 + (s0 - s1) (1 + cos(pi u)) / 2          (half-cosine anneal)
      logarithmic  s0 + (s1 - s0) ln(1 + (k - 1)) / ln(K)      (fast early decay)
    """
    if kind not in SCHEDULE_KINDS:
        raise ValueError("unknown schedule")
    if kind == "exponential":
        return aqn_sigma(stage, num_stages, sigma_start, sigma_end)
    if stage < 0 or stage > num_stages or num_stages < 1:
        raise ValueError("stage must be in 0..num_stages")
    if stage == 0:
        return 0.0
    if num_stages == 1:
        return float(sigma_start)
    s0, s1 = float(sigma_start), float(sigma_end)
    u = (stage - 1) / (num_stages - 1)
    if kind == "linear":
        return s0 + (s1 - s0) * u
    if kind == "cosine":
        return s1 + (s0 - s1) * (1.0 + math.cos(math.pi * u)) / 2.0
    return s0 + (s1 - s0) * math.log(1.0 + (stage - 1)) / math.log(num_stages)


# --- noise vector: counter-based generator + Box-Muller ---------------------------------
_PHILOX_M0, _PHILOX_M1 = 0xD2511F53, 0xCD9E8D57          # multipliers
_PHILOX_W0, _PHILOX_W1 = 0x9E3779B9, 0xBB67AE85          # key increments (golden ratio, sqrt 3 - 1)


def philox4x32_10(counter, key):
    """Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as
    easy as 1, 2, 3", SC'11).  counter: uint32 [n, 4]; key: two uint32.  Returns uint32 [n, 4].

    One round maps (c0, c1, c2, c3) to
        (hi(M1 c2) ^ c1 ^ k0,  lo(M1 c2),  hi(M0 c0) ^ c3 ^ k1,  lo(M0 c0))
    and the key is bumped by (W0, W1) before every round but the first."""
    c = np.asarray(counter, dtype=np.uint64).reshape(-1, 4).copy()
    k0, k1 = int(key[0]) & 0xFFFFFFFF, int(key[1]) & 0xFFFFFFFF
    mask = np.uint64(0xFFFFFFFF)
    for rnd in range(10):
        if rnd:
            k0 = (k0 + _PHILOX_W0) & 0xFFFFFFFF
            k1 = (k1 + _PHILOX_W1) & 0xFFFFFFFF
        p0 = np.uint64(_PHILOX_M0) * c[:, 0]
        p1 = np.uint64(_PHILOX_M1) * c[:, 2]
        c = np.stack([(p1 >> np.uint64(32)) ^ c[:, 1] ^ np.uint64(k0), p1 & mask,
                      (p0 >> np.uint64(32)) ^ c[:, 3] ^ np.uint64(k1), p0 & mask], axis=1)
    return c.astype(np.uint32)


def aqn_noise_philox(n, sigma, seed, subsequence):
    """Z[i] ~ N(0, sigma^2), i < n, float64 (the device rounds the same values to fp32).

    Construction (this build's; the paper fixes only the distribution): elements come in
    groups of four.  Group b uses counter (b mod 2^32, b >> 32, subsequence mod 2^32,
    subsequence >> 32) and key (seed mod 2^32, seed >> 32); the four outputs r0..r3 give two
    Box-Muller pairs from 24-bit uniforms (exact in fp32):
        u1 = ((r0 >> 8) + 1) 2^-24 in (0, 1],  u2 = (r1 >> 8) 2^-24 in [0, 1)
        z0 = sqrt(-2 ln u1) cos(2 pi u2),      z1 = sqrt(-2 ln u1) sin(2 pi u2)
    and likewise (r2, r3) -> (z2, z3);  Z[4 b + j] = sigma z_j.  A new forward pass takes a
    new subsequence; a new run a new seed."""
    n = int(n)
    nb = (n + 3) // 4
    b = np.arange(nb, dtype=np.uint64)
    ctr = np.stack([b & np.uint64(0xFFFFFFFF), b >> np.uint64(32),
                    np.full(nb, int(subsequence) & 0xFFFFFFFF, dtype=np.uint64),
                    np.full(nb, (int(subsequence) >> 32) & 0xFFFFFFFF, dtype=np.uint64)], axis=1)
    r = philox4x32_10(ctr, (int(seed) & 0xFFFFFFFF, (int(seed) >> 32) & 0xFFFFFFFF)).astype(np.float64)
    z = np.empty((nb, 4), dtype=np.float64)
    for pair in range(2):
        u1 = (np.floor(r[:, 2 * pair] / 256.0) + 1.0) * 2.0 ** -24
        u2 = np.floor(r[:, 2 * pair + 1] / 256.0) * 2.0 ** -24
        radius = np.sqrt(-2.0 * np.log(u1))
        z[:, 2 * pair] = radius * np.cos(2.0 * np.pi * u2)
        z[:, 2 * pair + 1] = radius * np.sin(2.0 * np.pi * u2)
    return float(sigma) * z.reshape(-1)[:n]

