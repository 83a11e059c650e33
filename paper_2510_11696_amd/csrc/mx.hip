// MXFP4 variant of the weight-only linear on CDNA4's scaled matrix instruction.
//
// Format (Preliminary, "Model Quantization"): FP4 E2M1 elements with one shared FP8 E8M0 scale -- a
// bare power of two -- per block of 32 elements; blocks run along K.  The paper evaluates it next to
// NVFP4 and states no conversion rule; this file follows the OCP Microscaling (MX) v1.0 conversion:
//   X = floor(log2(block max |v|)) - emax_elem   (emax_elem = 2 for E2M1, 8 for E4M3), clamped to
//   [-127, 127]; scale byte = X + 127; element = round-to-nearest-even of v / 2^X, saturating.
//
// v_mfma_scale_f32_32x32x64_f8f6f4 multiplies a 32 x 64 block of FP8/FP6/FP4 values by a 64 x 32 one and
// scales each block of 32 consecutive K elements of a row (column) by an E8M0 byte -- exactly an MX block.
// Operand order, as measured with one-hot inputs: registers are filled 16 bytes at a time, chunk c of lane
// l = (row l % 32, g = l / 32) being K-chunk 2 c + g.  An FP8 operand (two chunks of 16 elements per lane) thus
// holds inputs 16 g .. 16 g + 15 and 32 + 16 g .. 32 + 16 g + 15; an FP4 operand (one chunk of 32 elements)
// inputs 32 g .. 32 g + 31.  The scale bytes of lanes 0..31 belong to inputs 0..31, those of lanes 32..63 to
// inputs 32..63, for both operands.  So
// MXFP4 weights enter the matrix unit as stored: no conversion instruction, no scaling arithmetic.
// The price is the other operand: it has to be FP8/FP6/FP4 too.  mxfp4_linear_native therefore
// quantises the activations to MXFP8 (E4M3 elements, E8M0 per 32 along K) first -- which the paper
// does NOT do (its kernels keep bf16 activations); the result is the exact product of the two quantised
// operands, and how far that is from the weight-only result is measured in the tests, not assumed.
//
// Kernels:
//   mxfp4_quantize_kernel / mxfp8_quantize_kernel   one thread per block of 32 (bit-exact vs the rule)
//   mxfp4_prepack_kernel   canonical (codes [N, K/2], scales [N, K/32]) -> tiles of 32 rows x 128 inputs,
//                          2176 bytes: two steps of 64 inputs, each 1 KiB of codes (lane l = (n = l % 32,
//                          g = l / 32) owns the 16 bytes of inputs 64 s + 32 g .. + 31 of row n) and 64
//                          scale bytes (one per lane: the scale of those 32 inputs), i.e. MFMA operand order
//   mx_native_kernel       decode-sized batches (M <= 32): a workgroup's eight waves split the 64-input
//                          steps of its K-range and keep their x fragments in registers; each wave
//                          streams its steps of one row-tile after the other (the next tile's loads in
//                          flight while the current one is multiplied), the eight partial tiles are added
//                          through LDS in wave order.  Bound by streaming the packed weights:
//                          0.53125 B per weight.
#include "common.hpp"

namespace qerl {

typedef int v8i __attribute__((ext_vector_type(8)));

constexpr int kMxTileBytes = 2176;      // 32 rows x 128 inputs: 2 x 1024 B codes + 2 x 64 B scales
constexpr int kMxWaves = 8;
constexpr int kMxMaxSteps = 8;          // 64-input steps per wave and K-range held in registers

// ---- quantisers -----------------------------------------------------------------------------------
// One thread per block of 32 bf16 values.  EMAX: 2 (E2M1 elements, two per byte out) or 8 (E4M3, one per byte).
template <int EMAX>
__global__ __launch_bounds__(256) void mx_quantize_kernel(const uint16_t* __restrict__ V, int64_t R, int64_t K, int64_t ld,
                                                          uint8_t* __restrict__ codes, uint8_t* __restrict__ scales) {
  const int64_t blocks_per_row = K / 32;
  const int64_t total = R * blocks_per_row;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int64_t row = i / blocks_per_row, b = i - row * blocks_per_row;
    const uint16_t* src = V + row * ld + b * 32;
    uint32_t w[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) w[j] = reinterpret_cast<const uint32_t*>(src)[j];
    uint32_t m = 0;                       // largest magnitude as a bf16 bit pattern (integer order = magnitude order)
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const uint32_t lo = w[j] & 0x7fffu, hi = (w[j] >> 16) & 0x7fffu;
      m = lo > m ? lo : m;
      m = hi > m ? hi : m;
    }
    // floor(log2(amax)) = exponent field - 127 for normal values; X + 127 = field - EMAX, clamped at 0 (which
    // also covers subnormal maxima and the all-zero block)
    const int field = (int)(m >> 7);
    const int sbyte = field - EMAX > 0 ? field - EMAX : 0;
    const float inv = __uint_as_float((uint32_t)(254 - sbyte) << 23);   // 2^-(sbyte - 127), a normal fp32 for every sbyte <= 253
    scales[row * blocks_per_row + b] = (uint8_t)sbyte;
    if (EMAX == 2) {
      uint32_t out[4];
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        uint32_t acc = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const uint32_t pair = w[4 * d + j];
          const float a = bf16_bits_to_f32(pair & 0x7fffu) * inv, c = bf16_bits_to_f32((pair >> 16) & 0x7fffu) * inv;
          const uint32_t n0 = e2m1_encode_rne_sat(a) | ((pair >> 12) & 8u);
          const uint32_t n1 = e2m1_encode_rne_sat(c) | ((pair >> 28) & 8u);
          acc |= (n0 | (n1 << 4)) << (8 * j);
        }
        out[d] = acc;
      }
      uint32_t* dst = reinterpret_cast<uint32_t*>(codes + row * (K / 2) + b * 16);
#pragma unroll
      for (int d = 0; d < 4; ++d) dst[d] = out[d];
    } else {
      uint32_t* dst = reinterpret_cast<uint32_t*>(codes + row * K + b * 32);
#pragma unroll
      for (int d = 0; d < 8; ++d) {
        uint32_t acc = 0;
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const uint32_t pair = w[2 * d + j];
          const float a = bf16_bits_to_f32(pair & 0x7fffu) * inv, c = bf16_bits_to_f32((pair >> 16) & 0x7fffu) * inv;
          const uint32_t b0 = e4m3_encode_rne_sat(a) | ((pair >> 8) & 0x80u);
          const uint32_t b1 = e4m3_encode_rne_sat(c) | ((pair >> 24) & 0x80u);
          acc |= (b0 | (b1 << 8)) << (16 * j);
        }
        dst[d] = acc;
      }
    }
  }
}

__global__ __launch_bounds__(256) void mxfp4_dequantize_kernel(const uint8_t* __restrict__ codes, const uint8_t* __restrict__ scales,
                                                               int64_t N, int64_t K, float* __restrict__ W) {
  const int64_t total = N * (K / 2);
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int64_t row = i / (K / 2), c = i - row * (K / 2);
    const uint32_t byte = codes[i];
    const uint32_t sb = scales[row * (K / 32) + c / 16];
    const float s = sb ? __uint_as_float(sb << 23) : 0x1p-127f;   // 2^(byte - 127); for byte 0 that is an fp32 subnormal
    W[row * K + 2 * c] = e2m1_to_f32(byte & 0xFu) * s;
    W[row * K + 2 * c + 1] = e2m1_to_f32(byte >> 4) * s;
  }
}

// ---- prepack ----------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void mxfp4_prepack_kernel(const uint8_t* __restrict__ codes, const uint8_t* __restrict__ scales,
                                                            int64_t N, int64_t K, int64_t n_tiles, int64_t k_tiles, uint8_t* __restrict__ out) {
  // one thread per (tile, step, lane): 16 code bytes and one scale byte
  const int64_t total = n_tiles * k_tiles * 2 * 64;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int lane = (int)(i & 63), s = (int)((i >> 6) & 1);
    const int64_t tile = i >> 7, kt = tile % k_tiles, nt = tile / k_tiles;
    const int64_t n = nt * 32 + (lane & 31), k0 = kt * 128 + 64 * s + 32 * (lane >> 5);
    u32x4 c = {0u, 0u, 0u, 0u};
    uint8_t sc = 0;
    if (n < N && k0 < K) {               // K % 32 == 0: a block is inside or outside as a whole
      c = *reinterpret_cast<const u32x4*>(codes + n * (K / 2) + k0 / 2);
      sc = scales[n * (K / 32) + k0 / 32];
    }
    uint8_t* t = out + tile * kMxTileBytes;
    *reinterpret_cast<u32x4*>(t + s * 1024 + lane * 16) = c;
    t[2048 + s * 64 + lane] = sc;
  }
}

// ---- the linear ---------------------------------------------------------------------------------------
struct MxArgs {
  const uint8_t* xq; const uint8_t* xs; int M; int64_t K;      // MXFP8 activations: codes [M, K], scales [M, K/32]
  const uint8_t* packed; int k_tiles; int n_tiles; int64_t N;
  uint16_t* y; int64_t ldy;
  float* partial;                                               // [Sk][n_tiles][MR][64] when Sk > 1
  int Sk; int steps_per_range; int per_range; int units_base; int units_rem;
};

// NS: 64-input steps per wave; MR: accumulator registers with live tokens (4: M <= 8, 16: M <= 32)
template <int NS, int MR>
__global__ __launch_bounds__(kMxWaves * 64) void mx_native_kernel(const MxArgs a) {
  __shared__ float red[2][kMxWaves][MR][64];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n32 = lane & 31, kg = lane >> 5;
  const int range = (int)blockIdx.x / a.per_range, ci = (int)blockIdx.x - range * a.per_range;
  const int n_units = a.units_base + (ci < a.units_rem ? 1 : 0);
  const int u0 = ci * a.units_base + (ci < a.units_rem ? ci : a.units_rem);
  const int n_steps = 2 * a.k_tiles;                                   // 64-input steps of the padded K
  const int step0 = range * a.steps_per_range;                         // this range: steps [step0, step0 + 8 NS)

  // ---- this wave's steps: step0 + wave + 8 i; x fragments and scales stay in registers
  v8i xa[NS];
  int xsc[NS];
#pragma unroll
  for (int i = 0; i < NS; ++i) {
    const int s = step0 + wave + kMxWaves * i;
    const int64_t kb = (int64_t)s * 64, ka = kb + 16 * kg, kc = kb + 32 + 16 * kg, ks = kb + 32 * kg;
    u32x4 lo = {0u, 0u, 0u, 0u}, hi = {0u, 0u, 0u, 0u};   // a step past the end of K, or a row past the tokens: zeros
    xsc[i] = 0;
    if (s < n_steps && n32 < a.M) {
      if (ka < a.K) lo = *reinterpret_cast<const u32x4*>(a.xq + (int64_t)n32 * a.K + ka);
      if (kc < a.K) hi = *reinterpret_cast<const u32x4*>(a.xq + (int64_t)n32 * a.K + kc);
      if (ks < a.K) xsc[i] = a.xs[(int64_t)n32 * (a.K / 32) + ks / 32];
    }
    xa[i] = v8i{(int)lo[0], (int)lo[1], (int)lo[2], (int)lo[3], (int)hi[0], (int)hi[1], (int)hi[2], (int)hi[3]};
  }
  // ---- weights: this wave's steps of one row-tile = NS loads of 16 bytes + NS scale bytes per lane
  struct WTile { u32x4 c[NS]; uint32_t sc[NS]; };
  auto issue = [&](WTile& t, int u) {
    const int nt = u0 + (u < n_units ? u : n_units - 1);               // past the end: the last tile again (keeps the loads unconditional)
    const uint8_t* base = a.packed + (int64_t)nt * a.k_tiles * kMxTileBytes;
#pragma unroll
    for (int i = 0; i < NS; ++i) {
      int s = step0 + wave + kMxWaves * i;
      s = s < n_steps ? s : n_steps - 1;                               // a dead step multiplies a zero x fragment
      const uint8_t* tile = base + (int64_t)(s >> 1) * kMxTileBytes;
      t.c[i] = *reinterpret_cast<const u32x4*>(tile + (s & 1) * 1024 + lane * 16);
      t.sc[i] = tile[2048 + (s & 1) * 64 + lane];
    }
  };
  auto multiply = [&](const WTile& t, float (&out)[MR]) {
    f32x16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < NS; ++i) {
      const v8i b = v8i{(int)t.c[i][0], (int)t.c[i][1], (int)t.c[i][2], (int)t.c[i][3], 0, 0, 0, 0};
      // A = activations (FP8 E4M3, cbsz 0), B = weights (FP4 E2M1, blgp 4); byte 0 of each lane's scale register
      acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(xa[i], b, acc, 0, 4, 0, xsc[i], 0, (int)t.sc[i]);
    }
#pragma unroll
    for (int q = 0; q < MR; ++q) out[q] = acc[q];
  };
  if (n_units == 0) return;                                            // uniform per workgroup
  WTile t0, t1;
  issue(t0, 0);
  issue(t1, 1);
  for (int u = 0; u < n_units; u += 2) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      if (u + h >= n_units) break;
      float part[MR];
      if (h == 0) { multiply(t0, part); issue(t0, u + 2); }
      else { multiply(t1, part); issue(t1, u + 3); }
      // the eight waves' partial tiles, added in wave order by the first MR * 64 threads
      float (*rb)[MR][64] = red[h];
#pragma unroll
      for (int q = 0; q < MR; ++q) rb[wave][q][lane] = part[q];
      __syncthreads();
      const int nt = u0 + u + h;
      for (int e = tid; e < MR * 64; e += kMxWaves * 64) {
        const int q = e >> 6, l = e & 63;
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < kMxWaves; ++w) sum += rb[w][q][l];
        const int tok = 8 * (q >> 2) + 4 * (l >> 5) + (q & 3);
        const int64_t n = (int64_t)nt * 32 + (l & 31);
        if (a.Sk > 1) a.partial[(((int64_t)range * a.n_tiles + nt) * MR + q) * 64 + l] = sum;
        else if (tok < a.M && n < a.N) a.y[(int64_t)tok * a.ldy + n] = (uint16_t)f32_to_bf16_bits(sum);
      }
      // red[h] is written again two units later, after the barrier of unit u + h + 1: every read above is done by then
    }
  }
}

template <int MR>
__global__ __launch_bounds__(256) void mx_reduce_kernel(const float* partial, int Sk, int n_tiles, int M, int64_t N, uint16_t* y, int64_t ldy) {
  const int nt = blockIdx.x;
  for (int e = threadIdx.x; e < MR * 64; e += 256) {
    const int q = e >> 6, l = e & 63;
    float sum = 0.f;
    for (int r = 0; r < Sk; ++r) sum += partial[(((int64_t)r * n_tiles + nt) * MR + q) * 64 + l];
    const int tok = 8 * (q >> 2) + 4 * (l >> 5) + (q & 3);
    const int64_t n = (int64_t)nt * 32 + (l & 31);
    if (tok < M && n < N) y[(int64_t)tok * ldy + n] = (uint16_t)f32_to_bf16_bits(sum);
  }
}

static int64_t grid_for(int64_t items) {
  int64_t b = (items + 255) / 256;
  return b < 1 ? 1 : (b > 8192 ? 8192 : b);
}

// workspace of mxfp4_linear_native: activation codes, activation scales, K-range partial tiles
struct MxWorkspace { size_t xq_off, xs_off, partial_off, total; int Sk, NS; };
static MxWorkspace mx_workspace(int64_t M, int64_t N, int64_t K) {
  MxWorkspace w{};
  const int64_t n_steps = 2 * ceil_div(K > 0 ? K : 1, 128);
  w.Sk = (int)ceil_div(n_steps, kMxWaves * kMxMaxSteps);
  w.NS = (int)ceil_div(n_steps, (int64_t)kMxWaves * w.Sk);
  if (w.NS < 4) w.NS = 4;                                              // instantiated: 4..8
  auto al = [](size_t v) { return (v + 255) & ~(size_t)255; };
  const size_t rows = (size_t)(M > 0 ? M : 1), kk = (size_t)(K > 0 ? K : 32);
  w.xq_off = 0;
  w.xs_off = al(rows * kk);
  w.partial_off = w.xs_off + al(rows * (kk / 32));
  w.total = w.partial_off + al((size_t)w.Sk * (size_t)ceil_div(N > 0 ? N : 1, 32) * 16 * 64 * sizeof(float));
  return w;
}

template <int NS, int MR>
static int launch_mx_t(const MxArgs& a, int grid, hipStream_t st) {
  mx_native_kernel<NS, MR><<<dim3((unsigned)grid), dim3(kMxWaves * 64), 0, st>>>(a);
  return launch_status();
}
template <int MR>
static int launch_mx(const MxArgs& a, int NS, int grid, hipStream_t st) {
  switch (NS) {
    case 4: return launch_mx_t<4, MR>(a, grid, st);
    case 5: return launch_mx_t<5, MR>(a, grid, st);
    case 6: return launch_mx_t<6, MR>(a, grid, st);
    case 7: return launch_mx_t<7, MR>(a, grid, st);
    case 8: return launch_mx_t<8, MR>(a, grid, st);
    default: return QERL_ERR_SHAPE;
  }
}

}  // namespace qerl

using namespace qerl;

extern "C" int mxfp4_quantize(const void* W, int64_t N, int64_t K, int64_t ldw, uint8_t* codes, uint8_t* scales, void* stream) {
  if (N < 0 || K < 0 || K % 32 != 0 || ldw < K) return QERL_ERR_SHAPE;
  if (N == 0 || K == 0) return QERL_OK;
  if (!W || !codes || !scales) return QERL_ERR_NULL;
  if (!aligned(W, 4) || ldw % 2 != 0 || !aligned(codes, 4)) return QERL_ERR_ALIGN;
  mx_quantize_kernel<2><<<dim3((unsigned)grid_for(N * (K / 32))), dim3(256), 0, (hipStream_t)stream>>>(
      (const uint16_t*)W, N, K, ldw, codes, scales);
  return launch_status();
}

extern "C" int mxfp8_quantize(const void* x, int64_t M, int64_t K, int64_t ldx, uint8_t* codes, uint8_t* scales, void* stream) {
  if (M < 0 || K < 0 || K % 32 != 0 || ldx < K) return QERL_ERR_SHAPE;
  if (M == 0 || K == 0) return QERL_OK;
  if (!x || !codes || !scales) return QERL_ERR_NULL;
  if (!aligned(x, 4) || ldx % 2 != 0 || !aligned(codes, 4)) return QERL_ERR_ALIGN;
  mx_quantize_kernel<8><<<dim3((unsigned)grid_for(M * (K / 32))), dim3(256), 0, (hipStream_t)stream>>>(
      (const uint16_t*)x, M, K, ldx, codes, scales);
  return launch_status();
}

extern "C" int mxfp4_dequantize(const uint8_t* codes, const uint8_t* scales, int64_t N, int64_t K, float* W, void* stream) {
  if (N < 0 || K < 0 || K % 32 != 0) return QERL_ERR_SHAPE;
  if (N == 0 || K == 0) return QERL_OK;
  if (!codes || !scales || !W) return QERL_ERR_NULL;
  mxfp4_dequantize_kernel<<<dim3((unsigned)grid_for(N * (K / 2))), dim3(256), 0, (hipStream_t)stream>>>(codes, scales, N, K, W);
  return launch_status();
}

extern "C" size_t mxfp4_prepack_bytes(int64_t N, int64_t K) {
  if (N <= 0 || K <= 0) return 0;
  return (size_t)ceil_div(N, 32) * (size_t)ceil_div(K, 128) * kMxTileBytes;
}

extern "C" int mxfp4_prepack(const uint8_t* codes, const uint8_t* scales, int64_t N, int64_t K, void* packed, void* stream) {
  if (N < 0 || K < 0 || K % 32 != 0) return QERL_ERR_SHAPE;
  if (N == 0 || K == 0) return QERL_OK;
  if (!codes || !scales || !packed) return QERL_ERR_NULL;
  if (!aligned(packed, 16) || !aligned(codes, 16) || (K / 2) % 16 != 0) return QERL_ERR_ALIGN;
  const int64_t nt = ceil_div(N, 32), kt = ceil_div(K, 128);
  mxfp4_prepack_kernel<<<dim3((unsigned)grid_for(nt * kt * 128)), dim3(256), 0, (hipStream_t)stream>>>(codes, scales, N, K, nt, kt,
                                                                                                    (uint8_t*)packed);
  return launch_status();
}

extern "C" size_t mxfp4_linear_native_workspace_bytes(int64_t M, int64_t N, int64_t K) { return mx_workspace(M, N, K).total; }

extern "C" int mxfp4_linear_native(const void* x, int64_t M, int64_t K, int64_t ldx, const void* packed, int64_t N, void* y, int64_t ldy,
                                   void* workspace, size_t workspace_bytes, void* stream) {
  if (M < 0 || M > 32 || N < 0 || K < 0 || K % 32 != 0 || ldx < K || ldy < N || N >= ((int64_t)1 << 24)) return QERL_ERR_SHAPE;
  if (M == 0 || N == 0) return QERL_OK;
  if (K == 0) return QERL_ERR_SHAPE;
  if (!x || !packed || !y) return QERL_ERR_NULL;
  if (!aligned(x, 4) || ldx % 2 != 0 || !aligned(packed, 16) || !aligned(y, 2)) return QERL_ERR_ALIGN;
  const MxWorkspace w = mx_workspace(M, N, K);
  if (!workspace || !aligned(workspace, 256) || workspace_bytes < w.total) return QERL_ERR_WORKSPACE;
  uint8_t* ws = (uint8_t*)workspace;
  hipStream_t st = (hipStream_t)stream;
  mx_quantize_kernel<8><<<dim3((unsigned)grid_for(M * (K / 32))), dim3(256), 0, st>>>((const uint16_t*)x, M, K, ldx, ws + w.xq_off,
                                                                                    ws + w.xs_off);
  int rc = launch_status();
  if (rc != QERL_OK) return rc;
  MxArgs a{};
  a.xq = ws + w.xq_off; a.xs = ws + w.xs_off; a.M = (int)M; a.K = K;
  a.packed = (const uint8_t*)packed; a.k_tiles = (int)ceil_div(K, 128); a.n_tiles = (int)ceil_div(N, 32); a.N = N;
  a.y = (uint16_t*)y; a.ldy = ldy; a.partial = (float*)(ws + w.partial_off);
  a.Sk = w.Sk; a.steps_per_range = kMxWaves * w.NS;
  int per_range = 256 / w.Sk;
  if (per_range < 1) per_range = 1;
  if (per_range > a.n_tiles) per_range = a.n_tiles;
  a.per_range = per_range; a.units_base = a.n_tiles / per_range; a.units_rem = a.n_tiles % per_range;
  const int grid = per_range * w.Sk;
  rc = M <= 8 ? launch_mx<4>(a, w.NS, grid, st) : launch_mx<16>(a, w.NS, grid, st);
  if (rc != QERL_OK || w.Sk == 1) return rc;
  if (M <= 8) mx_reduce_kernel<4><<<dim3((unsigned)a.n_tiles), dim3(256), 0, st>>>(a.partial, w.Sk, a.n_tiles, (int)M, N, a.y, ldy);
  else mx_reduce_kernel<16><<<dim3((unsigned)a.n_tiles), dim3(256), 0, st>>>(a.partial, w.Sk, a.n_tiles, (int)M, N, a.y, ldy);
  return launch_status();
}
