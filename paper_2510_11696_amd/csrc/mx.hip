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
//   mxfp4_prepack_kernel   canonical (codes [N, K/2], scales [N, K/32]) -> tiles of 32 rows x 256 inputs,
//                          4352 bytes: four steps of 64 inputs, each 1 KiB of codes (lane l = (n = l % 32,
//                          g = l / 32) owns the 16 bytes of inputs 64 j + 32 g .. + 31 of row n), then 256
//                          scale bytes: one dword per lane whose byte j is the scale of its 32 inputs of
//                          step j -- the matrix instruction picks the byte by an immediate, so a lane's
//                          four scales arrive with one load and need no arithmetic
//   mx_native_kernel       decode-sized batches (M <= 32): a workgroup's eight waves split the 64-input
//                          steps of its K-range, quantise their x fragments to MXFP8 and keep them in registers; each wave
//                          streams its steps of one row-tile after the other (the next tile's loads in
//                          flight while the current one is multiplied), the seven partial tiles are added
//                          through LDS in wave order by the eighth wave, which also stores.  Bound by streaming the packed weights:
//                          0.53125 B per weight.
//   mx_gemm_kernel         more tokens: x quantised by a launch of mx_quantize_kernel, then a GEMM with
//                          128 x 256 tiles on the same instruction (described at the kernel).
// The LoRA branch of Eq. (2) rides on both: the adapter reads bf16 x (a launch of the NVFP4 path's down-projection
// kernels leaves lora_scale * x A^T as three bf16 terms), and the up-projection is 3 r more input columns on the bf16
// matrix instruction, whose 32 x 32 output layout is the block-scaled one's.
#include "linear.hpp"

namespace qerl {

typedef int v8i __attribute__((ext_vector_type(8)));

constexpr int kMxTileBytes = 4352;      // 32 rows x 256 inputs: 4 x 1024 B codes + 256 B scales
constexpr int kMxWaves = 8;             // seven that stream and multiply, one that adds their partial tiles and stores
constexpr int kMxMain = kMxWaves - 1;
constexpr int kMxMaxGroups = 2;         // tiles (groups of four 64-input steps) per wave and K-range held in registers
constexpr int kMxMaxRank = 128;         // LoRA rank: [hi | mid | lo] is at most 24 chunks of 16 columns, which the eighth wave holds in registers

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
  const int64_t total = n_tiles * k_tiles * 4 * 64;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int lane = (int)(i & 63), j = (int)((i >> 6) & 3);
    const int64_t tile = i >> 8, kt = tile % k_tiles, nt = tile / k_tiles;
    const int64_t n = nt * 32 + (lane & 31), k0 = kt * 256 + 64 * j + 32 * (lane >> 5);
    u32x4 c = {0u, 0u, 0u, 0u};
    uint8_t sc = 0;
    if (n < N && k0 < K) {               // K % 32 == 0: a block is inside or outside as a whole
      c = *reinterpret_cast<const u32x4*>(codes + n * (K / 2) + k0 / 2);
      sc = scales[n * (K / 32) + k0 / 32];
    }
    uint8_t* t = out + tile * kMxTileBytes;
    *reinterpret_cast<u32x4*>(t + j * 1024 + lane * 16) = c;
    t[4096 + lane * 4 + j] = sc;
  }
}

// ---- the linear ---------------------------------------------------------------------------------------
struct MxArgs {
  const uint16_t* x; int64_t ldx; int M; int64_t K;            // bf16 activations: quantised to MXFP8 by the waves that use them
  const uint8_t* packed; int k_tiles; int n_tiles; int64_t N;
  uint16_t* y; int64_t ldy;
  float* partial;                                               // [Sk][n_tiles][MR][64] when Sk > 1
  int Sk; int groups_per_range; int per_range; int units_base; int units_rem;
  // LoRA branch (Eq. 2) and bias: ts [M, ts_ld] bf16 = hi | mid | lo of lora_scale * x A^T (r columns each, zeros up
  // to ts_ld = 16 n_chunks), B [N, r] bf16; n_chunks == 0: no adapter.  bias [N] bf16 or null.
  const uint16_t* ts; int64_t ts_ld; int n_chunks; const uint16_t* B; int r;
  const uint16_t* bias;
};

// The 8 columns [col, col + 8) of [hi | mid | lo] meet the same 8 columns of B in each of the three parts (r % 8 == 0
// keeps a run inside one part); the zero padding past 3 r meets column 0.
__device__ __forceinline__ int lora_b_col(int col, int r) { return col < 3 * r ? col % r : 0; }

// NG: tiles (four 64-input steps each) per wave; MR: accumulator registers with live tokens (4: M <= 8, 16: M <= 32);
// LC: 16-column chunks of ts the eighth wave has registers for (0: no adapter).  The LoRA up-projection is the eighth
// wave's: in the first K-range it adds [hi | mid | lo] . [B B B]^T to the sum of the seven partial tiles with bf16
// matrix instructions of the same 32 x 32 output layout; its ts fragments wait in LDS, B's fragments of the next
// row-tile are requested while the streaming waves work on it.  The streaming waves are untouched.
template <int NG, int MR, int LC>
__global__ __launch_bounds__(kMxWaves * 64) void mx_native_kernel(const MxArgs a) {
  __shared__ float red[2][kMxMain][MR][64];
  __shared__ u32x4 tsl[(LC > 0 ? LC : 1) * 64];                         // chunk c of lane l at c * 64 + l
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n32 = lane & 31, kg = lane >> 5;
  const int range = (int)blockIdx.x / a.per_range, ci = (int)blockIdx.x - range * a.per_range;
  const int n_units = a.units_base + (ci < a.units_rem ? 1 : 0);
  const int u0 = ci * a.units_base + (ci < a.units_rem ? ci : a.units_rem);
  constexpr int NS = 4 * NG;
  const int n_groups = a.k_tiles;                                      // tiles along the padded K
  const int group0 = range * a.groups_per_range;                       // this range: tiles [group0, group0 + 7 NG)

  if (n_units == 0) return;                                            // uniform per workgroup
  const int n_rounds = 2 * ((n_units + 1) / 2);                        // barriers every wave of the workgroup passes
  if (wave == kMxMain) {
    // ---- the eighth wave adds the seven partial tiles of a unit in wave order and stores the result; the
    // streaming waves never store, so their loads are the only memory operations they ever wait for
    constexpr int LCA = LC > 0 ? LC : 1;
    const bool lora = LC > 0 && range == 0;                            // uniform per workgroup
    u32x4 bfr[LCA];
    auto request_b = [&](int u) {                                       // B's fragments of unit u: row n, 8 columns per chunk
      int64_t n = (int64_t)(u0 + (u < n_units ? u : n_units - 1)) * 32 + n32;
      n = n < a.N ? n : a.N - 1;
      const uint16_t* row = a.B + n * a.r;
      int col = 8 * kg % a.r;                                           // (16 c + 8 g) mod r, carried along: r % 8 == 0, so col + 8 <= r
#pragma unroll
      for (int c = 0; c < LCA; ++c) {
        bfr[c] = *reinterpret_cast<const u32x4*>(row + col);            // a chunk past 3 r meets zero ts
        col += 16;
        col = col >= a.r ? col - a.r : col;
        col = col >= a.r ? col - a.r : col;                             // r >= 8: two steps at most
      }
    };
    if (lora) {
#pragma unroll
      for (int c = 0; c < LCA; ++c) {
        u32x4 t = {0u, 0u, 0u, 0u};
        if (c < a.n_chunks && n32 < a.M) t = *reinterpret_cast<const u32x4*>(a.ts + (int64_t)n32 * a.ts_ld + 16 * c + 8 * kg);
        tsl[c * 64 + lane] = t;                                         // read back by this wave only
      }
      request_b(0);
    }
    for (int u = 0; u < n_rounds; ++u) {
      __syncthreads();
      if (u >= n_units) continue;
      const int nt = u0 + u;
      const int64_t n = (int64_t)nt * 32 + n32;
      f32x16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int q = 0; q < MR; ++q) {
        float sum = 0.f;
#pragma unroll
        for (int w = 0; w < kMxMain; ++w) sum += red[u & 1][w][q][lane];
        acc[q] = sum;
      }
      if (lora) {
#pragma unroll
        for (int c = 0; c < LCA; ++c)
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, tsl[c * 64 + lane]), __builtin_bit_cast(bf16x8, bfr[c]), acc, 0, 0, 0);
        request_b(u + 1);                                               // past the end: the last tile again
      }
      const float bias = (a.bias && a.Sk == 1 && n < a.N) ? bf16_bits_to_f32(a.bias[n]) : 0.f;
#pragma unroll
      for (int q = 0; q < MR; ++q) {
        const int tok = 8 * (q >> 2) + 4 * kg + (q & 3);
        if (a.Sk > 1) a.partial[(((int64_t)range * a.n_tiles + nt) * MR + q) * 64 + lane] = acc[q];
        else if (tok < a.M && n < a.N) a.y[(int64_t)tok * a.ldy + n] = (uint16_t)f32_to_bf16_bits(acc[q] + bias);
      }
    }
    return;
  }
  // ---- this wave's tiles along K: group0 + wave + 7 i, four steps each.  Their x fragments are quantised to MXFP8 here, once, and stay in
  // registers with their scales: lane (token, g) reads inputs 16 g .. + 15 (of block 0 of the step) and
  // 32 + 16 g .. + 15 (of block 1); the two lanes of a token exchange their chunk maxima to get both block
  // maxima, and each quantises its own 32 values -- the same function mxfp8_quantize computes.
  v8i xa[NS];
  int xsc[NS];
#pragma unroll
  for (int i = 0; i < NS; ++i) {
    const int grp = group0 + wave + kMxMain * (i >> 2);
    const int64_t kb = (int64_t)grp * 256 + 64 * (i & 3), ka = kb + 16 * kg, kc = kb + 32 + 16 * kg;
    u32x4 v[4] = {{0u, 0u, 0u, 0u}, {0u, 0u, 0u, 0u}, {0u, 0u, 0u, 0u}, {0u, 0u, 0u, 0u}};   // a step past the end of K, or a row past the tokens: zeros
    if (grp < n_groups && n32 < a.M) {
      const uint16_t* row = a.x + (int64_t)n32 * a.ldx;
      if (ka < a.K) { v[0] = *reinterpret_cast<const u32x4*>(row + ka); v[1] = *reinterpret_cast<const u32x4*>(row + ka + 8); }
      if (kc < a.K) { v[2] = *reinterpret_cast<const u32x4*>(row + kc); v[3] = *reinterpret_cast<const u32x4*>(row + kc + 8); }
    }
    uint32_t m01[2] = {0u, 0u};          // chunk maxima as bf16 bit patterns
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int d = 0; d < 8; ++d) {
        const uint32_t w = v[2 * h + (d >> 2)][d & 3];
        const uint32_t lo = w & 0x7fffu, hi = (w >> 16) & 0x7fffu;
        m01[h] = lo > m01[h] ? lo : m01[h];
        m01[h] = hi > m01[h] ? hi : m01[h];
      }
    const uint32_t mine = m01[0] | (m01[1] << 16);
    const uint32_t other = (uint32_t)__shfl_xor((int)mine, 32, 64);
    const uint32_t b0 = (mine & 0xffffu) > (other & 0xffffu) ? (mine & 0xffffu) : (other & 0xffffu);
    const uint32_t b1 = (mine >> 16) > (other >> 16) ? (mine >> 16) : (other >> 16);
    int sb[2];
    float inv[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int field = (int)((h ? b1 : b0) >> 7);
      sb[h] = field - 8 > 0 ? field - 8 : 0;                                  // scale byte = exponent field - emax(E4M3), clamped
      inv[h] = __uint_as_float((uint32_t)(254 - sb[h]) << 23);
    }
    uint32_t q[8];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        // four values per register: scaled by the exact power of two, clamped to the largest element, then the
        // hardware's round-to-nearest-even conversion to E4M3 (two values per instruction)
        int acc = 0;
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
          const uint32_t pair = v[2 * h + ((2 * d + jj) >> 2)][(2 * d + jj) & 3];
          const float x0 = __builtin_amdgcn_fmed3f(bf16_bits_to_f32(pair & 0xffffu) * inv[h], -448.0f, 448.0f);
          const float x1 = __builtin_amdgcn_fmed3f(__uint_as_float(pair & 0xffff0000u) * inv[h], -448.0f, 448.0f);
          acc = jj == 0 ? __builtin_amdgcn_cvt_pk_fp8_f32(x0, x1, acc, false) : __builtin_amdgcn_cvt_pk_fp8_f32(x0, x1, acc, true);
        }
        q[4 * h + d] = (uint32_t)acc;
      }
    xa[i] = v8i{(int)q[0], (int)q[1], (int)q[2], (int)q[3], (int)q[4], (int)q[5], (int)q[6], (int)q[7]};
    xsc[i] = kg ? sb[1] : sb[0];         // lanes 0..31 carry the scale of block 0, lanes 32..63 that of block 1
  }
  // ---- weights: this wave's NG tiles of one row-tile = 4 NG loads of 16 bytes + NG scale dwords per lane
  struct WTile { u32x4 c[NG][4]; uint32_t sc[NG]; };
  auto issue = [&](WTile& t, int u) {
    const int nt = u0 + (u < n_units ? u : n_units - 1);               // past the end: the last tile again (keeps the loads unconditional)
    const uint8_t* base = a.packed + (int64_t)nt * a.k_tiles * kMxTileBytes;
#pragma unroll
    for (int i = 0; i < NG; ++i) {
      int grp = group0 + wave + kMxMain * i;
      grp = grp < n_groups ? grp : n_groups - 1;                       // a dead tile multiplies zero x fragments
      const uint8_t* tile = base + (int64_t)grp * kMxTileBytes;
#pragma unroll
      for (int j = 0; j < 4; ++j) t.c[i][j] = *reinterpret_cast<const u32x4*>(tile + j * 1024 + lane * 16);
      t.sc[i] = *reinterpret_cast<const uint32_t*>(tile + 4096 + lane * 4);
    }
  };
  auto multiply = [&](const WTile& t, float (&out)[MR]) {
    f32x16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < NG; ++i) {
      auto step = [&](auto jc) {
        constexpr int j = decltype(jc)::value;
        const v8i b = v8i{(int)t.c[i][j][0], (int)t.c[i][j][1], (int)t.c[i][j][2], (int)t.c[i][j][3], 0, 0, 0, 0};
        // A = activations (FP8 E4M3, cbsz 0), scale in byte 0 of its register; B = weights (FP4 E2M1, blgp 4),
        // scale = byte j of the lane's scale dword
        acc = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(xa[4 * i + j], b, acc, 0, 4, 0, xsc[4 * i + j], j, (int)t.sc[i]);
      };
      step(std::integral_constant<int, 0>{});
      step(std::integral_constant<int, 1>{});
      step(std::integral_constant<int, 2>{});
      step(std::integral_constant<int, 3>{});
    }
#pragma unroll
    for (int q = 0; q < MR; ++q) out[q] = acc[q];
  };
  // Two tiles in flight per wave, in two fixed sets of registers.  The loop body has no branch around a load or
  // a barrier (past the end the last tile is loaded and multiplied again; the eighth wave skips its store): that
  // keeps the compiler's wait counts exact, so multiplying one tile never waits for the other tile's loads.
  WTile t0, t1;
  __builtin_amdgcn_sched_barrier(0);     // t0's loads strictly before t1's here too: the loop head's wait count is the
  issue(t0, 0);                          // minimum over the ways into it
  __builtin_amdgcn_sched_barrier(0);
  issue(t1, 1);
  __builtin_amdgcn_sched_barrier(0);
  for (int u = 0; u < n_units; u += 2) {
    float part[MR];
    multiply(t0, part);
    __builtin_amdgcn_sched_barrier(0);   // the refill is issued right here, in program order: the wait counts rely on it
    issue(t0, u + 2);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int q = 0; q < MR; ++q) red[0][wave][q][lane] = part[q];
    __syncthreads();
    multiply(t1, part);
    __builtin_amdgcn_sched_barrier(0);
    issue(t1, u + 3);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int q = 0; q < MR; ++q) red[1][wave][q][lane] = part[q];
    __syncthreads();
    // red[h] is written again two units later, after the barrier of the unit in between: the eighth wave has read it by then
  }
}

template <int MR>
__global__ __launch_bounds__(256) void mx_reduce_kernel(const float* partial, int Sk, int n_tiles, int M, int64_t N, uint16_t* y, int64_t ldy,
                                                        const uint16_t* bias) {
  const int nt = blockIdx.x;
  for (int e = threadIdx.x; e < MR * 64; e += 256) {
    const int q = e >> 6, l = e & 63;
    float sum = 0.f;
    for (int r = 0; r < Sk; ++r) sum += partial[(((int64_t)r * n_tiles + nt) * MR + q) * 64 + l];
    const int tok = 8 * (q >> 2) + 4 * (l >> 5) + (q & 3);
    const int64_t n = (int64_t)nt * 32 + (l & 31);
    if (tok < M && n < N) y[(int64_t)tok * ldy + n] = (uint16_t)f32_to_bf16_bits(sum + (bias ? bf16_bits_to_f32(bias[n]) : 0.f));
  }
}

static int64_t grid_for(int64_t items) {
  int64_t b = (items + 255) / 256;
  return b < 1 ? 1 : (b > 8192 ? 8192 : b);
}

// workspace of mxfp4_linear_native: K-range partial tiles
struct MxWorkspace { size_t partial_off, total; int Sk, NG; };
static MxWorkspace mx_workspace(int64_t M, int64_t N, int64_t K) {
  MxWorkspace w{};
  (void)M;
  const int64_t n_groups = ceil_div(K > 0 ? K : 1, 256);
  w.Sk = (int)ceil_div(n_groups, kMxMain * kMxMaxGroups);
  w.NG = (int)ceil_div(n_groups, (int64_t)kMxMain * w.Sk);             // 1 or 2
  auto al = [](size_t v) { return (v + 255) & ~(size_t)255; };
  w.partial_off = 0;
  w.total = w.partial_off + al((size_t)w.Sk * (size_t)ceil_div(N > 0 ? N : 1, 32) * 16 * 64 * sizeof(float));
  return w;
}

template <int NG, int MR, int LC>
static int launch_mx_t(const MxArgs& a, int grid, hipStream_t st) {
  mx_native_kernel<NG, MR, LC><<<dim3((unsigned)grid), dim3(kMxWaves * 64), 0, st>>>(a);
  return launch_status();
}
template <int NG, int MR>
static int launch_mx_lc(const MxArgs& a, int grid, hipStream_t st) {
  if (a.n_chunks == 0) return launch_mx_t<NG, MR, 0>(a, grid, st);
  if (a.n_chunks <= 6) return launch_mx_t<NG, MR, 6>(a, grid, st);     // r <= 32
  if (a.n_chunks <= 12) return launch_mx_t<NG, MR, 12>(a, grid, st);   // r <= 64
  if (a.n_chunks <= 24) return launch_mx_t<NG, MR, 24>(a, grid, st);   // r <= 128
  return QERL_ERR_SHAPE;
}
template <int MR>
static int launch_mx(const MxArgs& a, int NG, int grid, hipStream_t st) {
  if (NG == 1) return launch_mx_lc<1, MR>(a, grid, st);
  if (NG == 2) return launch_mx_lc<2, MR>(a, grid, st);
  return QERL_ERR_SHAPE;
}

// ---- more than 32 tokens: a GEMM on the block-scaled matrix instruction ---------------------------------------
// y = MXFP8(x) . MXFP4(W)^T, x quantised beforehand (mx_quantize_kernel<8>) into codes [M, K] and scales [M, K / 32].
// No conversion arithmetic at all: packed weights go global -> registers -> matrix instruction.  Workgroup tile
// 128 tokens x 256 rows, eight waves as 2 x 4: a wave owns 64 tokens x 64 rows (2 x 2 accumulator tiles), so every
// x fragment read from LDS and every weight fragment feeds two instructions.  A stage is one packed tile (256
// inputs, four instruction steps, 16 instructions per wave between barriers): its weights are requested one stage
// ahead into registers, its x slab (128 tokens x 256 bytes + 8 scale bytes per token) one stage ahead into
// registers and then into the other of two LDS buffers (16-byte chunks XOR-swizzled by row; the scale bytes of a
// row regrouped so that a lane finds the four bytes of its half in one dword and the instruction picks by an
// immediate).  No branch inside a stage depends on the thread or the stage: requests past the end are redirected
// to the last stage, so the compiler's wait counts stay exact.  Bound by the FP8 matrix rate.
struct MxGemmArgs {
  const uint8_t* xq; const uint8_t* xs; int64_t M, K;     // MXFP8 codes [M, K], scales [M, K / 32]
  const uint8_t* packed; int k_tiles; int n_tiles; int64_t N;
  uint16_t* y; int64_t ldy;
  int n_blocks, nblk_per_xcd;
  const uint16_t* ts; int64_t ts_ld; int n_chunks; const uint16_t* B; int r;   // as in MxArgs
  const uint16_t* bias;
};

constexpr int kMxgBM = 128, kMxgThreads = 512, kMxgMT = 2, kMxgNT = 2;
struct MxgW { u32x4 c[kMxgNT][4]; uint32_t sc[kMxgNT]; };          // one wave's weights of a stage
struct MxgX { u32x4 c[4]; uint32_t s0, s1; };                       // one thread's share of an x slab: four chunks, two scale bytes

__global__ __launch_bounds__(kMxgThreads) void mx_gemm_kernel(const MxGemmArgs a) {
  constexpr int BM = kMxgBM, MT = kMxgMT, NT = kMxgNT;
  constexpr int kChunks = BM * 16;                         // 16-byte chunks of one x slab (BM rows x 256 bytes)
  __shared__ u32x4 xs[2 * kChunks];                        // chunk c of row r at r * 16 + (c ^ (r & 15))
  __shared__ __attribute__((aligned(8))) uint8_t xsc[2 * BM * 8];   // row r: bytes [g * 4 + j] = scale of block 2 j + g
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 2, wn = wave & 3;                 // the wave's token half and row quarter
  const int n32 = lane & 31, kg = lane >> 5;
  const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;   // each XCD walks a contiguous eighth of the column blocks
  const int nb_local = local % a.nblk_per_xcd, mb = local / a.nblk_per_xcd;
  const int nb = xcd * a.nblk_per_xcd + nb_local;
  if (nb >= a.n_blocks) return;
  const int64_t m0 = (int64_t)mb * BM;
  const int nt0 = (nb * 4 + wn) * NT;
  const int64_t n_blk = a.K / 32;

  f32x16 acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[mt][nt][i] = 0.f;

  // thread -> (row, chunk) of the slab: chunks tid, tid + 512, ...; scale bytes: row tid / 4, blocks 2 (tid % 4), + 1
  auto gload_x = [&](MxgX& r, int kt) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int idx = tid + i * kMxgThreads, row = idx >> 4, ch = idx & 15;
      int64_t gr = m0 + row;
      gr = gr < a.M ? gr : a.M - 1;
      int64_t k = (int64_t)kt * 256 + ch * 16;
      k = k < a.K ? k : a.K - 16;                          // past the end of K: any bytes, zeroed before they reach LDS
      r.c[i] = *reinterpret_cast<const u32x4*>(a.xq + gr * a.K + k);
    }
    int64_t gr = m0 + (tid >> 2);
    gr = gr < a.M ? gr : a.M - 1;
    int64_t b0 = (int64_t)kt * 8 + 2 * (tid & 3), b1 = b0 + 1;
    b0 = b0 < n_blk ? b0 : n_blk - 1;
    b1 = b1 < n_blk ? b1 : n_blk - 1;
    r.s0 = a.xs[gr * n_blk + b0];
    r.s1 = a.xs[gr * n_blk + b1];
  };
  auto swrite_x = [&](int buf, const MxgX& r, int kt) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int idx = tid + i * kMxgThreads, row = idx >> 4, ch = idx & 15;
      // beyond K (K % 256 != 0): zero codes -- a stray byte could be an FP8 NaN, and the weights there are zero
      const u32x4 v = (int64_t)kt * 256 + ch * 16 < a.K ? r.c[i] : u32x4{0u, 0u, 0u, 0u};
      xs[buf * kChunks + row * 16 + (ch ^ (row & 15))] = v;
    }
    const int row = tid >> 2, j = tid & 3;                  // blocks 2 j (half 0) and 2 j + 1 (half 1) of the row
    const bool in0 = (int64_t)kt * 8 + 2 * j < n_blk, in1 = (int64_t)kt * 8 + 2 * j + 1 < n_blk;
    xsc[(buf * BM + row) * 8 + j] = in0 ? (uint8_t)r.s0 : (uint8_t)0;
    xsc[(buf * BM + row) * 8 + 4 + j] = in1 ? (uint8_t)r.s1 : (uint8_t)0;
  };
  auto gload_w = [&](MxgW& w, int kt) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      int tile = nt0 + nt;
      tile = tile < a.n_tiles ? tile : a.n_tiles - 1;
      const uint8_t* base = a.packed + ((int64_t)tile * a.k_tiles + kt) * kMxTileBytes;
#pragma unroll
      for (int j = 0; j < 4; ++j) w.c[nt][j] = *reinterpret_cast<const u32x4*>(base + j * 1024 + lane * 16);
      w.sc[nt] = *reinterpret_cast<const uint32_t*>(base + 4096 + lane * 4);
    }
  };
  auto compute = [&](int buf, const MxgW& w) {
    const u32x4* xst = xs + buf * kChunks;
    int xscale[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int row = wm * 64 + mt * 32 + n32;
      xscale[mt] = (int)*reinterpret_cast<const uint32_t*>(xsc + (buf * BM + row) * 8 + kg * 4);
    }
    // x fragments of step j + 1 are requested from LDS before the instructions of step j are issued
    auto frags = [&](v8i (&xa)[MT], int j) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        const int row = wm * 64 + mt * 32 + n32, sw = row & 15;
        const u32x4 c0 = xst[row * 16 + ((4 * j + kg) ^ sw)], c1 = xst[row * 16 + ((4 * j + 2 + kg) ^ sw)];
        xa[mt] = v8i{(int)c0[0], (int)c0[1], (int)c0[2], (int)c0[3], (int)c1[0], (int)c1[1], (int)c1[2], (int)c1[3]};
      }
    };
    auto step = [&](const v8i (&xa)[MT], auto jc) {
      constexpr int j = decltype(jc)::value;
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const v8i b = v8i{(int)w.c[nt][j][0], (int)w.c[nt][j][1], (int)w.c[nt][j][2], (int)w.c[nt][j][3], 0, 0, 0, 0};
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          acc[mt][nt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(xa[mt], b, acc[mt][nt], 0, 4, j, xscale[mt], j, (int)w.sc[nt]);
      }
    };
    v8i xa[MT], xb[MT];
    frags(xa, 0);
    frags(xb, 1);
    step(xa, std::integral_constant<int, 0>{});
    frags(xa, 2);
    step(xb, std::integral_constant<int, 1>{});
    frags(xb, 3);
    step(xa, std::integral_constant<int, 2>{});
    step(xb, std::integral_constant<int, 3>{});
  };

  {
    const int n = a.k_tiles, last = n - 1;
    auto clamp_kt = [&](int kt) { return kt < last ? kt : last; };
    MxgW w0, w1;
    MxgX x0, x1;
    gload_x(x0, 0);
    gload_x(x1, clamp_kt(1));
    gload_w(w0, 0);
    swrite_x(0, x0, 0);
    __syncthreads();
    // Two stages per round so that buffer and register names are constants.  Stage kt: the slab of kt + 2 and the
    // weights of kt + 1 are requested, kt is multiplied, the slab of kt + 1 (requested a stage ago) goes to LDS.
    auto stage = [&](int kt, int buf, MxgW& wcur, MxgW& wnext, MxgX& xfar, const MxgX& xnear) {
      gload_x(xfar, clamp_kt(kt + 2));
      gload_w(wnext, clamp_kt(kt + 1));
      __builtin_amdgcn_sched_barrier(0);   // the requests stay ahead of the stage's arithmetic
      compute(buf, wcur);
      __builtin_amdgcn_sched_barrier(0);
      swrite_x(buf ^ 1, xnear, clamp_kt(kt + 1));
      __syncthreads();
    };
    int kt = 0;
    for (; kt + 2 <= n; kt += 2) {
      stage(kt, 0, w0, w1, x0, x1);
      stage(kt + 1, 1, w1, w0, x1, x0);
    }
    if (kt < n) stage(kt, 0, w0, w1, x0, x1);
  }
  // ---- LoRA up-projection (Eq. 2): 3 r more input columns, [hi | mid | lo] . [B B B]^T, on the bf16 matrix
  // instruction of the same output layout; operands straight from memory, four chunks of 16 columns requested at a time
  for (int c0 = 0; c0 < a.n_chunks; c0 += 4) {
    u32x4 tf[4][MT], bf[4][NT];
#pragma unroll
    for (int cc = 0; cc < 4; ++cc) {
      const bool live = c0 + cc < a.n_chunks;
      const int col = 16 * (live ? c0 + cc : a.n_chunks - 1) + 8 * kg;
      const int bc = lora_b_col(col, a.r);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        int64_t row = m0 + wm * 64 + mt * 32 + n32;
        row = row < a.M ? row : a.M - 1;
        tf[cc][mt] = *reinterpret_cast<const u32x4*>(a.ts + row * a.ts_ld + col);
        if (!live) tf[cc][mt] = u32x4{0u, 0u, 0u, 0u};
      }
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        int64_t n = (int64_t)(nt0 + nt) * 32 + n32;
        n = n < a.N ? n : a.N - 1;
        bf[cc][nt] = *reinterpret_cast<const u32x4*>(a.B + n * a.r + bc);
      }
    }
#pragma unroll
    for (int cc = 0; cc < 4; ++cc)
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
          acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, tf[cc][mt]), __builtin_bit_cast(bf16x8, bf[cc][nt]),
                                                                acc[mt][nt], 0, 0, 0);
  }
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const int64_t nn = (int64_t)(nt0 + nt) * 32 + n32;
      const float bias = (a.bias && nn < a.N) ? bf16_bits_to_f32(a.bias[nn]) : 0.f;
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int64_t m = m0 + wm * 64 + mt * 32 + 8 * (i >> 2) + 4 * kg + (i & 3);
        if (m < a.M && nn < a.N) a.y[m * a.ldy + nn] = (uint16_t)f32_to_bf16_bits(acc[mt][nt][i] + bias);
      }
    }
}

static int launch_mx_gemm(MxGemmArgs a, hipStream_t st) {
  a.n_blocks = (int)ceil_div(a.n_tiles, 4 * kMxgNT);
  a.nblk_per_xcd = (int)ceil_div(a.n_blocks, 8);
  const int64_t m_blocks = ceil_div(a.M, kMxgBM);
  mx_gemm_kernel<<<dim3((unsigned)(8 * a.nblk_per_xcd * m_blocks)), dim3(kMxgThreads), 0, st>>>(a);
  return launch_status();
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
  return (size_t)ceil_div(N, 32) * (size_t)ceil_div(K, 256) * kMxTileBytes;
}

extern "C" int mxfp4_prepack(const uint8_t* codes, const uint8_t* scales, int64_t N, int64_t K, void* packed, void* stream) {
  if (N < 0 || K < 0 || K % 32 != 0) return QERL_ERR_SHAPE;
  if (N == 0 || K == 0) return QERL_OK;
  if (!codes || !scales || !packed) return QERL_ERR_NULL;
  if (!aligned(packed, 16) || !aligned(codes, 16) || (K / 2) % 16 != 0) return QERL_ERR_ALIGN;
  const int64_t nt = ceil_div(N, 32), kt = ceil_div(K, 256);
  mxfp4_prepack_kernel<<<dim3((unsigned)grid_for(nt * kt * 256)), dim3(256), 0, (hipStream_t)stream>>>(codes, scales, N, K, nt, kt,
                                                                                                    (uint8_t*)packed);
  return launch_status();
}

// beyond the decode kernel's 32 tokens: x as MXFP8 codes and scales
static size_t mx_gemm_workspace(int64_t M, int64_t K) {
  auto al = [](size_t v) { return (v + 255) & ~(size_t)255; };
  return al((size_t)M * (size_t)K) + al((size_t)M * (size_t)(K / 32));
}
extern "C" size_t mxfp4_linear_native_workspace_bytes(int64_t M, int64_t N, int64_t K) {
  if (M > 32) return mx_gemm_workspace(M, K > 0 ? K : 32);
  return mx_workspace(M, N, K).total;
}

// ---- the native linear, with or without the LoRA branch and bias -------------------------------------------------
namespace qerl {

// lora_down_block divides by the NVFP4 tensor scale it is handed; MXFP4 has none
static __device__ float mx_unit_scale = 1.0f;
constexpr int kMxMaxDevices = 64;
static const float* g_unit_scale_ptr[kMxMaxDevices];   // device address of mx_unit_scale per device, looked up once there

static int unit_scale_ptr(const float** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return launch_status();
  if (dev < 0 || dev >= kMxMaxDevices) return QERL_ERR_SHAPE;
  const float* p = __atomic_load_n(&g_unit_scale_ptr[dev], __ATOMIC_ACQUIRE);
  if (!p) {
    void* q = nullptr;
    const hipError_t e = hipGetSymbolAddress(&q, HIP_SYMBOL(mx_unit_scale));
    if (e != hipSuccess || !q) { set_last_hip_error((int)e); (void)hipGetLastError(); return QERL_ERR_LAUNCH; }
    p = (const float*)q;
    __atomic_store_n(&g_unit_scale_ptr[dev], p, __ATOMIC_RELEASE);   // racing first calls look up the same address
  }
  *out = p;
  return QERL_OK;
}

// workspace of the LoRA variant: arrival counters of the down-projection's K-parts (zero between calls), their
// partial sums, ts, then the plain variant's workspace
struct MxLoraWorkspace { size_t ctr_off, tpart_off, ts_off, base_off, total; int64_t ts_ld; int n_chunks; };
static MxLoraWorkspace mx_lora_workspace(int64_t M, int64_t N, int64_t K, int64_t r) {
  auto al = [](size_t v) { return (v + 255) & ~(size_t)255; };
  MxLoraWorkspace w{};
  w.n_chunks = (int)ceil_div(3 * r, 16);
  w.ts_ld = (int64_t)w.n_chunks * 16;
  w.ctr_off = 0;
  w.tpart_off = al(kCtrlDownWords * sizeof(uint32_t));
  w.ts_off = w.tpart_off + (r > 0 ? kDownExchangeBytes : 0);
  w.base_off = w.ts_off + al((size_t)(M > 0 ? M : 1) * (size_t)w.ts_ld * sizeof(uint16_t));
  w.total = w.base_off + mxfp4_linear_native_workspace_bytes(M, N, K);
  return w;
}

struct MxLora { const uint16_t* ts; int64_t ts_ld; int n_chunks; const uint16_t* B; int r; const uint16_t* bias; };

static int mx_linear(const void* x, int64_t M, int64_t K, int64_t ldx, const void* packed, int64_t N, void* y, int64_t ldy,
                     const MxLora& lo, void* workspace, size_t workspace_bytes, hipStream_t st) {
  if (M > 32) {
    // quantise x once, then the GEMM
    const size_t need = mx_gemm_workspace(M, K);
    if (!workspace || !aligned(workspace, 256) || workspace_bytes < need) return QERL_ERR_WORKSPACE;
    uint8_t* xq = (uint8_t*)workspace;
    uint8_t* xsc = xq + (((size_t)M * (size_t)K + 255) & ~(size_t)255);
    mx_quantize_kernel<8><<<dim3((unsigned)grid_for(M * (K / 32))), dim3(256), 0, st>>>((const uint16_t*)x, M, K, ldx, xq, xsc);
    int rc = launch_status();
    if (rc != QERL_OK) return rc;
    MxGemmArgs g{};
    g.xq = xq; g.xs = xsc; g.M = M; g.K = K; g.packed = (const uint8_t*)packed;
    g.k_tiles = (int)ceil_div(K, 256); g.n_tiles = (int)ceil_div(N, 32); g.N = N; g.y = (uint16_t*)y; g.ldy = ldy;
    g.ts = lo.ts; g.ts_ld = lo.ts_ld; g.n_chunks = lo.n_chunks; g.B = lo.B; g.r = lo.r; g.bias = lo.bias;
    return launch_mx_gemm(g, st);
  }
  const MxWorkspace w = mx_workspace(M, N, K);
  if (!workspace || !aligned(workspace, 256) || workspace_bytes < w.total) return QERL_ERR_WORKSPACE;
  uint8_t* ws = (uint8_t*)workspace;
  int rc = QERL_OK;
  MxArgs a{};
  a.x = (const uint16_t*)x; a.ldx = ldx; a.M = (int)M; a.K = K;
  a.packed = (const uint8_t*)packed; a.k_tiles = (int)ceil_div(K, 256); a.n_tiles = (int)ceil_div(N, 32); a.N = N;
  a.y = (uint16_t*)y; a.ldy = ldy; a.partial = (float*)(ws + w.partial_off);
  a.ts = lo.ts; a.ts_ld = lo.ts_ld; a.n_chunks = lo.n_chunks; a.B = lo.B; a.r = lo.r; a.bias = lo.bias;
  a.Sk = w.Sk; a.groups_per_range = kMxMain * w.NG;
  int per_range = 256 / w.Sk;
  if (per_range < 1) per_range = 1;
  if (per_range > a.n_tiles) per_range = a.n_tiles;
  a.per_range = per_range; a.units_base = a.n_tiles / per_range; a.units_rem = a.n_tiles % per_range;
  const int grid = per_range * w.Sk;
  rc = M <= 8 ? launch_mx<4>(a, w.NG, grid, st) : launch_mx<16>(a, w.NG, grid, st);
  if (rc != QERL_OK || w.Sk == 1) return rc;
  if (M <= 8) mx_reduce_kernel<4><<<dim3((unsigned)a.n_tiles), dim3(256), 0, st>>>(a.partial, w.Sk, a.n_tiles, (int)M, N, a.y, ldy, a.bias);
  else mx_reduce_kernel<16><<<dim3((unsigned)a.n_tiles), dim3(256), 0, st>>>(a.partial, w.Sk, a.n_tiles, (int)M, N, a.y, ldy, a.bias);
  return launch_status();
}

static int mx_validate(const void* x, int64_t M, int64_t K, int64_t ldx, const void* packed, int64_t N, const void* y, int64_t ldy) {
  if (M < 0 || N < 0 || K < 0 || K % 32 != 0 || ldx < K || ldy < N || N >= ((int64_t)1 << 24)) return QERL_ERR_SHAPE;
  if (M == 0 || N == 0) return 1;   // nothing to do
  if (K == 0) return QERL_ERR_SHAPE;
  if (!x || !packed || !y) return QERL_ERR_NULL;
  if (!aligned(x, 16) || ldx % 8 != 0 || !aligned(packed, 16) || !aligned(y, 2)) return QERL_ERR_ALIGN;
  return QERL_OK;
}

}  // namespace qerl

extern "C" int mxfp4_linear_native(const void* x, int64_t M, int64_t K, int64_t ldx, const void* packed, int64_t N, void* y, int64_t ldy,
                                   void* workspace, size_t workspace_bytes, void* stream) {
  const int vr = mx_validate(x, M, K, ldx, packed, N, y, ldy);
  if (vr != QERL_OK) return vr > 0 ? QERL_OK : vr;
  return mx_linear(x, M, K, ldx, packed, N, y, ldy, MxLora{}, workspace, workspace_bytes, (hipStream_t)stream);
}

extern "C" size_t mxfp4_lora_linear_native_workspace_bytes(int64_t M, int64_t N, int64_t K, int64_t r) {
  if (r < 0 || r > kMxMaxRank) return 0;
  return mx_lora_workspace(M, N, K, r).total;
}

extern "C" int mxfp4_lora_linear_native(const void* x, int64_t M, int64_t K, int64_t ldx, const void* packed, int64_t N, const void* A,
                                        const void* B, int64_t r, float lora_scale, const void* bias, void* y, int64_t ldy,
                                        void* workspace, size_t workspace_bytes, void* stream) {
  if (r < 0 || r > kMxMaxRank || r % 8 != 0) return QERL_ERR_SHAPE;
  const int vr = mx_validate(x, M, K, ldx, packed, N, y, ldy);
  if (vr != QERL_OK) return vr > 0 ? QERL_OK : vr;
  if (r > 0 && (!A || !B)) return QERL_ERR_NULL;
  if (r > 0 && (!aligned(A, 16) || !aligned(B, 16))) return QERL_ERR_ALIGN;
  if (bias && !aligned(bias, 2)) return QERL_ERR_ALIGN;
  const MxLoraWorkspace L = mx_lora_workspace(M, N, K, r);
  if (!workspace || !aligned(workspace, 256) || workspace_bytes < L.total) return QERL_ERR_WORKSPACE;
  uint8_t* ws = (uint8_t*)workspace;
  hipStream_t st = (hipStream_t)stream;
  MxLora lo{};
  lo.bias = (const uint16_t*)bias;
  if (r > 0) {
    const float* one = nullptr;
    int rc = unit_scale_ptr(&one);
    if (rc != QERL_OK) return rc;
    GemmArgs d{};
    d.x = (const uint16_t*)x; d.ldx = ldx; d.M = M; d.K = K; d.N = r; d.wbf16 = (const uint16_t*)A; d.n_tiles = (int)ceil_div(r, 32);
    d.tensor_scale = one; d.lora_scale = lora_scale; d.r = (int)r;
    d.ts = (const uint16_t*)(ws + L.ts_off); d.ts_ld = L.ts_ld;
    d.tpart = (uint32_t*)(ws + L.tpart_off); d.counters = (uint32_t*)(ws + L.ctr_off);
    rc = launch_lora_down_gemm(d, st);
    if (rc != QERL_OK) return rc;
    lo.ts = d.ts; lo.ts_ld = L.ts_ld; lo.n_chunks = L.n_chunks; lo.B = (const uint16_t*)B; lo.r = (int)r;
  }
  return mx_linear(x, M, K, ldx, packed, N, y, ldy, lo, ws + L.base_off, workspace_bytes - L.base_off, st);
}
