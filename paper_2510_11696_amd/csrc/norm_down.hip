// aqn_rmsnorm_lora_down: the noisy RMSNorm of Eq. 10 and the LoRA down-projections
//   y = (gain + noise) (.) x / sqrt(mean(x^2) + eps),     t_i = y A_i^T   (Eq. 2, first factor)
// of the adapters that read y (q/k/v or gate/up), in one launch, for decode batches (M <= 16).
//
// At these sizes x A^T is a few hundred MFMAs behind a chain of memory round trips; inside the
// linear kernel that chain sits on the critical path of every workgroup.  Here it runs where y is
// produced, and the linear kernel that follows finds t in memory -- as QERL_T_PARTS partial sums
// over slices of K, which its epilogue adds in slice order, so that no workgroup of this kernel has
// to wait for another either.
//
// QERL_T_PARTS x (32-rank tiles of the stacked adapters) workgroups of 512 threads; workgroup (p, tile) owns the
// p-th slice of K (whole 16-input steps) and one tile; the tile-0 workgroups write y:
//   1. wave w reads row w (and w + 8) whole and forms its sum of squares -- one wave per row, so no
//      exchange between waves; 1 / rms of every row goes to LDS;
//   2. the slice's columns of every row (requested at the start as well) are normalised, rounded,
//      written to y and kept in LDS.  y is the function aqn_rmsnorm computes; the mean of squares is
//      summed in another order, so a rare element can differ from aqn_rmsnorm's by one bf16 unit;
//   3. the eight waves split the slice's steps: x fragment from LDS, A fragments of all stacked ranks
//      (requested first thing in the kernel) from registers, one accumulator tile per 32 stacked ranks;
//   4. the eight waves' tiles are added in wave order and stored as part p of every adapter's t.
// No workgroup depends on another, and every sum has a fixed order.
#include "common.hpp"

namespace qerl {

constexpr int kNdThreads = 512, kNdWaves = 8;
constexpr int kNdMaxAdapters = 4;
constexpr int kNdParts = QERL_T_PARTS;
constexpr int kNdMaxTiles = 8;             // 32-rank tiles of the stacked adapters (one workgroup column each): four adapters of rank 64
constexpr int kNdStepsPerWave = 4;         // 16-input steps of the slice per wave held in registers at a time

#ifdef QERL_ND_TRACE
__device__ unsigned long long g_nd_trace[64 * 8 * 8];
#define NDT(p) do { if (lane == 0 && blockIdx.x < 64) g_nd_trace[((int)blockIdx.x * 8 + wave) * 8 + (p)] = wall_clock64(); } while (0)
#else
#define NDT(p) do { } while (0)
#endif

struct NormDownArgs {
  const uint16_t* x; int64_t ldx; int M; int64_t H;
  const uint16_t* gain; const float* noise; float eps;
  uint16_t* y; int64_t ldy;
  const uint16_t* A[kNdMaxAdapters]; float* t[kNdMaxAdapters]; int r[kNdMaxAdapters];
  int off1, off2, off3;                    // first stacked rank of adapters 1..3 (INT_MAX if absent)
  int r_total, n_tiles;
  int steps_per_part;                      // 16-input steps per K-slice
  int xs_stride;                           // bytes between token rows of the slice in LDS
};

// MR: accumulator registers that hold live tokens (4 for M <= 8, 8 for M <= 16); NCL: 16-byte chunks of a row
// per lane when one wave reads the row (8: H <= 4096, 16: H <= 8192); NT: 32-rank tiles
template <int MR, int NCL, int NT>
__global__ __launch_bounds__(kNdThreads) void norm_down_kernel(const NormDownArgs a) {
  extern __shared__ __attribute__((aligned(256))) unsigned char smem[];   // slice of y [(M+1) rows][xs_stride]; red after it
  __shared__ float s_inv[16];              // 1 / rms of every row
  constexpr int RPW = MR == 4 ? 1 : 2;     // rows per wave for the sums of squares: rows wave, wave + 8
  constexpr int NQ = MR == 4 ? 2 : 4;      // (row, chunk) items of the slice per thread: 128 chunk slots per row
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int chunks = (int)(a.H / 8);
  const int n32 = lane & 31, kg = lane >> 5;
  const int part = (int)blockIdx.x;
  const int tile0 = (int)blockIdx.y * NT;   // first 32-rank tile of the stacked adapters this workgroup multiplies
  const int n_steps = (int)(a.H / 16);
  const int step0 = part * a.steps_per_part;
  const int step1 = step0 + a.steps_per_part < n_steps ? step0 + a.steps_per_part : n_steps;
  const int c_lo = step0 * 2, nsc = (step1 - step0) * 2;   // 16-byte chunks of the slice: first, count (<= 128)
  NDT(0);

  // ---- everything this workgroup reads is requested up front, in the order it is needed:
  // (a) whole rows for the sums of squares: wave w reads row w (and w + 8), lane l the chunks l, l + 64, ...
  // (with two long rows per wave the second is read after the first is summed: registers)
  constexpr bool kSeqRows = RPW * NCL > 16;
  constexpr int XR = kSeqRows ? 1 : RPW;
  u32x4 xr[XR][NCL];
  auto load_row = [&](int p, int slot) {
    const int row = wave + 8 * p;
#pragma unroll
    for (int i = 0; i < NCL; ++i) {
      const int c = lane + 64 * i;
      xr[slot][i] = u32x4{0u, 0u, 0u, 0u};
      if (row < a.M && c < chunks) xr[slot][i] = reinterpret_cast<const u32x4*>(a.x + (int64_t)row * a.ldx)[c];
    }
  };
#pragma unroll
  for (int p = 0; p < XR; ++p) load_row(p, p);
  // (b) the slice's chunks of every row with their gain and noise: item = (row, chunk slot), 128 slots per row
  const u32x4* __restrict__ gr = reinterpret_cast<const u32x4*>(a.gain);
  const f32x4* __restrict__ zr = reinterpret_cast<const f32x4*>(a.noise);
  u32x4 xq[NQ], gq[NQ];
  f32x4 zq[NQ][2];
#pragma unroll
  for (int q = 0; q < NQ; ++q) {
    const int id = tid + kNdThreads * q, row = id >> 7, cs = id & 127;
    xq[q] = u32x4{0u, 0u, 0u, 0u}; gq[q] = xq[q];
    zq[q][0] = f32x4{0.f, 0.f, 0.f, 0.f}; zq[q][1] = zq[q][0];
    if (row < a.M && cs < nsc) {
      const int c = c_lo + cs;
      xq[q] = reinterpret_cast<const u32x4*>(a.x + (int64_t)row * a.ldx)[c];
      gq[q] = gr[c];
      if (zr) { zq[q][0] = zr[2 * c]; zq[q][1] = zr[2 * c + 1]; }
    }
  }
  // (c) A fragments of this wave's steps, all rank tiles (they depend on nothing, so their latency overlaps
  // the normalisation).  Wave w takes steps step0 + w, step0 + w + 8, ...
  const uint16_t* arow[NT];
  bool live[NT];
#pragma unroll
  for (int tl = 0; tl < NT; ++tl) {
    const int s = (tile0 + tl) * 32 + n32; // stacked rank this lane feeds in tile tl
    int ad = 0, off = 0;
    if (s >= a.off1) { ad = 1; off = a.off1; }
    if (s >= a.off2) { ad = 2; off = a.off2; }
    if (s >= a.off3) { ad = 3; off = a.off3; }
    const uint16_t* A = a.A[0];
#pragma unroll
    for (int i = 1; i < kNdMaxAdapters; ++i) A = ad == i ? a.A[i] : A;
    live[tl] = s < a.r_total;
    arow[tl] = A + (int64_t)(live[tl] ? s - off : 0) * a.H + 8 * kg;
  }
  u32x4 af[kNdStepsPerWave][NT];
  auto load_frags = [&](int s0) {
#pragma unroll
    for (int i = 0; i < kNdStepsPerWave; ++i) {
      const int s = s0 + i * kNdWaves;
#pragma unroll
      for (int tl = 0; tl < NT; ++tl) {
        af[i][tl] = u32x4{0u, 0u, 0u, 0u};
        if (s < step1 && live[tl]) af[i][tl] = *reinterpret_cast<const u32x4*>(arow[tl] + (int64_t)s * 16);
      }
    }
  };
  load_frags(step0 + wave);

  // ---- 1. sum of squares of a row: chunks in order per lane, then the lanes (wave_sum); 1 / rms to LDS
#pragma unroll
  for (int p = 0; p < RPW; ++p) {
    const int slot = kSeqRows ? 0 : p;
    if (kSeqRows && p > 0) load_row(p, 0);
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < NCL; ++i) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float lo = bf16_bits_to_f32(xr[slot][i][j] & 0xffffu), hi = bf16_bits_to_f32(xr[slot][i][j] >> 16);
        ss += lo * lo;
        ss += hi * hi;
      }
    }
    if (p == 0) NDT(1);
    const float total = wave_sum(ss);
    if (lane == 0) s_inv[wave + 8 * p] = 1.0f / sqrtf(total / (float)a.H + a.eps);
  }
  __syncthreads();
  NDT(2);

  // ---- 2. normalise and round the slice's columns: to y and to LDS (A-operand rows)
#pragma unroll
  for (int q = 0; q < NQ; ++q) {
    const int id = tid + kNdThreads * q, row = id >> 7, cs = id & 127;
    if (row < a.M && cs < nsc) {
      const float inv = s_inv[row];
      const float z[8] = {zq[q][0][0], zq[q][0][1], zq[q][0][2], zq[q][0][3], zq[q][1][0], zq[q][1][1], zq[q][1][2], zq[q][1][3]};
      u32x4 o;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float ga = bf16_bits_to_f32(gq[q][j] & 0xffffu) + z[2 * j];
        const float gb = bf16_bits_to_f32(gq[q][j] >> 16) + z[2 * j + 1];
        const float xa = bf16_bits_to_f32(xq[q][j] & 0xffffu), xb = bf16_bits_to_f32(xq[q][j] >> 16);
        o[j] = pack_bf16x2(ga * (xa * inv), gb * (xb * inv));
      }
      *reinterpret_cast<u32x4*>(smem + row * a.xs_stride + cs * 16) = o;
      if (blockIdx.y == 0) reinterpret_cast<u32x4*>(a.y + (int64_t)row * a.ldy)[c_lo + cs] = o;
    }
  }
  NDT(3);
  for (int c = tid; c < nsc; c += kNdThreads)   // tokens >= M read this zero row
    *reinterpret_cast<u32x4*>(smem + a.M * a.xs_stride + c * 16) = u32x4{0u, 0u, 0u, 0u};
  __syncthreads();
  NDT(4);

  // ---- 3. partial t over this slice: x fragments from LDS against the A fragments
  const int xrow = n32 < a.M ? n32 : a.M;
  const unsigned char* xbase = smem + xrow * a.xs_stride + kg * 16;
  f32x16 pa[NT];
#pragma unroll
  for (int tl = 0; tl < NT; ++tl)
#pragma unroll
    for (int i = 0; i < 16; ++i) pa[tl][i] = 0.f;
  for (int s0 = step0 + wave; s0 < step1; s0 += kNdWaves * kNdStepsPerWave) {
    if (s0 != step0 + wave) load_frags(s0);
#pragma unroll
    for (int i = 0; i < kNdStepsPerWave; ++i) {
      const int s = s0 + i * kNdWaves;
      if (s < step1) {
        const bf16x8 xf = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(xbase + (s - step0) * 32));
#pragma unroll
        for (int tl = 0; tl < NT; ++tl)
          pa[tl] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf, __builtin_bit_cast(bf16x8, af[i][tl]), pa[tl], 0, 0, 0);
      }
    }
  }
  NDT(5);

  // ---- 4. add the eight waves' tiles in wave order, store part `part` of every adapter's t
  float* red = reinterpret_cast<float*>(smem + (a.M + 1) * a.xs_stride);   // [8 waves][NT][MR][64]
#pragma unroll
  for (int tl = 0; tl < NT; ++tl)
#pragma unroll
    for (int q = 0; q < MR; ++q) red[((wave * NT + tl) * MR + q) * 64 + lane] = pa[tl][q];
  __syncthreads();
  NDT(6);
  for (int e = tid; e < NT * MR * 64; e += kNdThreads) {
    float sum = 0.f;
#pragma unroll
    for (int w = 0; w < kNdWaves; ++w) sum += red[w * NT * MR * 64 + e];
    const int tl = e / (MR * 64), q = (e >> 6) % MR, l = e & 63;
    const int tok = 8 * (q >> 2) + 4 * (l >> 5) + (q & 3), s = (tile0 + tl) * 32 + (l & 31);
    if (tok < a.M && s < a.r_total) {
      int ad = 0, off = 0;
      if (s >= a.off1) { ad = 1; off = a.off1; }
      if (s >= a.off2) { ad = 2; off = a.off2; }
      if (s >= a.off3) { ad = 3; off = a.off3; }
      float* t = a.t[0];
      int r = a.r[0];
#pragma unroll
      for (int i = 1; i < kNdMaxAdapters; ++i)
        if (ad == i) { t = a.t[i]; r = a.r[i]; }
      t[((int64_t)part * a.M + tok) * r + (s - off)] = sum;
    }
  }
  NDT(7);
}

}  // namespace qerl

using namespace qerl;

template <int MR, int NCL, int NT>
static int launch_norm_down_t(const NormDownArgs& a, size_t lds, hipStream_t st) {
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&norm_down_kernel<MR, NCL, NT>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024) != hipSuccess)
      return launch_status();
    attr_set = true;
  }
  norm_down_kernel<MR, NCL, NT><<<dim3(kNdParts, (unsigned)ceil_div(a.n_tiles, NT)), kNdThreads, lds, st>>>(a);
  return launch_status();
}
// One 32-rank tile per workgroup: the tiles' workgroups repeat the (cheap) normalisation, and each has a
// third or a quarter of the A fragments to wait for.
template <int MR, int NCL>
static int launch_norm_down(const NormDownArgs& a, size_t lds, hipStream_t st) {
  return launch_norm_down_t<MR, NCL, 1>(a, lds, st);
}

extern "C" int aqn_rmsnorm_lora_down(const void* x, int64_t M, int64_t H, int64_t ldx, const void* gain,
                                     const float* noise, float eps, void* y, int64_t ldy,
                                     const void* const* A, const int64_t* r, float* const* t, int n_adapters,
                                     void* stream) {
  if (M < 0 || M > 16 || H < 1 || ldx < H || ldy < H) return QERL_ERR_SHAPE;
  if (n_adapters < 1 || n_adapters > kNdMaxAdapters) return QERL_ERR_SHAPE;
  if (!x || !gain || !y || !A || !r || !t) return QERL_ERR_NULL;
  if (H % 16 != 0 || H > 8192) return QERL_ERR_SHAPE;
  if (ldx % 8 != 0 || ldy % 8 != 0 || !aligned(x, 16) || !aligned(y, 16) || !aligned(gain, 16) ||
      (noise && !aligned(noise, 16)))
    return QERL_ERR_ALIGN;
  NormDownArgs a{};
  int r_total = 0;
  int off[kNdMaxAdapters] = {0, 0x7fffffff, 0x7fffffff, 0x7fffffff};
  for (int i = 0; i < n_adapters; ++i) {
    if (!A[i] || !t[i]) return QERL_ERR_NULL;
    if (r[i] < 8 || r[i] > 64 || r[i] % 8 != 0) return QERL_ERR_SHAPE;
    if (!aligned(A[i], 16) || !aligned(t[i], 32)) return QERL_ERR_ALIGN;
    a.A[i] = (const uint16_t*)A[i]; a.t[i] = t[i]; a.r[i] = (int)r[i];
    off[i] = r_total;
    r_total += (int)r[i];
  }
  if (r_total > 32 * kNdMaxTiles) return QERL_ERR_SHAPE;
  if (M == 0) return QERL_OK;
  for (int i = n_adapters; i < kNdMaxAdapters; ++i) { a.A[i] = a.A[0]; a.t[i] = a.t[0]; a.r[i] = a.r[0]; }
  a.off1 = off[1]; a.off2 = off[2]; a.off3 = off[3];
  a.r_total = r_total; a.n_tiles = (int)ceil_div(r_total, 32);
  a.x = (const uint16_t*)x; a.ldx = ldx; a.M = (int)M; a.H = H;
  a.gain = (const uint16_t*)gain; a.noise = noise; a.eps = eps; a.y = (uint16_t*)y; a.ldy = ldy;
  a.steps_per_part = (int)ceil_div(H / 16, kNdParts);
  a.xs_stride = a.steps_per_part * 32 + 16;                // rows 16 bytes apart in bank space
  const int MR = M <= 8 ? 4 : 8;
  const size_t lds = (size_t)(M + 1) * a.xs_stride + (size_t)kNdWaves * 1 * MR * 64 * sizeof(float);
  if (lds > 128 * 1024) return QERL_ERR_SHAPE;             // cannot happen for H <= 8192; keeps the launch legal
  hipStream_t st = (hipStream_t)stream;
  const bool wide = H > 4096;
  if (MR == 4) return wide ? launch_norm_down<4, 16>(a, lds, st) : launch_norm_down<4, 8>(a, lds, st);
  return wide ? launch_norm_down<8, 16>(a, lds, st) : launch_norm_down<8, 8>(a, lds, st);
}

#ifdef QERL_ND_TRACE
extern "C" QERL_API int qerl_debug_read_nd_trace(void* dst, size_t bytes) {
  return (int)hipMemcpyFromSymbol(dst, HIP_SYMBOL(qerl::g_nd_trace), bytes, 0, hipMemcpyDeviceToHost);
}
#endif
