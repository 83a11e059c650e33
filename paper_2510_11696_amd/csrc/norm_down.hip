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
// QERL_T_PARTS workgroups of 512 threads; workgroup p owns the p-th slice of K (whole 16-input steps):
//   1. all of x is read once, rows in registers, and each row's sum of squares is formed exactly as
//      aqn_rmsnorm forms it (256 threads per row, same element order, same reduction tree), so y is
//      bit-identical to what aqn_rmsnorm writes;
//   2. the slice's columns of every row are normalised, rounded, written to y and kept in LDS;
//   3. the eight waves split the slice's steps: x fragment from LDS, A fragments of all stacked ranks
//      (requested first thing in the kernel) from registers, one accumulator tile per 32 stacked ranks;
//   4. the eight waves' tiles are added in wave order and stored as part p of every adapter's t.
// No workgroup depends on another, and every sum has a fixed order.
#include "common.hpp"

namespace qerl {

constexpr int kNdThreads = 512, kNdWaves = 8, kNdRowThreads = 256;
constexpr int kNdMaxAdapters = 4;
constexpr int kNdParts = QERL_T_PARTS;
constexpr int kNdMaxTiles = 4;             // 32-rank tiles of the stacked adapters: sum of ranks <= 128
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

// MR: accumulator registers that hold live tokens (4 for M <= 8, 8 for M <= 16); NCH: 16-byte chunks of a row
// per thread (2: H <= 4096, 4: H <= 8192); NT: 32-rank tiles
template <int MR, int NCH, int NT>
__global__ __launch_bounds__(kNdThreads) void norm_down_kernel(const NormDownArgs a) {
  extern __shared__ __attribute__((aligned(256))) unsigned char smem[];   // slice of y [(M+1) rows][xs_stride]; red after it
  __shared__ float s_part[16][4];          // per row: the four wave sums of its 256 threads
  constexpr int kRowsPerThread = MR == 4 ? 4 : 8;   // rows half, half + 2, ... of this thread's half
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int half = wave >> 2, rt = tid & (kNdRowThreads - 1);   // which of two concurrent rows; thread within the row
  const int chunks = (int)(a.H / 8);
  const int n32 = lane & 31, kg = lane >> 5;
  const int part = (int)blockIdx.x;
  const int n_steps = (int)(a.H / 16);
  const int step0 = part * a.steps_per_part;
  const int step1 = step0 + a.steps_per_part < n_steps ? step0 + a.steps_per_part : n_steps;
  NDT(0);

  // ---- 1. read x (requested first: it is needed first) ...
  u32x4 reg[kRowsPerThread][NCH];
  float ss[kRowsPerThread];
#pragma unroll
  for (int p = 0; p < kRowsPerThread; ++p) {
    const int row = 2 * p + half;
    ss[p] = 0.f;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = rt + i * kNdRowThreads;
      reg[p][i] = u32x4{0u, 0u, 0u, 0u};
      if (row < a.M && c < chunks) reg[p][i] = reinterpret_cast<const u32x4*>(a.x + (int64_t)row * a.ldx)[c];
    }
  }
  // gain and noise of the chunks this thread normalises: also requested up front
  const int c_lo = step0 * 2, c_hi = step1 * 2;          // 16-byte chunks of the slice
  const u32x4* __restrict__ gr = reinterpret_cast<const u32x4*>(a.gain);
  const f32x4* __restrict__ zr = reinterpret_cast<const f32x4*>(a.noise);
  u32x4 gq[NCH];
  f32x4 zq[NCH][2];
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = rt + i * kNdRowThreads;
    gq[i] = u32x4{0u, 0u, 0u, 0u};
    zq[i][0] = f32x4{0.f, 0.f, 0.f, 0.f}; zq[i][1] = zq[i][0];
    if (c >= c_lo && c < c_hi) {
      gq[i] = gr[c];
      if (zr) { zq[i][0] = zr[2 * c]; zq[i][1] = zr[2 * c + 1]; }
    }
  }

  // ---- A fragments of this wave's steps, all rank tiles: requested before x is even looked at (they depend on
  // nothing), so their latency overlaps the normalisation; behind x, which is needed first.  Wave w takes steps step0 + w, step0 + w + 8, ...
  const uint16_t* arow[NT];
  bool live[NT];
#pragma unroll
  for (int tl = 0; tl < NT; ++tl) {
    const int s = tl * 32 + n32;           // stacked rank this lane feeds in tile tl
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

  // ... sum of squares per row in aqn_rmsnorm's order
#pragma unroll
  for (int p = 0; p < kRowsPerThread; ++p) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      if (rt + i * kNdRowThreads < chunks) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float lo = bf16_bits_to_f32(reg[p][i][j] & 0xffffu), hi = bf16_bits_to_f32(reg[p][i][j] >> 16);
          ss[p] += lo * lo;
          ss[p] += hi * hi;
        }
      }
    }
    if (p == 0) NDT(1);
    const float ws = wave_sum(ss[p]);
    if (lane == 0 && 2 * p + half < 16) s_part[2 * p + half][wave & 3] = ws;
  }
  __syncthreads();
  NDT(2);

  // ---- 2. normalise and round the slice's columns: to y and to LDS (A-operand rows)
  float inv[kRowsPerThread];
#pragma unroll
  for (int p = 0; p < kRowsPerThread; ++p) {
    const int row = (2 * p + half) & 15;
    const float total = ((s_part[row][0] + s_part[row][1]) + s_part[row][2]) + s_part[row][3];
    inv[p] = 1.0f / sqrtf(total / (float)a.H + a.eps);
  }
#pragma unroll
  for (int p = 0; p < kRowsPerThread; ++p) {
    const int row = 2 * p + half;
    if (row < a.M) {
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
        const int c = rt + i * kNdRowThreads;
        if (c >= c_lo && c < c_hi) {
          const float z[8] = {zq[i][0][0], zq[i][0][1], zq[i][0][2], zq[i][0][3], zq[i][1][0], zq[i][1][1], zq[i][1][2], zq[i][1][3]};
          u32x4 o;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const float ga = bf16_bits_to_f32(gq[i][j] & 0xffffu) + z[2 * j];
            const float gb = bf16_bits_to_f32(gq[i][j] >> 16) + z[2 * j + 1];
            const float xa = bf16_bits_to_f32(reg[p][i][j] & 0xffffu), xb = bf16_bits_to_f32(reg[p][i][j] >> 16);
            o[j] = pack_bf16x2(ga * (xa * inv[p]), gb * (xb * inv[p]));
          }
          *reinterpret_cast<u32x4*>(smem + row * a.xs_stride + (c - c_lo) * 16) = o;
          reinterpret_cast<u32x4*>(a.y + (int64_t)row * a.ldy)[c] = o;
        }
      }
    }
  }
  NDT(3);
  for (int c = tid; c < c_hi - c_lo; c += kNdThreads)   // tokens >= M read this zero row
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
    const int tok = 8 * (q >> 2) + 4 * (l >> 5) + (q & 3), s = tl * 32 + (l & 31);
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

template <int MR, int NCH, int NT>
static int launch_norm_down_t(const NormDownArgs& a, size_t lds, hipStream_t st) {
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&norm_down_kernel<MR, NCH, NT>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024) != hipSuccess)
      return launch_status();
    attr_set = true;
  }
  norm_down_kernel<MR, NCH, NT><<<kNdParts, kNdThreads, lds, st>>>(a);
  return launch_status();
}
template <int MR, int NCH>
static int launch_norm_down(const NormDownArgs& a, size_t lds, hipStream_t st) {
  switch (a.n_tiles) {
    case 1: return launch_norm_down_t<MR, NCH, 1>(a, lds, st);
    case 2: return launch_norm_down_t<MR, NCH, 2>(a, lds, st);
    case 3: return launch_norm_down_t<MR, NCH, 3>(a, lds, st);
    default: return launch_norm_down_t<MR, NCH, 4>(a, lds, st);
  }
}

extern "C" int aqn_rmsnorm_lora_down(const void* x, int64_t M, int64_t H, int64_t ldx, const void* gain,
                                     const float* noise, float eps, void* y, int64_t ldy,
                                     const void* const* A, const int64_t* r, float* const* t, int n_adapters,
                                     void* stream) {
  if (M < 0 || M > 16 || H < 1 || ldx < H || ldy < H) return QERL_ERR_SHAPE;
  if (n_adapters < 1 || n_adapters > kNdMaxAdapters) return QERL_ERR_SHAPE;
  if (!x || !gain || !y || !A || !r || !t) return QERL_ERR_NULL;
  if (H % 16 != 0 || H > 8 * kNdRowThreads * 4) return QERL_ERR_SHAPE;
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
  const size_t lds = (size_t)(M + 1) * a.xs_stride + (size_t)kNdWaves * a.n_tiles * MR * 64 * sizeof(float);
  if (lds > 128 * 1024) return QERL_ERR_SHAPE;             // cannot happen for H <= 8192; keeps the launch legal
  hipStream_t st = (hipStream_t)stream;
  const bool wide = H > 8 * kNdRowThreads * 2;
  if (MR == 4) return wide ? launch_norm_down<4, 4>(a, lds, st) : launch_norm_down<4, 2>(a, lds, st);
  return wide ? launch_norm_down<8, 4>(a, lds, st) : launch_norm_down<8, 2>(a, lds, st);
}

#ifdef QERL_ND_TRACE
extern "C" QERL_API int qerl_debug_read_nd_trace(void* dst, size_t bytes) {
  return (int)hipMemcpyFromSymbol(dst, HIP_SYMBOL(qerl::g_nd_trace), bytes, 0, hipMemcpyDeviceToHost);
}
#endif
