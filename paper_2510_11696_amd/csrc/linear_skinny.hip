// Decode-sized NVFP4 + LoRA linear for gfx950: up to 16 tokens per pass.
//
//   y[m,n] = S32 * sum_k x[m,k] * (s[n,k/16] * e[n,k])  +  lora_scale * sum_j t[m,j] * B[n,j]
//   t[m,j] = sum_k x[m,k] * A[j,k]                                   (Eq. 6 and Eq. 2)
//
// The op is bound by streaming the packed weights (0.5625 B per weight), so
// the kernel is organised around getting every byte requested early and
// touching it once:
//   * A wave owns a K-slice of KT*256 inputs.  It loads x for that slice once,
//     directly in the MFMA B-operand layout, and keeps it in registers
//     (tokens beyond M are zero columns).  No LDS and no barrier in the loop.
//   * It then walks T tiles of 16 output rows.  Per tile and 256 inputs a lane
//     owns 64 consecutive weights of one row: two 16-byte loads of codes and
//     one 4-byte load of scales, all issued before the first use.
//   * E2M1 -> fp32 by v_cvt_scalef32_pk_f32_fp4, times the E4M3 scale in fp32,
//     packed to bf16.  The product has at most 6 significant bits, so the bf16
//     operand is exact and v_mfma_f32_16x16x32_bf16 accumulates in fp32.
//     S32 is applied once per wave, after its K-slice is summed.
//   * Waves of a workgroup cover different K-slices of the same rows and are
//     summed through LDS in wave order.  If K needs more than one workgroup
//     (gridDim.y = S > 1) each writes its partial tile to the workspace and the
//     last one to arrive adds the S partials in slice order, so the result does
//     not depend on arrival order.  Arrival counters reset themselves.
//   * The same kernel with bf16 "weights" computes the LoRA down-projection t.
//
// Lane layout of v_mfma_f32_16x16x32_bf16 (A: 16 x 32, B: 32 x 16, D: 16 x 16):
//   A: lane l holds row l%16, k = 8*(l/16) .. +7      (weights, row = output n)
//   B: lane l holds col l%16, k = 8*(l/16) .. +7      (x, col = token)
//   D: lane l holds col l%16, rows 4*(l/16) .. +3
// Within a 256-input tile the MFMA issued at step j (0..7) multiplies the
// inputs k = 64*g + 8*j + i (g = l/16, i = 0..7) -- any bijection works as
// long as both operands use it, and this one makes every lane's weights
// contiguous in memory.
#include "linear.hpp"

namespace qerl {

__device__ __forceinline__ bf16x8 dequant8(uint32_t codes, float s) {
  const f32x2 p0 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(codes, 1.0f, 0);
  const f32x2 p1 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(codes, 1.0f, 1);
  const f32x2 p2 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(codes, 1.0f, 2);
  const f32x2 p3 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(codes, 1.0f, 3);
  u32x4 o;
  o[0] = pack_bf16x2(p0.x * s, p0.y * s);
  o[1] = pack_bf16x2(p1.x * s, p1.y * s);
  o[2] = pack_bf16x2(p2.x * s, p2.y * s);
  o[3] = pack_bf16x2(p3.x * s, p3.y * s);
  return __builtin_bit_cast(bf16x8, o);
}

// Byte `b` of `v` as an OCP E4M3 value (v_cvt_f32_fp8 with a byte select; on
// gfx950 the instruction follows the OCP format).  `b` folds to a constant once
// the caller's loop is unrolled.
__device__ __forceinline__ float e4m3_byte_to_f32(uint32_t v, int b) {
  switch (b) {
    case 0: return __builtin_amdgcn_cvt_f32_fp8(v, 0);
    case 1: return __builtin_amdgcn_cvt_f32_fp8(v, 1);
    case 2: return __builtin_amdgcn_cvt_f32_fp8(v, 2);
    default: return __builtin_amdgcn_cvt_f32_fp8(v, 3);
  }
}

constexpr int kMaxWaves = 8;

template <int KT, int T, int FMT>
__global__ __launch_bounds__(kMaxWaves * 64) void skinny_kernel(const SkinnyArgs a) {
  const int tid = threadIdx.x, lane = tid & 63, nwaves = blockDim.x >> 6;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform
  const int r16 = lane & 15, g = lane >> 4;
  const int64_t kwave = ((int64_t)blockIdx.y * nwaves + wave) * (KT * 256) + 64 * g;
  const int tile0 = blockIdx.x * T;

  // ---- x fragments for this wave's K-slice (B operand), kept in registers
  bf16x8 xf[KT][8];
#pragma unroll
  for (int i = 0; i < KT; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int64_t k = kwave + i * 256 + 8 * j;
      u32x4 v = {0u, 0u, 0u, 0u};
      if (r16 < a.M && k < a.K) v = *reinterpret_cast<const u32x4*>(a.x + (int64_t)r16 * a.ldx + k);
      xf[i][j] = __builtin_bit_cast(bf16x8, v);
    }

  f32x4 acc[T];
#pragma unroll
  for (int t = 0; t < T; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};

  // LoRA up-projection  sum_j t[m,j] * B[n,j]  as MFMAs over j, done by one
  // wave per output tile (wave 0 of the first K-slice).  t is fp32; it is split
  // into three bf16 terms (t = hi + mid + lo up to 2^-27 |t|), whose products
  // with the bf16 B are exact, so the branch keeps fp32 accuracy.
  f32x4 lacc[T];
#pragma unroll
  for (int t = 0; t < T; ++t) lacc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
  if constexpr (FMT == kFmtNvfp4) {
    if (a.r > 0 && wave == 0 && blockIdx.y == 0) {
      for (int jb = 0; jb < a.r; jb += 32) {
        const int j0 = jb + 8 * g;
        float tv[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) tv[i] = 0.f;
        if (r16 < a.M) {
          const float* tp = a.t_in + (int64_t)r16 * a.r + j0;
          if (a.b_vec) {
            if (j0 < a.r) {
              const f32x4 t0 = *reinterpret_cast<const f32x4*>(tp), t1 = *reinterpret_cast<const f32x4*>(tp + 4);
              tv[0] = t0[0]; tv[1] = t0[1]; tv[2] = t0[2]; tv[3] = t0[3];
              tv[4] = t1[0]; tv[5] = t1[1]; tv[6] = t1[2]; tv[7] = t1[3];
            }
          } else {
#pragma unroll
            for (int i = 0; i < 8; ++i)
              if (j0 + i < a.r) tv[i] = tp[i];
          }
        }
        u32x4 th, tm, tl;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const uint32_t h = pack_bf16x2(tv[2 * i], tv[2 * i + 1]);
          const float r0 = tv[2 * i] - bf16_bits_to_f32(h & 0xffffu), r1 = tv[2 * i + 1] - __uint_as_float(h & 0xffff0000u);
          const uint32_t m = pack_bf16x2(r0, r1);
          const float q0 = r0 - bf16_bits_to_f32(m & 0xffffu), q1 = r1 - __uint_as_float(m & 0xffff0000u);
          th[i] = h; tm[i] = m; tl[i] = pack_bf16x2(q0, q1);
        }
#pragma unroll
        for (int t = 0; t < T; ++t) {
          int64_t row = (int64_t)(tile0 + t) * 16 + r16;
          row = row < a.N ? row : a.N - 1;
          const uint16_t* bp = a.B + row * a.r + j0;
          u32x4 b = {0u, 0u, 0u, 0u};
          if (a.b_vec) {
            if (j0 < a.r) b = *reinterpret_cast<const u32x4*>(bp);
          } else {
#pragma unroll
            for (int i = 0; i < 8; ++i)
              if (j0 + i < a.r) b[i >> 1] |= (uint32_t)bp[i] << (16 * (i & 1));
          }
          const bf16x8 bf = __builtin_bit_cast(bf16x8, b);
          lacc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bf, __builtin_bit_cast(bf16x8, th), lacc[t], 0, 0, 0);
          lacc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bf, __builtin_bit_cast(bf16x8, tm), lacc[t], 0, 0, 0);
          lacc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bf, __builtin_bit_cast(bf16x8, tl), lacc[t], 0, 0, 0);
        }
      }
    }
  }

  if constexpr (FMT == kFmtNvfp4) {
    u32x4 c0[T][KT], c1[T][KT];
    uint32_t sc[T][KT];
#pragma unroll
    for (int t = 0; t < T; ++t) {
      int64_t row = (int64_t)(tile0 + t) * 16 + r16;
      row = row < a.N ? row : a.N - 1;
#pragma unroll
      for (int i = 0; i < KT; ++i) {
        const int64_t k = kwave + i * 256;
        c0[t][i] = u32x4{0u, 0u, 0u, 0u};
        c1[t][i] = u32x4{0u, 0u, 0u, 0u};
        sc[t][i] = 0u;
        if (k < a.K) {
          const uint8_t* cp = a.codes + row * (a.K / 2) + k / 2;
          c0[t][i] = *reinterpret_cast<const u32x4*>(cp);
          c1[t][i] = *reinterpret_cast<const u32x4*>(cp + 16);
          sc[t][i] = *reinterpret_cast<const uint32_t*>(a.scales + row * (a.K / 16) + k / 16);
        }
      }
    }
#pragma unroll
    for (int t = 0; t < T; ++t)
#pragma unroll
      for (int i = 0; i < KT; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const uint32_t d = j < 4 ? c0[t][i][j & 3] : c1[t][i][j & 3];
          const float s = e4m3_byte_to_f32(sc[t][i], j >> 1);
          acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(dequant8(d, s), xf[i][j], acc[t], 0, 0, 0);
        }
  } else {
    // bf16 rows (LoRA A): a lane's 64 inputs are 128 contiguous bytes.
#pragma unroll
    for (int t = 0; t < T; ++t) {
      int64_t row = (int64_t)(tile0 + t) * 16 + r16;
      row = row < a.N ? row : a.N - 1;
      u32x4 w[KT][8];
#pragma unroll
      for (int i = 0; i < KT; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int64_t k = kwave + i * 256 + 8 * j;
          w[i][j] = u32x4{0u, 0u, 0u, 0u};
          if (k < a.K) w[i][j] = *reinterpret_cast<const u32x4*>(a.wbf16 + row * a.K + k);
        }
#pragma unroll
      for (int i = 0; i < KT; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j)
          acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, w[i][j]), xf[i][j],
                                                           acc[t], 0, 0, 0);
    }
  }

  // ---- sum the waves of this workgroup (different K-slices), in wave order
  __shared__ f32x4 red[kMaxWaves][T][64];
  __shared__ int s_last;
  if constexpr (FMT == kFmtNvfp4) {
    const float S32 = *a.tensor_scale;
#pragma unroll
    for (int t = 0; t < T; ++t) acc[t] = acc[t] * S32 + lacc[t] * a.lora_scale;
  }
#pragma unroll
  for (int t = 0; t < T; ++t) red[wave][t][lane] = acc[t];
  __syncthreads();
  constexpr int kSlots = T * 64;
  f32x4 v[T];   // a thread owns slots tid, tid + blockDim.x, ... (at most T of them)
#pragma unroll
  for (int q = 0; q < T; ++q) {
    const int slot = tid + q * (int)blockDim.x;
    v[q] = f32x4{0.f, 0.f, 0.f, 0.f};
    if (slot < kSlots) {
      f32x4 s = red[0][slot >> 6][slot & 63];
      for (int w = 1; w < nwaves; ++w) s += red[w][slot >> 6][slot & 63];
      v[q] = s;
    }
  }

  // ---- more than one workgroup along K: exchange partial tiles
  const int S = gridDim.y;
  if (S > 1) {
    // Partial tiles travel through memory with agent-scope atomic accesses
    // (sc1: written through / read past the per-XCD L2), so no cache-wide
    // write-back or invalidate is needed; each wave waits for its own stores
    // to complete before the barrier that precedes the arrival count.
    uint32_t* pw = reinterpret_cast<uint32_t*>(a.partial);
#pragma unroll
    for (int q = 0; q < T; ++q) {
      const int slot = tid + q * (int)blockDim.x;
      const int tile = tile0 + (slot >> 6);
      if (slot < kSlots && tile < a.n_tiles) {
        uint32_t* dst = pw + (((int64_t)blockIdx.y * a.n_tiles + tile) * 64 + (slot & 63)) * 4;
#pragma unroll
        for (int i = 0; i < 4; ++i)
          __hip_atomic_store(dst + i, __float_as_uint(v[q][i]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's partial stores have completed
    __syncthreads();
    if (tid == 0) {
      const uint32_t old = __hip_atomic_fetch_add(a.counters + blockIdx.x, 1u, __ATOMIC_RELAXED,
                                                  __HIP_MEMORY_SCOPE_AGENT);
      s_last = (old == (uint32_t)(S - 1));
    }
    __syncthreads();
    if (!s_last) return;
#pragma unroll
    for (int q = 0; q < T; ++q) {
      const int slot = tid + q * (int)blockDim.x;
      const int tile = tile0 + (slot >> 6);
      if (slot < kSlots && tile < a.n_tiles) {
        const uint32_t* src = pw + ((int64_t)tile * 64 + (slot & 63)) * 4;
        f32x4 s;
#pragma unroll
        for (int i = 0; i < 4; ++i) s[i] = ordered_sum_sc1(src + i, (int64_t)a.n_tiles * 256, S);
        v[q] = s;
      }
    }
    if (tid == 0) __hip_atomic_store(a.counters + blockIdx.x, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }

  // ---- epilogue
#pragma unroll
  for (int nv = 0; nv < T; ++nv) {
    const int slot = tid + nv * (int)blockDim.x;
    const int l = slot & 63, token = l & 15;
    const int64_t nb = (int64_t)(tile0 + (slot >> 6)) * 16 + 4 * (l >> 4);
    if (slot >= kSlots || token >= a.M || nb >= a.N) continue;
    if constexpr (FMT == kFmtBf16) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (nb + i < a.N) a.t_out[(int64_t)token * a.N + nb + i] = v[nv][i];
    } else {
      const float o[4] = {v[nv][0], v[nv][1], v[nv][2], v[nv][3]};
      uint16_t* yp = a.y + (int64_t)token * a.ldy + nb;
      if (a.y_vec && nb + 3 < a.N) {
        *reinterpret_cast<u32x2*>(yp) = u32x2{pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3])};
      } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (nb + i < a.N) yp[i] = (uint16_t)f32_to_bf16_bits(o[i]);
      }
    }
  }
}

// ---- host ---------------------------------------------------------------------------------

static int g_force_kt = 0, g_force_t = 0;

SkinnyPlan plan_skinny(int64_t N, int64_t K, int fmt) {
  SkinnyPlan p;
  const int64_t tiles = ceil_div(K, 256);
  p.n_tiles = (int)ceil_div(N, 16);
  if (fmt == kFmtBf16) {
    // LoRA down-projection: few rows, so spread K over many small workgroups
    // (two waves, 512 inputs) and let the last one to arrive add the partials.
    p.KT = 1;
    p.T = 1;
    p.waves = tiles >= 2 ? 2 : 1;
    p.S = (int)ceil_div(tiles, p.waves);
    p.groups = p.n_tiles;
    return p;
  }
  p.KT = (tiles >= 2) ? 2 : 1;
  if (g_force_kt) p.KT = g_force_kt;
  const int64_t slices = ceil_div(tiles, p.KT);
  p.S = (int)ceil_div(slices, kMaxWaves);
  p.waves = (int)ceil_div(slices, p.S);
  // rows per workgroup: aim at one resident round of workgroups on 256 CUs
  const int64_t want = 256;
  int T = 1;
  const int cand[3] = {1, 2, 4};
  for (int c : cand)
    if (ceil_div(p.n_tiles, c) * p.S >= want) T = c;
  if (g_force_t) T = g_force_t;
  p.T = T;
  p.groups = (int)ceil_div(p.n_tiles, p.T);
  return p;
}

template <int KT, int T, int FMT>
static void launch_one(const SkinnyPlan& p, const SkinnyArgs& a, hipStream_t st) {
  skinny_kernel<KT, T, FMT><<<dim3(p.groups, p.S), dim3(p.waves * 64), 0, st>>>(a);
}

int launch_skinny(const SkinnyPlan& p, const SkinnyArgs& a, int fmt, hipStream_t st) {
  // every pointer the kernel dereferences must be set by the caller
  if (!a.x || !a.partial || !a.counters) return QERL_ERR_NULL;
  if (fmt == kFmtNvfp4 && (!a.codes || !a.scales || !a.tensor_scale || !a.y || (a.r > 0 && (!a.t_in || !a.B))))
    return QERL_ERR_NULL;
  if (fmt == kFmtBf16 && (!a.wbf16 || !a.t_out)) return QERL_ERR_NULL;
  if (a.M < 1 || a.M > 16 || a.N < 1 || a.K < 64 || a.K % 64 != 0 || p.waves < 1 || p.waves > kMaxWaves)
    return QERL_ERR_SHAPE;
#define QERL_CASE(kt, t)                                                     \
  if (p.KT == kt && p.T == t) {                                              \
    if (fmt == kFmtNvfp4) launch_one<kt, t, kFmtNvfp4>(p, a, st);            \
    else launch_one<kt, t, kFmtBf16>(p, a, st);                              \
    return launch_status();                                                  \
  }
  QERL_CASE(1, 1) QERL_CASE(1, 2) QERL_CASE(1, 4)
  QERL_CASE(2, 1) QERL_CASE(2, 2) QERL_CASE(2, 4)
#undef QERL_CASE
  return QERL_ERR_SHAPE;
}

}  // namespace qerl

// Tuning hook for experiments (not part of the public header): force the
// K-tiles per wave (1 or 2) and rows-per-workgroup factor (1, 2, 4); 0 = automatic.
#ifdef QERL_TUNING_HOOKS   // built only for tuning sessions: they change process-wide state
extern "C" QERL_API void qerl_debug_force_skinny(int kt, int t) {
  qerl::g_force_kt = kt;
  qerl::g_force_t = t;
}
#endif  // QERL_TUNING_HOOKS
