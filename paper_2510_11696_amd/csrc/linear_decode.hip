// Decode path (M <= 16 tokens) of the NVFP4 + LoRA linear on tile-packed weights.
//
//   y[m,n] = S32 * sum_b s[n,b] * ( sum_{k in block b} x[m,k] * e[n,k] )        (Eq. 6)
//          + lora_scale * sum_j t[m,j] * B[n,j]                                  (Eq. 2)
//
// Memory bound: 0.5625 B per weight must stream from HBM once.  Everything
// else is arranged so the vector ALU does not become the limit before HBM does:
//
//   * The E4M3 block scale is applied to the ACCUMULATOR, not to the weights.
//     One v_mfma_f32_32x32x16_bf16 multiplies 16 inputs -- exactly one scale
//     block -- of 32 output rows by the tokens; the weights enter it as bare
//     E2M1 values (v_cvt_scalef32_pk_bf16_fp4, 4 per step), and the 32x32
//     product is folded into the running sums with one fp32 FMA per live token
//     row: acc += s * tmp.  With the weights as the MFMA's B operand a lane
//     owns one output row n in both the operand and the result, so the scale
//     it needs is its own.  Per 512 weights: 4 cvt + 1 scale decode + MR FMAs
//     (MR = 4 for M <= 8, 8 for M <= 16) instead of ~20 ops for dequantising
//     to bf16 first.  Every product and partial sum is exact or fp32.
//   * Weights are read from the tile-packed layout below: each wave load
//     instruction covers 1 KiB of consecutive bytes.
//   * A wave owns KW K-tiles (128 inputs each) of T row-tiles (32 rows each),
//     keeps its x slice in registers in operand layout (tokens >= M are zero
//     rows) and issues every load before the first use.  The waves of a
//     workgroup cover different K-tiles of the same rows and are summed through
//     LDS in wave order; if K needs several workgroups (gridDim.y = S) they
//     exchange partial tiles through the workspace and the last to arrive adds
//     them in slice order (deterministic).
//   * LoRA in the same launch: the first few workgroups of the grid compute
//     t = x A^T (bf16 MFMAs, partial sums exchanged through the workspace) and
//     raise a ready word; in every other workgroup one wave is set aside for
//     the up-projection: it preloads its B rows, waits for the ready word
//     (bounded; workgroups are dispatched in index order, so the producers are
//     already running), reads t, splits it into three bf16 terms (exact to
//     2^-27 |t|) and multiplies by B with MFMAs over j while the other waves
//     stream the weights.  The last reader re-arms the control words.
//
// Packed layout ("P32"): rows padded to 32, K padded to 128, zero filled.
//   tile (nt, kt) at byte ((nt * k_tiles + kt) * 2304):
//     [   0, 1024)  codes, steps 0..3 : lane l owns 16 bytes at l*16
//     [1024, 2048)  codes, steps 4..7 : same
//     [2048, 2304)  scales            : row n owns 8 bytes at n*8 (one per step)
//   lane l = (n = l % 32, kg = l / 32); step j = 16-input block j of the tile;
//   dword (j % 4) of the lane's 16 bytes holds the 8 codes of inputs
//   128*kt + 16*j + 8*kg + (0..7) of row 32*nt + n, low nibble first.
//
// v_mfma_f32_32x32x16_bf16 operand layout (A: 32x16, B: 16x32, D: 32x32):
//   A: lane l -> row l%32, k = 8*(l/32) + i       (x: row = token)
//   B: lane l -> col l%32, k = 8*(l/32) + i       (weights: col = output row n)
//   D: lane l -> col l%32, register i -> row 8*(i/4) + 4*(l/32) + i%4
#include "linear.hpp"

namespace qerl {

constexpr int kDecMaxWaves = 8;

__device__ __forceinline__ bf16x8 e2m1x8_to_bf16(uint32_t codes) {
  const bf16x2 p0 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(codes, 1.0f, 0);
  const bf16x2 p1 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(codes, 1.0f, 1);
  const bf16x2 p2 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(codes, 1.0f, 2);
  const bf16x2 p3 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(codes, 1.0f, 3);
  u32x4 o = {__builtin_bit_cast(uint32_t, p0), __builtin_bit_cast(uint32_t, p1),
             __builtin_bit_cast(uint32_t, p2), __builtin_bit_cast(uint32_t, p3)};
  return __builtin_bit_cast(bf16x8, o);
}

__device__ __forceinline__ float e4m3_byte(uint32_t v, int b) {
  switch (b) {
    case 0: return __builtin_amdgcn_cvt_f32_fp8(v, 0);
    case 1: return __builtin_amdgcn_cvt_f32_fp8(v, 1);
    case 2: return __builtin_amdgcn_cvt_f32_fp8(v, 2);
    default: return __builtin_amdgcn_cvt_f32_fp8(v, 3);
  }
}

// fp32 x8 -> three bf16 x8 terms with hi + mid + lo = v up to 2^-27 |v|
__device__ __forceinline__ void split3(const float (&v)[8], u32x4& hi, u32x4& mid, u32x4& lo) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t h = pack_bf16x2(v[2 * i], v[2 * i + 1]);
    const float r0 = v[2 * i] - bf16_bits_to_f32(h & 0xffffu), r1 = v[2 * i + 1] - __uint_as_float(h & 0xffff0000u);
    const uint32_t m = pack_bf16x2(r0, r1);
    const float q0 = r0 - bf16_bits_to_f32(m & 0xffffu), q1 = r1 - __uint_as_float(m & 0xffff0000u);
    hi[i] = h; mid[i] = m; lo[i] = pack_bf16x2(q0, q1);
  }
}

// Control words of the in-kernel LoRA hand-over (in the workspace, zero between calls).
constexpr int kCtlArrive = 0;   // producer workgroups that have stored their partial t
constexpr int kCtlReady = 1;    // 1 once t is complete
constexpr int kCtlDone = 2;     // consumer workgroups that have read t
constexpr uint32_t kSpinLimit = 1u << 14;   // polls, about a microsecond apart, before giving up with NaN

// ---- LoRA down-projection  t[tok][j] = sum_k x[tok,k] * A[j,k]  (r <= 64) on the first workgroups of
// the grid.  Their waves stride over the K-tiles, are summed through LDS, exchange partial sums through
// the workspace, and the last one to arrive publishes t and raises the ready word.
template <int MR>
__device__ __forceinline__ void lora_down_producer(const DecodeArgs& a, float* red, int* s_last) {
  const int tid = threadIdx.x, lane = tid & 63, nthreads = blockDim.x, nwaves = nthreads >> 6;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform
  const int n32 = lane & 31, kg = lane >> 5;
  const int P = a.n_producers, n_at = (a.r + 31) >> 5;
  f32x16 pacc[2];
#pragma unroll
  for (int at = 0; at < 2; ++at)
#pragma unroll
    for (int i = 0; i < 16; ++i) pacc[at][i] = 0.f;
  // half K-tiles (64 inputs, 4 MFMA steps) keep the register footprint below the consumer path's
  for (int64_t h = (int64_t)blockIdx.x * nwaves + wave; h < 2 * a.k_tiles; h += (int64_t)P * nwaves) {
    u32x4 xa[4], af[2][4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int64_t k = h * 64 + 16 * j + 8 * kg;
      xa[j] = u32x4{0u, 0u, 0u, 0u};
      if (n32 < a.M && k < a.K) xa[j] = *reinterpret_cast<const u32x4*>(a.x + (int64_t)n32 * a.ldx + k);
#pragma unroll
      for (int at = 0; at < 2; ++at) {
        const int row = at * 32 + n32;
        af[at][j] = u32x4{0u, 0u, 0u, 0u};
        if (row < a.r && k < a.K) af[at][j] = *reinterpret_cast<const u32x4*>(a.A + (int64_t)row * a.K + k);
      }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      pacc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, xa[j]),
                                                        __builtin_bit_cast(bf16x8, af[0][j]), pacc[0], 0, 0, 0);
      if (n_at > 1)
        pacc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, xa[j]),
                                                          __builtin_bit_cast(bf16x8, af[1][j]), pacc[1], 0, 0, 0);
    }
  }
  // red[wave][at][q][lane]
  constexpr int kElems = 2 * MR * 64;
#pragma unroll
  for (int at = 0; at < 2; ++at)
#pragma unroll
    for (int q = 0; q < MR; ++q) red[(wave * 2 + at) * MR * 64 + q * 64 + lane] = pacc[at][q];
  __syncthreads();
  constexpr int kPer = 2 * MR;   // elements per thread with a single wave
  float v[kPer];
#pragma unroll
  for (int i = 0; i < kPer; ++i) {
    const int e = tid + i * nthreads;
    v[i] = 0.f;
    if (e < kElems) {
      float s = red[e];
      for (int w = 1; w < nwaves; ++w) s += red[w * kElems + e];
      v[i] = s;
    }
  }
  if (P > 1) {
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
      const int e = tid + i * nthreads;
      if (e < kElems)
        __hip_atomic_store(a.tpart + (int64_t)blockIdx.x * kElems + e, __float_as_uint(v[i]), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    __syncthreads();
    if (tid == 0) {
      const uint32_t old = __hip_atomic_fetch_add(a.lora_ctl + kCtlArrive, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      *s_last = (old == (uint32_t)(P - 1));
    }
    __syncthreads();
    if (!*s_last) return;
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
      const int e = tid + i * nthreads;
      if (e < kElems) v[i] = ordered_sum_sc1(a.tpart + e, kElems, P);
    }
  }
#pragma unroll
  for (int i = 0; i < kPer; ++i) {
    const int e = tid + i * nthreads;
    if (e >= kElems) continue;
    const int at = e / (MR * 64), q = (e / 64) % MR, l = e & 63;
    const int tok = 8 * (q >> 2) + 4 * (l >> 5) + (q & 3), j = at * 32 + (l & 31);
    if (tok < a.M && j < a.r)
      __hip_atomic_store(reinterpret_cast<uint32_t*>(a.t) + tok * a.r + j, __float_as_uint(v[i]), __ATOMIC_RELAXED,
                         __HIP_MEMORY_SCOPE_AGENT);
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): t is written before the ready word
  __syncthreads();
  if (tid == 0) {
    __hip_atomic_store(a.lora_ctl + kCtlArrive, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(a.lora_ctl + kCtlReady, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

template <int KW, int T, int MR>
__global__ __launch_bounds__(kDecMaxWaves * 64) void decode32_kernel(const DecodeArgs a) {
  constexpr int kRedConsumer = kDecMaxWaves * T * MR * 64, kRedProducer = kDecMaxWaves * 2 * MR * 64;
  __shared__ float red[kRedConsumer > kRedProducer ? kRedConsumer : kRedProducer];
  __shared__ int s_last;
  if ((int)blockIdx.x < a.n_producers) {
    lora_down_producer<MR>(a, red, &s_last);
    return;
  }
  const int tid = threadIdx.x, lane = tid & 63, nthreads = blockDim.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps everything derived from it in SGPRs
  const int nwaves = nthreads >> 6;
  const int n32 = lane & 31, kg = lane >> 5;
  const int S = a.S;
  const int cid = (int)blockIdx.x - a.n_producers, group = cid / S, slice = cid - group * S;
  const int tile0 = group * T;
  // With LoRA the last wave of the block does the up-projection instead of a K-slice.
  const bool lora_wave = a.r > 0 && wave == nwaves - 1;
  const int main_waves = a.r > 0 ? nwaves - 1 : nwaves;
  auto red_at = [&](int w, int t, int q) -> float& { return red[((w * T + t) * MR + q) * 64 + lane]; };

  if (!lora_wave) {
    const int64_t kt0 = ((int64_t)slice * main_waves + wave) * KW;
    // ---- x slice in A-operand layout
    u32x4 xa[KW][8];
#pragma unroll
    for (int i = 0; i < KW; ++i)
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int64_t k = (kt0 + i) * 128 + 16 * j + 8 * kg;
        xa[i][j] = u32x4{0u, 0u, 0u, 0u};
        if (n32 < a.M && k < a.K) xa[i][j] = *reinterpret_cast<const u32x4*>(a.x + (int64_t)n32 * a.ldx + k);
      }
    // ---- packed weights: every load issued before the first use
    u32x4 c[T][KW][2];
    u32x2 sc[T][KW];
#pragma unroll
    for (int t = 0; t < T; ++t) {
      int nt = tile0 + t;
      nt = nt < a.n_tiles ? nt : a.n_tiles - 1;
#pragma unroll
      for (int i = 0; i < KW; ++i) {
        c[t][i][0] = u32x4{0u, 0u, 0u, 0u};
        c[t][i][1] = u32x4{0u, 0u, 0u, 0u};
        sc[t][i] = u32x2{0u, 0u};
        if (kt0 + i < a.k_tiles) {
          const uint8_t* base = a.packed + ((int64_t)nt * a.k_tiles + kt0 + i) * kPackTileBytes;
          c[t][i][0] = *reinterpret_cast<const u32x4*>(base + lane * 16);
          c[t][i][1] = *reinterpret_cast<const u32x4*>(base + 1024 + lane * 16);
          sc[t][i] = *reinterpret_cast<const u32x2*>(base + 2048 + n32 * 8);
        }
      }
    }
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    const float S32 = *a.tensor_scale;
#pragma unroll
    for (int t = 0; t < T; ++t) {
      float acc[MR];
#pragma unroll
      for (int q = 0; q < MR; ++q) acc[q] = 0.f;
#pragma unroll
      for (int i = 0; i < KW; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const bf16x8 w = e2m1x8_to_bf16(c[t][i][j >> 2][j & 3]);
          const f32x16 tmp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, xa[i][j]), w,
                                                                     zero, 0, 0, 0);
          const float s = e4m3_byte(sc[t][i][j >> 2], j & 3);
#pragma unroll
          for (int q = 0; q < MR; ++q) acc[q] = __builtin_fmaf(s, tmp[q], acc[q]);
        }
#pragma unroll
      for (int q = 0; q < MR; ++q) red_at(wave, t, q) = acc[q] * S32;
    }
  } else {
    // ---- LoRA up-projection  lo[tok][n] = sum_j t[tok][j] * B[n][j]  on this wave
    constexpr int kPre = 4;   // 16-wide j steps whose operands are loaded up front (r <= 64)
    u32x4 th[kPre], tm[kPre], tl[kPre];
    u32x4 bq[T][kPre];
    const bool first = slice == 0;   // only the first K-slice adds the branch
#pragma unroll
    for (int s = 0; s < kPre; ++s) {
      const int j0 = 16 * s + 8 * kg;
#pragma unroll
      for (int t = 0; t < T; ++t) {
        int64_t row = (int64_t)(tile0 + t) * 32 + n32;
        row = row < a.N ? row : a.N - 1;
        bq[t][s] = u32x4{0u, 0u, 0u, 0u};
        if (first && j0 < a.r) {
          const uint16_t* bp = a.B + row * a.r + j0;
          if (a.b_vec) {
            bq[t][s] = *reinterpret_cast<const u32x4*>(bp);
          } else {
#pragma unroll
            for (int i = 0; i < 8; ++i)
              if (j0 + i < a.r) bq[t][s][i >> 1] |= (uint32_t)bp[i] << (16 * (i & 1));
          }
        }
      }
    }
    // t comes either from an earlier launch or from the producer workgroups of this launch.  In the
    // second case wait for the ready word (polled past the caches, about once a microsecond so that
    // hundreds of waiting workgroups do not crowd the one memory channel that holds it).  The producers
    // wrote t through to memory before raising the word and no cache can hold an older copy of it (caches
    // are invalidated when a kernel starts and nobody reads t before the word is up), so ordinary loads
    // are enough afterwards; the workgroup-scope fence only keeps the compiler from hoisting them.
    bool poisoned = false;
    if (first && a.n_producers > 0) {
      uint32_t spins = 0;
      while (__hip_atomic_load(a.lora_ctl + kCtlReady, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u) {
        if (++spins > kSpinLimit) {
          poisoned = true;
          if (lane == 0) __hip_atomic_fetch_or(a.lora_ctl + kCtlErr, 4u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          break;
        }
        __builtin_amdgcn_s_sleep(32);
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    }
#pragma unroll
    for (int s = 0; s < kPre; ++s) {
      const int j0 = 16 * s + 8 * kg;
      float tv[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) tv[i] = 0.f;
      if (first && n32 < a.M && j0 < a.r) {
        const float* tp = a.t + (int64_t)n32 * a.r + j0;
        if (a.b_vec) {
          const f32x4 t0 = *reinterpret_cast<const f32x4*>(tp), t1 = *reinterpret_cast<const f32x4*>(tp + 4);
          tv[0] = t0[0]; tv[1] = t0[1]; tv[2] = t0[2]; tv[3] = t0[3];
          tv[4] = t1[0]; tv[5] = t1[1]; tv[6] = t1[2]; tv[7] = t1[3];
        } else {
#pragma unroll
          for (int i = 0; i < 8; ++i)
            if (j0 + i < a.r) tv[i] = tp[i];
        }
        if (poisoned) tv[0] = __uint_as_float(0x7fc00000u);   // the hand-over timed out: make it visible
      }
      split3(tv, th[s], tm[s], tl[s]);
    }
    if (first && a.n_producers > 0 && lane == 0) {
      // every first-slice workgroup has now read t; the last of them re-arms the control words
      const uint32_t old = __hip_atomic_fetch_add(a.lora_ctl + kCtlDone, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (old == (uint32_t)(a.n_groups - 1) && __hip_atomic_load(a.lora_ctl + kCtlErr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u) {   // (not after a wait that gave up)
        __hip_atomic_store(a.lora_ctl + kCtlReady, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(a.lora_ctl + kCtlDone, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
#pragma unroll
    for (int t = 0; t < T; ++t) {
      f32x16 lo = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s = 0; s < kPre; ++s) {
        const bf16x8 bf = __builtin_bit_cast(bf16x8, bq[t][s]);
        lo = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, th[s]), bf, lo, 0, 0, 0);
        lo = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, tm[s]), bf, lo, 0, 0, 0);
        lo = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, tl[s]), bf, lo, 0, 0, 0);
      }
      // ranks beyond 64 (never with in-kernel producers): remaining steps, loaded as they come
      if (first) {
        int64_t row = (int64_t)(tile0 + t) * 32 + n32;
        row = row < a.N ? row : a.N - 1;
        for (int jb = 16 * kPre; jb < a.r; jb += 16) {
          const int j0 = jb + 8 * kg;
          float tv[8];
          u32x4 b = {0u, 0u, 0u, 0u};
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            tv[i] = 0.f;
            if (j0 + i < a.r) {
              if (n32 < a.M) tv[i] = a.t[(int64_t)n32 * a.r + j0 + i];
              b[i >> 1] |= (uint32_t)a.B[row * a.r + j0 + i] << (16 * (i & 1));
            }
          }
          u32x4 h, m, l;
          split3(tv, h, m, l);
          const bf16x8 bf = __builtin_bit_cast(bf16x8, b);
          lo = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, h), bf, lo, 0, 0, 0);
          lo = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, m), bf, lo, 0, 0, 0);
          lo = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, l), bf, lo, 0, 0, 0);
        }
      }
#pragma unroll
      for (int q = 0; q < MR; ++q) red_at(wave, t, q) = lo[q] * a.lora_scale;
    }
  }
  __syncthreads();

  // ---- sum the waves in wave order; element e = (t, q, lane)
  constexpr int kElems = T * MR * 64;
  constexpr int kPer = T * MR;       // elements per thread when the block has a single wave
  float v[kPer];
#pragma unroll
  for (int p = 0; p < kPer; ++p) {
    const int e = tid + p * nthreads;
    v[p] = 0.f;
    if (e < kElems) {
      const float* src = red + e;
      float s = src[0];
      for (int w = 1; w < nwaves; ++w) s += src[w * kElems];
      v[p] = s;
    }
  }

  if (S > 1) {
    // Partial tiles go through memory with agent-scope atomic accesses (written
    // through / read past the per-XCD L2): no cache-wide write-back or
    // invalidate.  A wave waits for its own stores before the barrier that
    // precedes the arrival count.
#pragma unroll
    for (int p = 0; p < kPer; ++p) {
      const int e = tid + p * nthreads;
      const int tile = tile0 + e / (MR * 64);
      if (e < kElems && tile < a.n_tiles)
        __hip_atomic_store(a.partial + ((int64_t)slice * a.n_tiles + tile) * (MR * 64) + e % (MR * 64),
                           __float_as_uint(v[p]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    __syncthreads();
    if (tid == 0) {
      const uint32_t old = __hip_atomic_fetch_add(a.counters + group, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      s_last = (old == (uint32_t)(S - 1));
    }
    __syncthreads();
    if (!s_last) return;
#pragma unroll
    for (int p = 0; p < kPer; ++p) {
      const int e = tid + p * nthreads;
      const int tile = tile0 + e / (MR * 64);
      if (e < kElems && tile < a.n_tiles)
        v[p] = ordered_sum_sc1(a.partial + (int64_t)tile * (MR * 64) + e % (MR * 64), (int64_t)a.n_tiles * (MR * 64), S);
    }
    if (tid == 0) __hip_atomic_store(a.counters + group, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }

  // ---- store: element (t, q, lane) is output row 32*(tile0+t) + lane%32 of token 8*(q/4) + 4*(lane/32) + q%4
#pragma unroll
  for (int p = 0; p < kPer; ++p) {
    const int e = tid + p * nthreads;
    if (e >= kElems) continue;
    const int t = e / (MR * 64), q = (e / 64) % MR, l = e & 63;
    const int token = 8 * (q >> 2) + 4 * (l >> 5) + (q & 3);
    const int64_t n = (int64_t)(tile0 + t) * 32 + (l & 31);
    if (token < a.M && n < a.N) a.y[(int64_t)token * a.ldy + n] = (uint16_t)f32_to_bf16_bits(v[p]);
  }
}

// ---- prepack: canonical (codes [N,K/2], scales [N,K/16]) -> P32 tiles -----------------------------
__global__ __launch_bounds__(256) void prepack_kernel(const uint8_t* __restrict__ codes,
                                                      const uint8_t* __restrict__ scales, int64_t N, int64_t K,
                                                      int64_t n_tiles, int64_t k_tiles, uint8_t* __restrict__ out) {
  const int64_t tile = blockIdx.x;               // nt * k_tiles + kt
  const int64_t nt = tile / k_tiles, kt = tile - nt * k_tiles;
  uint8_t* dst = out + tile * kPackTileBytes;
  // 512 code dwords + 64 scale dwords per tile
  for (int d = threadIdx.x; d < 576; d += 256) {
    uint32_t val = 0;
    if (d < 512) {
      const int plane = d >> 8, lane = (d >> 2) & 63, dw = d & 3;
      const int64_t row = nt * 32 + (lane & 31);
      const int64_t k = kt * 128 + 16 * (4 * plane + dw) + 8 * (lane >> 5);
      if (row < N && k < K) {
        const uint8_t* src = codes + row * (K / 2) + k / 2;
        val = (uint32_t)src[0] | ((uint32_t)src[1] << 8) | ((uint32_t)src[2] << 16) | ((uint32_t)src[3] << 24);
      }
      *reinterpret_cast<uint32_t*>(dst + plane * 1024 + lane * 16 + dw * 4) = val;
    } else {
      const int sd = d - 512;                    // row = sd / 2, half = sd % 2 -> steps 4*half .. +3
      const int64_t row = nt * 32 + (sd >> 1);
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const int64_t blk = kt * 8 + 4 * (sd & 1) + b;
        if (row < N && blk < K / 16) val |= (uint32_t)scales[row * (K / 16) + blk] << (8 * b);
      }
      *reinterpret_cast<uint32_t*>(dst + 2048 + sd * 4) = val;
    }
  }
}

// ---- host ------------------------------------------------------------------------------------------

static int g_force_kw = 0, g_force_t = 0;

DecodePlan plan_decode(int64_t M, int64_t N, int64_t K, int64_t r) {
  DecodePlan p;
  p.k_tiles = ceil_div(K, kPackTileK);
  p.n_tiles = (int)ceil_div(N, kPackTileRows);
  p.MR = M <= 8 ? 4 : 8;
  p.KW = p.k_tiles >= 8 ? 2 : 1;
  if (g_force_kw) p.KW = g_force_kw;
  const int max_main = r > 0 ? kDecMaxWaves - 1 : kDecMaxWaves;
  const int64_t slices = ceil_div(p.k_tiles, p.KW);
  p.S = (int)ceil_div(slices, max_main);
  p.main_waves = (int)ceil_div(slices, p.S);
  p.waves = p.main_waves + (r > 0 ? 1 : 0);
  int T = 1;
  const int tmax = p.MR == 8 ? 2 : 4;
  for (int c = 2; c <= tmax; c *= 2)
    if (ceil_div(p.n_tiles, c) * p.S >= 240) T = c;
  if (g_force_t) T = g_force_t > tmax ? tmax : g_force_t;
  p.T = T;
  p.groups = (int)ceil_div(p.n_tiles, p.T);
  return p;
}

template <int KW, int T, int MR>
static void launch_dec(const DecodePlan& p, const DecodeArgs& a, hipStream_t st) {
  decode32_kernel<KW, T, MR><<<dim3(a.n_producers + p.groups * p.S), dim3(p.waves * 64), 0, st>>>(a);
}

int launch_decode(const DecodePlan& p, const DecodeArgs& a, hipStream_t st) {
  // every pointer the kernel dereferences must be set by the caller
  if (!a.x || !a.packed || !a.tensor_scale || !a.y || !a.partial || !a.counters || (a.r > 0 && (!a.t || !a.B)))
    return QERL_ERR_NULL;
  if (a.n_producers > 0 && (!a.A || !a.lora_ctl || !a.tpart || a.r < 1 || a.r > 64 || a.n_producers > 16))
    return QERL_ERR_NULL;
  if (a.M < 1 || a.M > 16 || a.N < 1 || a.K < 16 || p.waves < 1 || p.waves > kDecMaxWaves || a.S != p.S ||
      a.n_groups != p.groups)
    return QERL_ERR_SHAPE;
#define QERL_CASE(kw, t, mr)                                   \
  if (p.KW == kw && p.T == t && p.MR == mr) {                  \
    launch_dec<kw, t, mr>(p, a, st);                           \
    return launch_status();                                    \
  }
  QERL_CASE(1, 1, 4) QERL_CASE(1, 2, 4) QERL_CASE(1, 4, 4) QERL_CASE(1, 1, 8) QERL_CASE(1, 2, 8)
  QERL_CASE(2, 1, 4) QERL_CASE(2, 2, 4) QERL_CASE(2, 4, 4) QERL_CASE(2, 1, 8) QERL_CASE(2, 2, 8)
#undef QERL_CASE
  return QERL_ERR_SHAPE;
}

int launch_prepack(const uint8_t* codes, const uint8_t* scales, int64_t N, int64_t K, uint8_t* out,
                   hipStream_t st) {
  const int64_t n_tiles = ceil_div(N, kPackTileRows), k_tiles = ceil_div(K, kPackTileK);
  prepack_kernel<<<(unsigned)(n_tiles * k_tiles), 256, 0, st>>>(codes, scales, N, K, n_tiles, k_tiles, out);
  return launch_status();
}

}  // namespace qerl

// Tuning hook for experiments (not part of the public header): force K-tiles per
// wave (1, 2) and row-tiles per workgroup (1, 2, 4); 0 = automatic.
#ifdef QERL_TUNING_HOOKS   // built only for tuning sessions: they change process-wide state
extern "C" QERL_API void qerl_debug_force_decode(int kw, int t) {
  qerl::g_force_kw = kw;
  qerl::g_force_t = t;
}
#endif  // QERL_TUNING_HOOKS
