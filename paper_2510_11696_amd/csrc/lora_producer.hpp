// LoRA down-projection inside a decode launch (Eq. 2's inner factor): producer workgroups at the front of the
// grid compute t[tok][j] = sum_k x[tok,k] * Astack[j,k] for the stacked A of all members of the launch, each
// over its own run of K, and leave their partial sums in memory; the consumers add the partials in producer
// order once an arrival counter says they are all there.
//
// Producer p of P owns a run of 16-input steps of K.  Its share of x and of up to 64 stacked rows of A is first
// copied to LDS with row-contiguous loads (a wave instruction reads 1 KiB of ONE row: few pages and full cache
// lines per request, which matters because these requests queue behind the weight streams of all other
// workgroups), everything requested before anything is stored; then the waves take MFMA operands from LDS,
// steps interleaved over the waves.
//
// MODE 0: x is used as it is.  MODE 1: the input is SiLU(x) (.) x2 (the gated activation of the feed-forward
// block), formed in LDS.  MODE 2: the input is the AQN RMSNorm of x (Eq. 10): rows scaled by rstd[tok] and by
// gain + noise, rounded to bf16 in LDS exactly as the consumers round their slice.
#pragma once
#include "common.hpp"

namespace qerl {

constexpr int kProdMaxSteps = 96;          // steps per column block: 3 chunks of 16 bytes per lane and row
constexpr int kTpartTokens = 16;           // token rows per producer in the partial-t area
constexpr int kProdMaxGroup = 4;

struct LoraProducerArgs {
  const uint16_t* x; int64_t ldx; const uint16_t* x2; int64_t ldx2;
  int M; int64_t K; int r_total; int n_members;
  const uint16_t* A[kProdMaxGroup]; int t_off[kProdMaxGroup];   // stacked rows [t_off[i], ...) are member i's (INT_MAX: not stacked)
  int index;                                   // this producer's number along K
  int only_pair;                               // >= 0: this producer computes stacked rows [64 * only_pair, 64 * only_pair + 64) only (others have the other rows); -1: all rows
  int n_arrivals;                              // arrivals that complete t (publishing producers only): the last one adds the partials
  int n_k;                                     // producers along K (partials per element)
  float* tfinal; uint32_t* ready;              // not null: the last producer to arrive adds the partials in producer order, stores t[tok][r_total] here and sets *ready
  int prod_steps, prod_cb, prod_red_off;       // 16-input steps of K per producer, steps per LDS column block, byte offset of the reduction area
  uint32_t* tpart;                             // [producer][kTpartTokens][r_total] fp32 bit patterns
  uint32_t* arrive;                            // counter the consumers watch
  const uint16_t* gain; const float* noise; const float* rstd;   // MODE 2: gain [K], noise [K] or null, rstd[tok] (LDS or memory)
};

// LDS needed by a producer: rows x (cb * 32 + 16) bytes, rounded up to 256, then WAVES x 2 x MR x 64 floats.
inline size_t lora_producer_red_bytes(int waves, int MR) { return (size_t)waves * 2 * MR * 64 * sizeof(float); }

template <int MR, int MODE, int WAVES>
__device__ __forceinline__ void lora_producer(const LoraProducerArgs& a, unsigned char* smem) {
  constexpr int kRowsPerWave = (64 + 16 + WAVES - 1) / WAVES;   // 64 rows of A + 16 tokens over the waves
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps everything derived from it in SGPRs
  const int n32 = lane & 31, kg = lane >> 5;
  const int n_at = (a.r_total + 31) >> 5, n_pairs = (n_at + 1) >> 1;
  constexpr int kElems = 2 * MR * 64;
  const int steps = (int)(a.K / 16);
  const int p_s0 = a.index * a.prod_steps;
  const int p_s1 = p_s0 + a.prod_steps < steps ? p_s0 + a.prod_steps : steps;
  float* red = reinterpret_cast<float*>(smem + a.prod_red_off);
  for (int pair = a.only_pair >= 0 ? a.only_pair : 0; pair < (a.only_pair >= 0 ? a.only_pair + 1 : n_pairs); ++pair) {
    f32x16 pacc[2];
#pragma unroll
    for (int at = 0; at < 2; ++at)
#pragma unroll
      for (int i = 0; i < 16; ++i) pacc[at][i] = 0.f;
    const int rows_a = a.r_total - 64 * pair < 64 ? a.r_total - 64 * pair : 64;   // stacked rows of this pass
    const int n_rows = rows_a + a.M;                                              // LDS rows: A rows, then tokens, then a zero row
    for (int cb0 = p_s0; cb0 < p_s1; cb0 += a.prod_cb) {
      const int nsb = cb0 + a.prod_cb < p_s1 ? a.prod_cb : p_s1 - cb0;            // steps of this column block
      const int row_chunks = 2 * nsb, stride = row_chunks * 16 + 16;              // bytes between LDS rows
      // wave w copies rows w, w + WAVES, ...; lane l the chunks l, l + 64, l + 128
      u32x4 v[kRowsPerWave][3];
#pragma unroll
      for (int ri = 0; ri < kRowsPerWave; ++ri) {
        const int row = wave + WAVES * ri;
        const uint16_t* src = nullptr;
        if (row < rows_a) {
          const int srow = 64 * pair + row;               // row of the stacked A: lives in member mi at srow - t_off
          int mi = 0;
#pragma unroll
          for (int i = 1; i < kProdMaxGroup; ++i)
            if (i < a.n_members && srow >= a.t_off[i]) mi = i;
          const uint16_t* Am = a.A[0];
          int toff = a.t_off[0];
#pragma unroll
          for (int i = 1; i < kProdMaxGroup; ++i)
            if (mi == i) { Am = a.A[i]; toff = a.t_off[i]; }
          src = Am + (int64_t)(srow - toff) * a.K;
        } else if (row < n_rows) {
          src = a.x + (int64_t)(row - rows_a) * a.ldx;
        }
#pragma unroll
        for (int ci = 0; ci < 3; ++ci) {
          const int c = lane + 64 * ci;
          v[ri][ci] = u32x4{0u, 0u, 0u, 0u};
          if (src && c < row_chunks) v[ri][ci] = *reinterpret_cast<const u32x4*>(src + (int64_t)cb0 * 16 + c * 8);
        }
      }
#pragma unroll
      for (int ri = 0; ri < kRowsPerWave; ++ri) {
        const int row = wave + WAVES * ri;
#pragma unroll
        for (int ci = 0; ci < 3; ++ci) {
          const int c = lane + 64 * ci;
          if (row < n_rows && c < row_chunks) *reinterpret_cast<u32x4*>(smem + row * stride + c * 16) = v[ri][ci];
        }
      }
      for (int c = tid; c < row_chunks; c += WAVES * 64)   // MFMA rows beyond the tokens / the stacked ranks read zeros
        *reinterpret_cast<u32x4*>(smem + n_rows * stride + c * 16) = u32x4{0u, 0u, 0u, 0u};
      if constexpr (MODE == 1) {         // gated input: the token rows in LDS become SiLU(x) (.) x2
        __syncthreads();
        for (int idx = tid; idx < a.M * row_chunks; idx += WAVES * 64) {
          const int row = idx / row_chunks, c = idx - row * row_chunks;
          u32x4* p = reinterpret_cast<u32x4*>(smem + (rows_a + row) * stride + c * 16);
          const u32x4 u = *reinterpret_cast<const u32x4*>(a.x2 + (int64_t)row * a.ldx2 + (int64_t)cb0 * 16 + c * 8);
          *p = silu_mul8(*p, u);
        }
      }
      if constexpr (MODE == 2) {         // normalised input: the token rows in LDS become (gain + noise) (.) x * rstd
        __syncthreads();
        for (int idx = tid; idx < a.M * row_chunks; idx += WAVES * 64) {
          const int row = idx / row_chunks, c = idx - row * row_chunks;
          u32x4* p = reinterpret_cast<u32x4*>(smem + (rows_a + row) * stride + c * 16);
          *p = norm_scale8(*p, a.rstd[row], a.gain, a.noise, (int64_t)cb0 * 16 + c * 8);
        }
      }
      __syncthreads();
      const unsigned char* xrow = smem + (rows_a + (n32 < a.M ? n32 : a.M)) * stride + kg * 16;
      const unsigned char* arow0 = smem + (n32 < rows_a ? n32 : n_rows) * stride + kg * 16;
      const unsigned char* arow1 = smem + (32 + n32 < rows_a ? 32 + n32 : n_rows) * stride + kg * 16;
      for (int sidx = wave; sidx < nsb; sidx += WAVES) {
        const bf16x8 xf = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(xrow + sidx * 32));
        const bf16x8 a0 = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(arow0 + sidx * 32));
        const bf16x8 a1 = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(arow1 + sidx * 32));
        pacc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf, a0, pacc[0], 0, 0, 0);
        pacc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf, a1, pacc[1], 0, 0, 0);
      }
      __syncthreads();   // all fragments read before the next block (or the sums below) overwrite them
    }
#pragma unroll
    for (int at = 0; at < 2; ++at)
#pragma unroll
      for (int q = 0; q < MR; ++q) red[(wave * 2 + at) * MR * 64 + q * 64 + lane] = pacc[at][q];
    __syncthreads();
    // this workgroup's partial of t, in [token][stacked rank] order (what the consumers' MFMA operand wants)
    for (int e = tid; e < kElems; e += WAVES * 64) {
      float sum = red[e];
      for (int w = 1; w < WAVES; ++w) sum += red[w * kElems + e];
      const int at = e / (MR * 64), q = (e / 64) % MR, l = e & 63;
      const int tok = 8 * (q >> 2) + 4 * (l >> 5) + (q & 3), j = (2 * pair + at) * 32 + (l & 31);
      if (tok < a.M && j < a.r_total)
        __hip_atomic_store(a.tpart + ((int64_t)a.index * kTpartTokens + tok) * a.r_total + j, __float_as_uint(sum),
                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();   // red is reused by the next pair
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's partial stores have completed
  __syncthreads();
  if (!a.tfinal) {
    // Consumers wait for all P arrivals and add the P partials themselves, in producer order: one
    // memory round trip less than electing a producer to publish the sum.
    if (tid == 0) __hip_atomic_fetch_add(a.arrive, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return;
  }
  // Publishing variant: the producer that arrives last adds the partials of all producers in producer order and
  // stores the finished t, so that every consumer workgroup fetches M x r_total floats in one round of loads
  // instead of adding P partials itself (P dependent rounds of loads on the critical path of its first tile).
  uint32_t* flag = reinterpret_cast<uint32_t*>(red);
  if (tid == 0) *flag = __hip_atomic_fetch_add(a.arrive, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __syncthreads();
  if (*flag != (uint32_t)(a.n_arrivals - 1)) return;
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
  const int n4 = a.M * (a.r_total >> 2);                 // groups of four ranks
  for (int e = tid; e < n4; e += WAVES * 64) {
    const int tok = e / (a.r_total >> 2), j4 = e - tok * (a.r_total >> 2);
    f32x4 sum = {0.f, 0.f, 0.f, 0.f};
    for (int p0 = 0; p0 < a.n_k; p0 += 32) {   // all partials of the element in flight together: one round of loads
      f32x4 tq[32];
#pragma unroll
      for (int b = 0; b < 32; ++b) {
        tq[b] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (p0 + b < a.n_k)
          tq[b] = *reinterpret_cast<const f32x4*>(reinterpret_cast<const float*>(a.tpart) + ((int64_t)(p0 + b) * kTpartTokens + tok) * a.r_total + 4 * j4);
      }
#pragma unroll
      for (int b = 0; b < 32; ++b) sum += tq[b];
    }
    uint64_t* dst = reinterpret_cast<uint64_t*>(a.tfinal + (int64_t)tok * a.r_total + 4 * j4);
    __hip_atomic_store(dst, (uint64_t)__float_as_uint(sum[0]) | ((uint64_t)__float_as_uint(sum[1]) << 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(dst + 1, (uint64_t)__float_as_uint(sum[2]) | ((uint64_t)__float_as_uint(sum[3]) << 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's share of t is in memory
  __syncthreads();
  if (tid == 0) __hip_atomic_store(a.ready, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

}  // namespace qerl
