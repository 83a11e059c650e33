// LoRA down-projection for 17 tokens and more: ts = three bf16 terms of (lora_scale / S32) * x A^T   (Eq. 2, first factor)
// as a block-level routine, so that it can run as a kernel of its own (prefill) or as the leading workgroups of
// the 17..128-token kernel's launch.
#pragma once
#include "linear.hpp"

namespace qerl {

constexpr int kDownMaxParts = 8;   // K-parts of the LoRA down-projection when there are few token blocks: summed eight at a time
constexpr int kDownMaxPartsWide = 32;   // ... when it is a launch of its own and would otherwise leave most of the chip idle

// One workgroup of WAVES waves: token block bx (32 tokens), rank tile(s) by, K-part bz of P; gx, gy: numbers of token
// blocks and tile columns.  red: kLoraDownLdsBytes(NT, WAVES) of LDS.  With a.ready set, the workgroup that writes
// ts makes it visible to the whole device and counts itself there.
// The waves take the 64-column slabs of the K-part in turn.  A slab of x (32 tokens x 128 bytes) and of each rank
// tile is fetched row-contiguously -- eight lanes per 128-byte row segment, two slabs ahead in registers -- and
// reaches the MFMA operand layout (one row per lane) through a wave-private LDS area (row-XOR swizzle as in the
// GEMM's x slab; no barrier: a wave's LDS operations complete in order).  Fetching in operand layout instead, 16
// bytes of 64 different rows per instruction, is served at an eighth of the rate.
constexpr size_t kLoraDownLdsBytes(int NT, int WAVES) { return (size_t)WAVES * (1 + NT) * 4096; }
template <int NT, int WAVES>
__device__ __forceinline__ void lora_down_block(const GemmArgs& a, int bx, int by, int bz, int P, int gx, int gy, float* red) {
  constexpr int kWaves = WAVES;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps everything derived from it in SGPRs
  const int n32 = lane & 31, kg = lane >> 5;
  const int64_t m0 = (int64_t)bx * 32;
  // one adapter, or (NT == 1) the adapter that owns tile `by` of the group
  int nt0 = by * NT;
  const uint16_t* Aw = a.wbf16;
  uint16_t* ts = const_cast<uint16_t*>(a.ts);
  int64_t ts_ld = a.ts_ld, rN = a.N;
  float lora_scale = a.lora_scale;
  const float* tensor_scale = a.tensor_scale;
  bool first_tile = by == 0;
  if (a.g_n > 0) {
    int mi = 0;
#pragma unroll
    for (int i = 1; i < kMaxGroup; ++i) mi = (i < a.g_n && by >= a.g_tile0[i]) ? i : mi;
#pragma unroll
    for (int i = 0; i < kMaxGroup; ++i)
      if (mi == i) {
        Aw = a.g_A[i]; ts = const_cast<uint16_t*>(a.g_ts[i]); ts_ld = a.g_ts_ld[i]; rN = a.g_r[i];
        lora_scale = a.g_lora_scale[i]; tensor_scale = a.g_tensor_scale[i];
        nt0 = by - a.g_tile0[i];
      }
    first_tile = nt0 == 0;
  }

  // K-part of this workgroup (P parts, whole 64-column chunks each)
  const int64_t part_cols = ceil_div_dev(ceil_div_dev(a.K, 64), P) * 64;
  const int64_t k_lo = (int64_t)bz * part_cols;
  const int64_t k_hi = k_lo + part_cols < a.K ? k_lo + part_cols : a.K;

  struct Chunk { u32x4 x[4]; u32x4 w[NT][4]; };   // 64 columns = 4 MFMA steps: as requested (instruction i: row 8 i + lane / 8,
                                                   // 16-byte segment lane % 8) or as operands (step j: row lane % 32, columns 16 j + 8 (lane / 32))
  const int seg = lane & 7, rr = lane >> 3;
  const uint16_t* xsrc[4];
  const uint16_t* asrc[NT][4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int64_t m = m0 + 8 * i + rr;
    m = m < a.M ? m : a.M - 1;
    xsrc[i] = a.x + m * a.ldx + 8 * seg;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      int64_t row = (int64_t)(nt0 + nt) * 32 + 8 * i + rr;
      row = row < rN ? row : rN - 1;
      asrc[nt][i] = Aw + row * a.K + 8 * seg;
    }
  }
  auto request = [&](Chunk& c, int64_t kb) {       // past the part's end: zeros, no access
    const bool in = kb + 8 * seg < k_hi;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      c.x[i] = u32x4{0u, 0u, 0u, 0u};
      if (in) c.x[i] = *reinterpret_cast<const u32x4*>(xsrc[i] + kb);
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        c.w[nt][i] = u32x4{0u, 0u, 0u, 0u};
        if (in) c.w[nt][i] = *reinterpret_cast<const u32x4*>(asrc[nt][i] + kb);
      }
    }
  };
  u32x4* stage = reinterpret_cast<u32x4*>(red) + wave * (1 + NT) * 256;   // this wave's slabs: 256 chunks of 16 bytes each
  auto to_operands = [&](Chunk& c) {               // in place: the requested slab becomes the MFMA fragments
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = 8 * i + rr, at = row * 8 + (seg ^ ((row >> 1) & 7));
      stage[at] = c.x[i];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) stage[(1 + nt) * 256 + at] = c.w[nt][i];
    }
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int at = n32 * 8 + ((2 * j + kg) ^ ((n32 >> 1) & 7));
      c.x[j] = stage[at];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) c.w[nt][j] = stage[(1 + nt) * 256 + at];
    }
    __builtin_amdgcn_wave_barrier();
  };
  f32x16 acc[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[nt][i] = 0.f;
  auto mma = [&](const Chunk& c) {
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, c.x[j]),
                                                          __builtin_bit_cast(bf16x8, c.w[nt][j]), acc[nt], 0, 0, 0);
  };
  Chunk c0, c1;
  const int64_t step = (int64_t)kWaves * 64;
  int64_t kb = k_lo + (int64_t)wave * 64;
  if (kb < k_hi) {
    request(c0, kb);
    request(c1, kb + step);
  }
  while (kb < k_hi) {
    Chunk f = c0;
    request(c0, kb + 2 * step);
    to_operands(f);
    mma(f);
    if (kb + step >= k_hi) break;
    f = c1;
    request(c1, kb + 3 * step);
    to_operands(f);
    mma(f);
    kb += 2 * step;
  }
  __syncthreads();   // the staging areas become the reduction's

  if (wave > 0) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int i = 0; i < 16; ++i) red[((wave - 1) * NT * 16 + nt * 16 + i) * 64 + lane] = acc[nt][i];
  }
  __syncthreads();
  if (wave != 0) return;
#pragma unroll
  for (int nt = 0; nt < NT; ++nt)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
#pragma unroll
      for (int w = 0; w < kWaves - 1; ++w) acc[nt][i] += red[(w * NT * 16 + nt * 16 + i) * 64 + lane];
    }
  if (P > 1) {
    // Several K-parts: every part leaves its sums in the workspace (written through to memory before its
    // arrival is counted); the workgroup that arrives last adds all parts in part order and goes on.
    const int slot = bx * gy + by;
    const int64_t part_stride = (int64_t)gx * gy * (NT * 16 * 64);
    uint32_t* mine = a.tpart + (int64_t)bz * part_stride + (int64_t)slot * (NT * 16 * 64) + lane;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int i = 0; i < 16; ++i)
        __hip_atomic_store(mine + (nt * 16 + i) * 64, __float_as_uint(acc[nt][i]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    uint32_t old = 0;
    if (lane == 0) old = __hip_atomic_fetch_add(a.counters + slot, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    old = __builtin_amdgcn_readfirstlane(old);
    if (old != (uint32_t)(P - 1)) return;
    const uint32_t* all = a.tpart + (int64_t)slot * (NT * 16 * 64) + lane;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[nt][i] = 0.f;
      for (int z0 = 0; z0 < P; z0 += kDownMaxParts) {   // in part order, eight parts requested together
        uint32_t v[kDownMaxParts][16];
#pragma unroll
        for (int z = 0; z < kDownMaxParts; ++z)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            v[z][i] = 0u;
            if (z0 + z < P) v[z][i] = __hip_atomic_load(all + (int64_t)(z0 + z) * part_stride + (nt * 16 + i) * 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          }
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          float sum = acc[nt][i];
#pragma unroll
          for (int z = 0; z < kDownMaxParts; ++z) sum += __uint_as_float(v[z][i]);
          acc[nt][i] = sum;
        }
      }
    }
    if (lane == 0) __hip_atomic_store(a.counters + slot, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next call
  }
  const float t_mult = lora_scale / *tensor_scale;   // undone by the final * S32 of the main launch
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int64_t n = (int64_t)(nt0 + nt) * 32 + n32;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const float sum = acc[nt][i];
      const int64_t m = m0 + 8 * (i >> 2) + 4 * kg + (i & 3);
      if (m < a.M && n < rN) {
        const float v = sum * t_mult;
        const uint32_t h = f32_to_bf16_bits(v);
        const float r1 = v - bf16_bits_to_f32(h);
        const uint32_t md = f32_to_bf16_bits(r1);
        const uint32_t l = f32_to_bf16_bits(r1 - bf16_bits_to_f32(md));
        uint16_t* row = ts + m * ts_ld;
        row[n] = (uint16_t)h;
        row[rN + n] = (uint16_t)md;
        row[2 * rN + n] = (uint16_t)l;
      }
    }
  }
  if (first_tile) {   // zero the padding columns [3 r, ts_ld)
    const int pad = (int)(ts_ld - 3 * rN);
    for (int idx = lane; idx < 32 * pad; idx += 64) {
      const int64_t m = m0 + idx / pad;
      if (m < a.M) ts[m * ts_ld + 3 * rN + idx % pad] = 0;
    }
  }
  if (a.ready) {   // consumers in the same launch wait for this count
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    if (lane == 0) __hip_atomic_fetch_add(a.ready, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}


}  // namespace qerl
