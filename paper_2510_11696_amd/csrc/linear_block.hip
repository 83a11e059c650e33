// Persistent block kernel for decode (M <= 16 tokens): up to three dependent stages of NVFP4 + LoRA linears in ONE
// launch, each stage one linear or a group of linears that share their input,
//
//   y_g[m,n] = S32_g * sum_b s_g[n,b] * ( sum_{k in block b} x[m,k] * e_g[n,k] )           (Eq. 6)
//            + lora_scale_g * sum_j t_g[m,j] * B_g[n,j] (+ bias_g[n]),    t_g = x A_g^T     (Eq. 2)
//
// with, optionally, the AQN RMSNorm (Eq. 10) applied to the stage's input while it is staged, and -- for a
// gate_proj / up_proj pair -- SiLU(gate) (.) up formed in the epilogue, so that the next stage (down_proj)
// reads the gated activation.  Launches it replaces: norm + LoRA-down, group, (reduce), SiLU-mul, linear, (reduce).
//
// Why one launch: the weights do not depend on the activations.  A launch per linear pays start-up, ring fill,
// drain and the spread of its workgroups (about 10 us) each time; here the weight stream never stops -- while a
// wave waits at a stage boundary for the other workgroups' outputs, the first tiles of its next unit are already
// on their way.
//
// Structure:
//   * One workgroup of 16 waves per CU.  A unit of work is one row tile (32 output rows) over one K-range of a
//     stage; a wave owns its units outright: it streams the unit's packed tiles through a ring of kBlkD tiles in
//     registers (refilled in place, across unit and stage boundaries), multiplies them -- bare E2M1 values into one
//     v_mfma_f32_32x32x16_bf16 per 16-input scale block, then acc += E4M3 scale * product, as in
//     linear_stream.hip -- and finishes the unit itself: tensor scale, LoRA up-projection (B rows requested one
//     ring round ahead), bias, store.  No wave ever hands anything to another wave of its workgroup, so there is
//     no per-unit synchronisation at all, and 16 independent streams per CU keep ~150 KB in flight.
//   * The K-range's slice of the stage input lives in LDS for the whole stage, shared by the 16 waves (rows
//     16 bytes apart in bank space; MFMA rows beyond the tokens read a zero row).  When the slice of all of K
//     does not fit (or the linear has too few row tiles to occupy the chip), K is split over ranges of
//     workgroups: every range leaves fp32 partial tiles in the workspace, counts itself in the tile's arrival
//     word, and the wave that arrives last adds the partials in range order and stores -- fixed order, so
//     results do not depend on timing.
//   * t = x A^T of a stage comes from producer workgroups at the front of the grid (lora_producer.hpp); the first
//     wave of a workgroup that needs a member's t adds the producers' partials in producer order and leaves them
//     in LDS as three bf16 terms (exact to 2^-24 relative) for the other waves.
//   * Stage boundary: every workgroup releases its outputs (agent-scope release, counter), waits until all have
//     (bounded spin), acquires, stages the next input.
// Every wait on another workgroup is bounded; a wait that gives up sets the sticky error word of the workspace
// (qerl_workspace_status), poisons nothing silently, and the control words are then left as they are.
#include <stdio.h>
#include <stdlib.h>
#include "linear.hpp"
#include "lora_producer.hpp"

namespace qerl {

constexpr int kBlkThreads = kBlkWaves * 64;
constexpr int kBlkD = 4;                        // ring depth in tiles; every K-range length is a multiple of it
constexpr uint32_t kBlkSpinLimit = 1u << 17;    // polls of a bounded wait (x s_sleep: tens of milliseconds)

struct BlkTile { u32x4 c0, c1; u32x2 sc; };

__device__ __forceinline__ bf16x8 blk_e2m1x8(uint32_t codes) {
  const bf16x2 p0 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(codes, 1.0f, 0);
  const bf16x2 p1 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(codes, 1.0f, 1);
  const bf16x2 p2 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(codes, 1.0f, 2);
  const bf16x2 p3 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(codes, 1.0f, 3);
  u32x4 o = {__builtin_bit_cast(uint32_t, p0), __builtin_bit_cast(uint32_t, p1),
             __builtin_bit_cast(uint32_t, p2), __builtin_bit_cast(uint32_t, p3)};
  return __builtin_bit_cast(bf16x8, o);
}

__device__ __forceinline__ void blk_issue(BlkTile& t, const uint8_t* base, int lane, int n32) {
  t.c0 = *reinterpret_cast<const u32x4*>(base + lane * 16);
  t.c1 = *reinterpret_cast<const u32x4*>(base + 1024 + lane * 16);
  t.sc = *reinterpret_cast<const u32x2*>(base + 2048 + n32 * 8);
}

// One packed tile (32 rows x 128 inputs = 8 scale blocks) times the x fragments at xk.
template <int MR>
__device__ __forceinline__ void blk_consume(const BlkTile& t, const unsigned char* xk, float (&acc)[MR]) {
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  f32x16 tmp[2];
  tmp[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(xk)),
                                                   blk_e2m1x8(t.c0[0]), zero, 0, 0, 0);
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    if (j + 1 < 8) {   // the product of the next scale block is on its way while this one is scaled and added
      const bf16x8 xa = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(xk + (j + 1) * 32));
      const bf16x8 w = blk_e2m1x8(j + 1 < 4 ? t.c0[(j + 1) & 3] : t.c1[(j + 1) & 3]);
      tmp[(j + 1) & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa, w, zero, 0, 0, 0);
    }
    const float s = e4m3_byte_f32(t.sc[j >> 2], j & 3);
#pragma unroll
    for (int q = 0; q < MR; ++q) acc[q] = __builtin_fmaf(s, tmp[j & 1][q], acc[q]);
  }
}

// Bounded wait until *word >= target (agent scope).  Returns false when it gave up.
__device__ __forceinline__ bool blk_wait_ge(const uint32_t* word, uint32_t target, int sleep) {
  for (uint32_t spins = 0; spins < kBlkSpinLimit; ++spins) {
    if (__hip_atomic_load(word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= target) return true;
    if (sleep > 8) __builtin_amdgcn_s_sleep(32); else __builtin_amdgcn_s_sleep(2);
  }
  return false;
}

template <int MR>
__global__ __launch_bounds__(kBlkThreads) void block_kernel(const BlkArgs a) {
  // dynamic LDS: x slice [M + 1 rows][xs_stride], then the split t of up to four members, then one output tile
  // per wave.  256-byte alignment matters: 16-byte LDS accesses from a misaligned base run several times slower.
  extern __shared__ __attribute__((aligned(256))) unsigned char smem[];
  __shared__ float s_ss[kBlkWaves][16];
  __shared__ float s_rstd[16];
  __shared__ uint32_t s_tstate[kMaxGroup];   // per member: 0 t not loaded, 1 being loaded, 2 in LDS, 3 in LDS but the producers never arrived
  constexpr int MT = MR == 4 ? 8 : 16;
  constexpr int D = kBlkD;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n32 = lane & 31, kg = lane >> 5;
  const int wg = (int)blockIdx.x;
  const bool prod_wg = wg < a.n_prod_max;
  const int cons = wg - a.n_prod_max;         // consumer workgroup index
  uint32_t* const err_word = a.ctl + kCtlErr;
  unsigned char* const tarea = smem + a.t_lds_off;
  uint16_t* const ytile = reinterpret_cast<uint16_t*>(smem + a.y_lds_off) + wave * (16 * 32);

  // ---- stage boundary: everybody's outputs of the previous stage are complete and visible ----------------------
  auto stage_boundary = [&](int s) {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    __syncthreads();
    if (tid == 0) {
      __hip_atomic_fetch_add(a.ctl + kBlkBarrier, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (!blk_wait_ge(a.ctl + kBlkBarrier, (uint32_t)(a.n_wgs * s), 1))
        __hip_atomic_fetch_or(err_word, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
  };
  // ---- exit: the last workgroup to leave re-arms the control words, unless a wait gave up somewhere -------------
  auto leave = [&]() {
    __syncthreads();
    if (tid == 0) {
      const uint32_t old = __hip_atomic_fetch_add(a.ctl + kBlkExit, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (old == (uint32_t)(a.n_wgs - 1) &&
          __hip_atomic_load(err_word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u) {
        for (int s = 0; s < kBlkMaxStages; ++s)
          __hip_atomic_store(a.ctl + kBlkArrive + s, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(a.ctl + kBlkBarrier, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(a.ctl + kBlkExit, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
  };
  auto sumsq = [](const u32x4& v) {
    float r = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float lo = bf16_bits_to_f32(v[i] & 0xffffu), hi = bf16_bits_to_f32(v[i] >> 16);
      r = __builtin_fmaf(lo, lo, r);
      r = __builtin_fmaf(hi, hi, r);
    }
    return r;
  };

  // ---- producer workgroups: per stage, the LoRA down-projection of its input (normalised first, if the stage
  // normalises); they take no units, so none of the streaming state below exists on this path
  if (prod_wg) {
    for (int s = 0; s < a.n_stages; ++s) {
      const BlkStage& S = a.st[s];
      if (s > 0) stage_boundary(s);
      if (wg >= S.n_producers) continue;
      const bool norm = S.gain != nullptr;
      if (norm) {                      // row statistics over all of K
        const int chunks_row = (int)(S.K / 8);
        float ss[MT];
#pragma unroll
        for (int t = 0; t < MT; ++t) ss[t] = 0.f;
        for (int ch = tid; ch < chunks_row; ch += kBlkThreads) {
#pragma unroll
          for (int t = 0; t < MT; ++t)
            if (t < a.M) ss[t] += sumsq(*reinterpret_cast<const u32x4*>(S.x + (int64_t)t * S.ldx + (int64_t)ch * 8));
        }
#pragma unroll
        for (int t = 0; t < MT; ++t) {
          const float w = wave_sum(ss[t]);
          if (lane == 0) s_ss[wave][t] = w;
        }
        __syncthreads();
        if (tid < a.M) {
          float total = 0.f;
#pragma unroll
          for (int w = 0; w < kBlkWaves; ++w) total += s_ss[w][tid];
          s_rstd[tid] = 1.0f / sqrtf(total / (float)S.K + S.eps);
        }
        __syncthreads();
      }
      LoraProducerArgs p;
      p.x = S.x; p.ldx = S.ldx; p.x2 = nullptr; p.ldx2 = 0;
      p.M = a.M; p.K = S.K; p.r_total = S.r_total; p.n_members = S.n_members;
#pragma unroll
      for (int i = 0; i < kMaxGroup; ++i) { p.A[i] = S.mem[i].A; p.t_off[i] = S.mem[i].t_off; }
      p.index = wg;
      p.prod_steps = S.prod_steps; p.prod_cb = S.prod_cb; p.prod_red_off = S.prod_red_off;
      p.tpart = a.tpart + (int64_t)s * kBlkTpartWords; p.arrive = a.ctl + kBlkArrive + s;
      p.gain = S.gain; p.noise = S.noise; p.rstd = s_rstd;
      if (norm) lora_producer<MR, 2, kBlkWaves>(p, smem);
      else lora_producer<MR, 0, kBlkWaves>(p, smem);
    }
    leave();
    return;
  }

  // ---- which units are mine ----------------------------------------------------------------------------------
  struct Geo { int range, slot, slots_r, n_my, kr0, nvalid; };
  auto geo = [&](int s) {
    const BlkStage& S = a.st[s];
    Geo g;
    g.range = cons / S.per_range;
    const int ci = cons - g.range * S.per_range;
    g.slot = ci * kBlkWaves + wave;
    g.slots_r = S.per_range * kBlkWaves;
    g.n_my = (g.range < S.Sk && g.slot < S.total_v) ? (S.total_v - g.slot + g.slots_r - 1) / g.slots_r : 0;
    g.kr0 = g.range * S.kr_len;
    const int left = S.k_tiles - g.kr0;
    g.nvalid = left < S.kr_len ? left : S.kr_len;
    return g;
  };
  struct Pass { int s, j, h; Geo g; };
  // row tile (within the stage's stacked members) of a pass
  auto pass_tile = [&](const Pass& p) {
    const BlkStage& S = a.st[p.s];
    const int v = p.g.slot + p.j * p.g.slots_r;
    return (S.pairs && p.h) ? S.mem[1].tile_begin + v : v;
  };
  auto member_of = [&](const BlkStage& S, int nt) {
    return (nt >= S.mem[1].tile_begin ? 1 : 0) + (nt >= S.mem[2].tile_begin ? 1 : 0) + (nt >= S.mem[3].tile_begin ? 1 : 0);
  };
  auto pass_base = [&](const Pass& p) {
    const BlkStage& S = a.st[p.s];
    const int nt = pass_tile(p);
    int tb = 0;
    const uint8_t* mp = S.mem[0].packed;
    if (nt >= S.mem[1].tile_begin) { tb = S.mem[1].tile_begin; mp = S.mem[1].packed; }
    if (nt >= S.mem[2].tile_begin) { tb = S.mem[2].tile_begin; mp = S.mem[2].packed; }
    if (nt >= S.mem[3].tile_begin) { tb = S.mem[3].tile_begin; mp = S.mem[3].packed; }
    return mp + ((int64_t)(nt - tb) * S.k_tiles + p.g.kr0) * kPackTileBytes;
  };
  auto next_pass = [&](Pass& p) {     // false: there is none
    if (a.st[p.s].pairs && p.h == 0) { p.h = 1; return true; }
    p.h = 0;
    ++p.j;
    while (p.j >= p.g.n_my) {
      ++p.s;
      if (p.s >= a.n_stages) return false;
      p.g = geo(p.s);
      p.j = 0;
    }
    return true;
  };

  Pass cur;
  cur.s = 0; cur.j = -1; cur.h = 0; cur.g = geo(0);
  if (a.st[0].pairs) cur.h = 1;        // so that next_pass() steps to (j = 0, h = 0)
  bool have_cur = next_pass(cur);
  const uint8_t* const park = a.st[0].mem[0].packed;   // where loads go that nobody needs: always valid memory

  // ---- the ring: first D tiles of my first unit, requested before anything else ---------------------------------
  BlkTile ring[D];
  {
    const uint8_t* b0 = have_cur ? pass_base(cur) : park;
    const int nv = have_cur ? cur.g.nvalid : 1;
#pragma unroll
    for (int d = 0; d < D; ++d) blk_issue(ring[d], b0 + (int64_t)(d < nv ? d : nv - 1) * kPackTileBytes, lane, n32);
  }

  float held[MR];                      // gate_proj's finished tile while up_proj's is being computed (pairs, one K-range)
#pragma unroll
  for (int q = 0; q < MR; ++q) held[q] = 0.f;

  for (int s = 0; s < a.n_stages; ++s) {
    const BlkStage& S = a.st[s];
    if (s > 0) stage_boundary(s);
    if (tid < kMaxGroup) s_tstate[tid] = 0u;

    // ---- stage input: this workgroup's K-range slice into LDS (all of K for a producer's row statistics) --------
    const Geo g0 = geo(s);             // range and K-tiles are the same for all waves of the workgroup
    const int xs_stride = S.kr_len * 256 + 16;
    const int chunks_row = (int)(S.K / 8);                 // 16-byte chunks of a row
    const int sl_chunks = S.kr_len * 16;                   // chunks of the slice (K-tiles padded)
    const int sl0 = g0.kr0 * 16;
    const bool stage_slice = g0.range < S.Sk;
    const bool norm = S.gain != nullptr;
    float ss[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) ss[t] = 0.f;
    if (stage_slice) {
      for (int lc = tid; lc < sl_chunks; lc += kBlkThreads) {
        const int ch = sl0 + lc;
#pragma unroll
        for (int t0 = 0; t0 < MT; t0 += 8) {
          u32x4 v[8];
#pragma unroll
          for (int t = 0; t < 8; ++t) {
            v[t] = u32x4{0u, 0u, 0u, 0u};
            if (t0 + t < a.M && ch < chunks_row) v[t] = *reinterpret_cast<const u32x4*>(S.x + (int64_t)(t0 + t) * S.ldx + (int64_t)ch * 8);
          }
#pragma unroll
          for (int t = 0; t < 8; ++t) {
            if (t0 + t < a.M) *reinterpret_cast<u32x4*>(smem + (t0 + t) * xs_stride + lc * 16) = v[t];
            if (norm) ss[t0 + t] += sumsq(v[t]);
          }
        }
        *reinterpret_cast<u32x4*>(smem + a.M * xs_stride + lc * 16) = u32x4{0u, 0u, 0u, 0u};   // the zero row
      }
    }
    if (norm && stage_slice) {
      // the rest of the rows, for the statistics only
      for (int ch = tid; ch < chunks_row; ch += kBlkThreads) {
        if (ch >= sl0 && ch < sl0 + sl_chunks) continue;
#pragma unroll
        for (int t = 0; t < MT; ++t)
          if (t < a.M) ss[t] += sumsq(*reinterpret_cast<const u32x4*>(S.x + (int64_t)t * S.ldx + (int64_t)ch * 8));
      }
#pragma unroll
      for (int t = 0; t < MT; ++t) {
        const float w = wave_sum(ss[t]);
        if (lane == 0) s_ss[wave][t] = w;
      }
    }
    __syncthreads();
    if (norm && tid < a.M) {
      float total = 0.f;
#pragma unroll
      for (int w = 0; w < kBlkWaves; ++w) total += s_ss[w][tid];
      s_rstd[tid] = 1.0f / sqrtf(total / (float)S.K + S.eps);
    }
    __syncthreads();
    if (norm && stage_slice) {
      for (int lc = tid; lc < sl_chunks; lc += kBlkThreads) {
        const int ch = sl0 + lc;
        if (ch < chunks_row) {
          for (int t = 0; t < a.M; ++t) {
            u32x4* p = reinterpret_cast<u32x4*>(smem + t * xs_stride + lc * 16);
            *p = norm_scale8(*p, s_rstd[t], S.gain, S.noise, (int64_t)ch * 8);
          }
        }
      }
    }
    __syncthreads();

    // ---- my units of this stage ----------------------------------------------------------------------------------
    const int xrow = n32 < a.M ? n32 : a.M;
    const unsigned char* const xbase = smem + xrow * xs_stride + kg * 16;
    const bool first_range = g0.range == 0;
    while (have_cur && cur.s == s) {
      const int nt = pass_tile(cur);
      const int mi = member_of(S, nt);
      const BlkMember& mem = S.mem[mi];
      const uint8_t* const base = pass_base(cur);
      const int nvalid = cur.g.nvalid;
      float acc[MR];
#pragma unroll
      for (int q = 0; q < MR; ++q) acc[q] = 0.f;
      int i0 = 0;
      for (; i0 + D < S.kr_len; i0 += D) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
          if (i0 + d < nvalid) blk_consume<MR>(ring[d], xbase + (i0 + d) * 256, acc);
          // the refill stays below the last use of the slot (see linear_stream.hip): same registers, no copies
#pragma unroll
          for (int q = 0; q < MR; ++q) asm volatile("" : "+v"(acc[q]));
          __builtin_amdgcn_sched_barrier(0);
          const int nx = i0 + D + d;
          blk_issue(ring[d], base + (int64_t)(nx < nvalid ? nx : nvalid - 1) * kPackTileBytes, lane, n32);
        }
      }
      // last ring round of the unit: what the epilogue reads from memory is requested now, then the refills go
      // to the next unit (of this or the next stage)
      Pass nxt = cur;
      const bool have_next = next_pass(nxt);
      const uint8_t* const nbase = have_next ? pass_base(nxt) : park;
      const int nnv = have_next ? nxt.g.nvalid : 1;
      const bool lora = first_range && mem.r > 0;
      const int64_t row0 = (int64_t)(nt - mem.tile_begin) * 32;
      u32x4 bfrag[4];
      {
        int64_t brow = row0 + n32;
        brow = brow < mem.N ? brow : mem.N - 1;
#pragma unroll
        for (int st = 0; st < 4; ++st) {
          const int j0 = 16 * st + 8 * kg;
          const bool live = lora && j0 < mem.r;   // (every unit issues the same number of loads: the wait counts stay exact)
          const uint16_t* src = live ? mem.B + brow * mem.r + j0 : reinterpret_cast<const uint16_t*>(park) + lane * 8;
          bfrag[st] = *reinterpret_cast<const u32x4*>(src);
          if (!live) bfrag[st] = u32x4{0u, 0u, 0u, 0u};
        }
      }
      uint16_t bias_bits = 0;
      {
        const uint16_t* src = (first_range && mem.bias && row0 + n32 < mem.N) ? mem.bias + row0 + n32
                                                                            : reinterpret_cast<const uint16_t*>(park);
        bias_bits = *src;
        if (!(first_range && mem.bias && row0 + n32 < mem.N)) bias_bits = 0;
      }
#pragma unroll
      for (int d = 0; d < D; ++d) {
        if (i0 + d < nvalid) blk_consume<MR>(ring[d], xbase + (i0 + d) * 256, acc);
#pragma unroll
        for (int q = 0; q < MR; ++q) asm volatile("" : "+v"(acc[q]));
        __builtin_amdgcn_sched_barrier(0);
        blk_issue(ring[d], nbase + (int64_t)(d < nnv ? d : nnv - 1) * kPackTileBytes, lane, n32);
      }

      // ---- epilogue of the unit ------------------------------------------------------------------------------------
      const float S32 = *mem.tensor_scale;
      float out[MR];
#pragma unroll
      for (int q = 0; q < MR; ++q) out[q] = acc[q] * S32;
      if (lora) {
        // t of this member in LDS as three bf16 terms; the first wave of the workgroup that needs it puts it there
        uint32_t ts = __hip_atomic_load(&s_tstate[mi], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP);
        if (ts < 2u) {
          int won = 0;
          if (lane == 0) {
            uint32_t expect = 0u;
            won = __hip_atomic_compare_exchange_strong(&s_tstate[mi], &expect, 1u, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                                       __HIP_MEMORY_SCOPE_WORKGROUP) ? 1 : 0;
          }
          won = __builtin_amdgcn_readfirstlane(won);
          if (won) {
            const bool arrived = blk_wait_ge(a.ctl + kBlkArrive + s, (uint32_t)S.n_producers, 32);
            if (!arrived && lane == 0) __hip_atomic_fetch_or(err_word, 2u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
            const int r4 = mem.r >> 2, n4 = a.M * r4;
            const float* src = reinterpret_cast<const float*>(a.tpart + (int64_t)s * kBlkTpartWords) + mem.t_off;
            uint16_t* th = reinterpret_cast<uint16_t*>(tarea) + (mi * 3) * MT * 64;
            for (int e0 = 0; e0 < n4; e0 += 64) {
              const int e = e0 + lane, tok = e / r4, j4 = e - tok * r4;
              f32x4 sum = {0.f, 0.f, 0.f, 0.f};
              for (int p0 = 0; p0 < S.n_producers; p0 += 8) {
                f32x4 tq[8];
#pragma unroll
                for (int b = 0; b < 8; ++b) {
                  tq[b] = f32x4{0.f, 0.f, 0.f, 0.f};
                  if (e < n4 && p0 + b < S.n_producers)
                    tq[b] = *reinterpret_cast<const f32x4*>(src + ((int64_t)(p0 + b) * kTpartTokens + tok) * S.r_total + 4 * j4);
                }
#pragma unroll
                for (int b = 0; b < 8; ++b) sum += tq[b];
              }
              if (e < n4) {
                if (!arrived) sum[0] = __uint_as_float(0x7fc00000u);   // the producers never came: make it visible
                uint32_t hi[2], mid[2], lo[2];
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                  const float v0 = sum[2 * i], v1 = sum[2 * i + 1];
                  const uint32_t h = pack_bf16x2(v0, v1);
                  const float r0 = v0 - bf16_bits_to_f32(h & 0xffffu), r1 = v1 - __uint_as_float(h & 0xffff0000u);
                  const uint32_t m = pack_bf16x2(r0, r1);
                  const float q0 = r0 - bf16_bits_to_f32(m & 0xffffu), q1 = r1 - __uint_as_float(m & 0xffff0000u);
                  hi[i] = h; mid[i] = m; lo[i] = pack_bf16x2(q0, q1);
                }
                uint16_t* dst = th + tok * 64 + 4 * j4;
                *reinterpret_cast<u32x2*>(dst) = u32x2{hi[0], hi[1]};
                *reinterpret_cast<u32x2*>(dst + MT * 64) = u32x2{mid[0], mid[1]};
                *reinterpret_cast<u32x2*>(dst + 2 * MT * 64) = u32x2{lo[0], lo[1]};
              }
            }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            if (lane == 0) __hip_atomic_store(&s_tstate[mi], arrived ? 2u : 3u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
          } else {
            uint32_t spins = 0;
            while (__hip_atomic_load(&s_tstate[mi], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) < 2u) {
              if (++spins > 4 * kBlkSpinLimit) break;   // the loading wave itself gives up long before this
              __builtin_amdgcn_s_sleep(8);
            }
          }
        }
        f32x16 l;
#pragma unroll
        for (int i = 0; i < 16; ++i) l[i] = 0.f;
        const unsigned char* trow = tarea + ((mi * 3) * MT + (n32 < MT ? n32 : 0)) * 128 + kg * 16;
#pragma unroll
        for (int st = 0; st < 4; ++st) {
          if (16 * st < mem.r) {
            const bf16x8 bf = __builtin_bit_cast(bf16x8, bfrag[st]);
#pragma unroll
            for (int term = 0; term < 3; ++term) {
              u32x4 tv = *reinterpret_cast<const u32x4*>(trow + term * MT * 128 + st * 32);
              if (n32 >= a.M || 16 * st + 8 * kg >= mem.r) tv = u32x4{0u, 0u, 0u, 0u};   // rows beyond the tokens, ranks beyond r: never written
              l = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, tv), bf, l, 0, 0, 0);
            }
          }
        }
#pragma unroll
        for (int q = 0; q < MR; ++q) out[q] += l[q] * mem.lora_scale;
      }
      {
        const float bias = bf16_bits_to_f32(bias_bits);   // +0 without one
#pragma unroll
        for (int q = 0; q < MR; ++q) out[q] += bias;
      }

      bool finish = true;              // this wave stores the tile (or the pair's activation)
      if (S.Sk > 1) {
        // K is split over ranges of workgroups: leave this range's share in the workspace and count; the wave that
        // arrives last adds the shares in range order.  (A gate / up pair counts once, after up.)
        uint64_t* mine = reinterpret_cast<uint64_t*>(a.partial + S.partial_off + (((int64_t)cur.g.range * S.total_tiles + nt) * 64 + lane) * MR);
#pragma unroll
        for (int q2 = 0; q2 < MR / 2; ++q2) {
          const uint64_t v = (uint64_t)__float_as_uint(out[2 * q2]) | ((uint64_t)__float_as_uint(out[2 * q2 + 1]) << 32);
          __hip_atomic_store(mine + q2, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        finish = false;
        if (!(S.pairs && cur.h == 0)) {
          __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): the shares are in memory before the count
          const int v = cur.g.slot + cur.j * cur.g.slots_r;
          uint32_t* ctr = a.counters + S.ctr_off + v;
          uint32_t old = 0;
          if (lane == 0) old = __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          old = __builtin_amdgcn_readfirstlane(old);
          if (old == (uint32_t)(S.Sk - 1)) {
            finish = true;
            if (lane == 0) __hip_atomic_store(ctr, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next call
            auto range_sum = [&](int tile, float (&dst)[MR]) {
              const uint64_t* p = reinterpret_cast<const uint64_t*>(a.partial + S.partial_off + ((int64_t)tile * 64 + lane) * MR);
              const int64_t stride = (int64_t)S.total_tiles * 64 * MR / 2;
#pragma unroll
              for (int q = 0; q < MR; ++q) dst[q] = 0.f;
              for (int z0 = 0; z0 < S.Sk; z0 += 4) {
                uint64_t w[4][MR / 2];
#pragma unroll
                for (int b = 0; b < 4; ++b)
#pragma unroll
                  for (int q2 = 0; q2 < MR / 2; ++q2) {
                    w[b][q2] = 0ull;   // +0.0f twice
                    if (z0 + b < S.Sk) w[b][q2] = __hip_atomic_load(p + (int64_t)(z0 + b) * stride + q2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                  }
#pragma unroll
                for (int b = 0; b < 4; ++b)
#pragma unroll
                  for (int q2 = 0; q2 < MR / 2; ++q2) {
                    dst[2 * q2] += __uint_as_float((uint32_t)w[b][q2]);
                    dst[2 * q2 + 1] += __uint_as_float((uint32_t)(w[b][q2] >> 32));
                  }
              }
            };
            range_sum(nt, out);
            if (S.pairs) range_sum(v, held);   // gate_proj's tile of the pair
          }
        }
      } else if (S.pairs && cur.h == 0) {
#pragma unroll
        for (int q = 0; q < MR; ++q) held[q] = out[q];
        finish = false;
      }

      if (finish) {
        uint32_t bits[MR];
        uint16_t* ybase; int64_t ldy, n0, nlim; bool vec;
        if (S.pairs) {
          // act = bf16(bf16(SiLU(gate)) * up) on the bf16-rounded projections: what a bf16 model evaluated operator
          // by operator gives
#pragma unroll
          for (int q = 0; q < MR; q += 2) {
            const uint32_t gpk = pack_bf16x2(held[q], held[q + 1]), upk = pack_bf16x2(out[q], out[q + 1]);
            const uint32_t r = silu_mul2(gpk, upk);
            bits[q] = r & 0xffffu; bits[q + 1] = r >> 16;
          }
          ybase = S.act; ldy = S.ld_act; n0 = (int64_t)(nt - S.mem[1].tile_begin) * 32; nlim = S.mem[0].N; vec = S.act_vec != 0;
        } else {
#pragma unroll
          for (int q = 0; q < MR; ++q) bits[q] = f32_to_bf16_bits(out[q]);
          ybase = mem.y; ldy = mem.ldy; n0 = row0; nlim = mem.N; vec = mem.y_vec != 0;
        }
        if (vec && n0 + 32 <= nlim) {
          // whole tile, 16-byte aligned rows: transposed through LDS, one 16-byte store per lane
#pragma unroll
          for (int q = 0; q < MR; ++q) {
            const int tok = 8 * (q >> 2) + 4 * kg + (q & 3);
            ytile[tok * 32 + n32] = (uint16_t)bits[q];
          }
          asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
          const int tok = lane >> 2, part = lane & 3;
          if (tok < a.M) {
            const u32x4 v = *reinterpret_cast<const u32x4*>(ytile + tok * 32 + part * 8);
            *reinterpret_cast<u32x4*>(ybase + (int64_t)tok * ldy + n0 + part * 8) = v;
          }
          asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // read before the next unit overwrites the tile
        } else {
#pragma unroll
          for (int q = 0; q < MR; ++q) {
            const int tok = 8 * (q >> 2) + 4 * kg + (q & 3);
            if (tok < a.M && n0 + n32 < nlim) ybase[(int64_t)tok * ldy + n0 + n32] = (uint16_t)bits[q];
          }
        }
      }
      cur = nxt;
      have_cur = have_next;
    }
  }

  leave();
}

// ---- host ------------------------------------------------------------------------------------------------------

constexpr size_t kBlkLdsMax = 160 * 1024 - 2048;   // the static words (row statistics, t states) take the first aligned slots of the CU's 160 KiB

static int g_blk_cus = 0;     // compute units of the device (one persistent workgroup each)
static int g_blk_force_kr = 0;

// Chooses the K-ranges of a stage for n_cons consumer workgroups and fills the stage's plan fields.  Model: a wave
// multiplies one tile in about t_tile us when nothing holds it up, the chip streams about 6.5 MB per us; a unit is
// as long as its K-range, a wave's units run one after the other, and splitting K costs a trip through memory.
static int plan_block_stage(BlkStage& S, int M, int MR, int n_cons, size_t x_budget) {
  const int D = kBlkD;
  int cap = (int)(((int64_t)(x_budget / (size_t)(M + 1)) - 16) / 256);
  cap -= cap % D;
  if (cap < D) return QERL_ERR_SHAPE;
  const int kt_pad = (int)(ceil_div(S.k_tiles, D) * D);
  const double t_tile = MR == 4 ? 0.55 : 0.65, chip_rate = 6.5e6, wave_rate = kPackTileBytes / t_tile;   // bytes per us
  const double bytes = (double)S.total_tiles * S.k_tiles * kPackTileBytes;
  int best = 0;
  double best_cost = 0;
  for (int kr = D; kr <= (cap < kt_pad ? cap : kt_pad); kr += D) {
    if (g_blk_force_kr > 0 && kr != g_blk_force_kr) continue;
    const int Sk = (int)ceil_div(S.k_tiles, kr);
    if (Sk > n_cons) continue;
    const int per_range = n_cons / Sk;
    const int64_t slots_r = (int64_t)per_range * kBlkWaves;
    const int64_t rounds = ceil_div(S.total_v, slots_r);
    const int passes = (int)rounds * (S.pairs ? 2 : 1);
    const int64_t active = (S.total_v < slots_r ? S.total_v : slots_r) * Sk;
    const double rate = active * wave_rate < chip_rate ? active * wave_rate : chip_rate;
    const double extra = Sk > 1 ? 1.5 * Sk * S.total_tiles * 64.0 * MR * 4 : 0.0;   // partial tiles out and back
    double cost = (bytes + extra) / rate;
    const double chain = passes * kr * t_tile;
    cost = cost > chain ? cost : chain;
    cost += 0.5 * passes + (Sk > 1 ? 3.0 : 0.0);
    if (best == 0 || cost < best_cost - 1e-9) { best = kr; best_cost = cost; }
  }
  if (best == 0) return QERL_ERR_SHAPE;
  S.kr_len = best;
  S.Sk = (int)ceil_div(S.k_tiles, best);
  S.per_range = n_cons / S.Sk;
  return QERL_OK;
}

// Fills in the plan of every stage and the LDS layout; returns the LDS bytes and workspace needs.
int plan_block(BlkArgs& a, size_t* lds_bytes, int* MR_out, size_t* partial_floats, size_t* counter_words) {
  if (g_blk_cus == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) {
      (void)hipGetLastError();
      n = 256;   // MI355X; also lets the plan be computed on a host without a GPU (workspace sizing)
    }
    g_blk_cus = n;
  }
  const int MR = a.M <= 8 ? 4 : 8, MT = MR == 4 ? 8 : 16;
  *MR_out = MR;
  a.n_wgs = g_blk_cus;
  int n_lora = 0, pmax = 0;
  for (int s = 0; s < a.n_stages; ++s) {
    BlkStage& S = a.st[s];
    int rt = 0;
    for (int i = 0; i < S.n_members; ++i) if (S.mem[i].r > 0) { S.mem[i].t_off = rt; rt += S.mem[i].r; ++n_lora; } else S.mem[i].t_off = 0x7fffffff;
    for (int i = S.n_members; i < kMaxGroup; ++i) S.mem[i].t_off = 0x7fffffff;
    S.r_total = rt;
    S.n_producers = 0;
    if (rt > 0) {
      int64_t np = ceil_div(2 * (int64_t)S.k_tiles, kBlkWaves);   // one half K-tile per producer wave and tile pair
      S.n_producers = (int)(np < 1 ? 1 : (np > 16 ? 16 : np));
    }
    pmax = S.n_producers > pmax ? S.n_producers : pmax;
  }
  a.n_prod_max = pmax;
  const int n_cons = a.n_wgs - pmax;
  if (n_cons < 1) return QERL_ERR_SHAPE;
  // LDS: x slice first, then the split t of the four member slots, then the waves' output tiles
  const size_t t_bytes = (size_t)kMaxGroup * 3 * MT * 64 * 2, y_bytes = (size_t)kBlkWaves * 16 * 32 * 2;
  const size_t x_budget = (kBlkLdsMax - t_bytes - y_bytes - 512) & ~(size_t)255;
  size_t xs_max = 0, part = 0, ctrs = 0, prod_need = 0;
  for (int s = 0; s < a.n_stages; ++s) {
    BlkStage& S = a.st[s];
    const int rc = plan_block_stage(S, a.M, MR, n_cons, x_budget);
    if (rc != QERL_OK) return rc;
    const size_t xs = (size_t)(a.M + 1) * (size_t)(S.kr_len * 256 + 16);
    xs_max = xs > xs_max ? xs : xs_max;
    S.ctr_off = (int)ctrs; S.partial_off = (int64_t)part;
    if (S.Sk > 1) { ctrs += (size_t)S.total_v; part += (size_t)S.Sk * S.total_tiles * 64 * MR; }
    if (S.n_producers > 0) {
      const int64_t steps = S.K / 16;
      S.prod_steps = (int)ceil_div(steps, S.n_producers);
      const size_t rows = (size_t)(S.r_total < 64 ? S.r_total : 64) + a.M + 1;
      const size_t red = lora_producer_red_bytes(kBlkWaves, MR);
      int64_t cb = ((int64_t)((kBlkLdsMax - red - 256) / rows) - 16) / 32;
      cb = cb < S.prod_steps ? cb : S.prod_steps;
      cb = cb < kProdMaxSteps ? cb : kProdMaxSteps;
      if (cb < 1) return QERL_ERR_SHAPE;
      S.prod_cb = (int)cb;
      S.prod_red_off = (int)((rows * (size_t)(cb * 32 + 16) + 255) & ~(size_t)255);
      const size_t need = S.prod_red_off + red;
      prod_need = need > prod_need ? need : prod_need;
    }
  }
#ifdef QERL_TUNING_HOOKS
  if (getenv("QERL_BLK_TRACE"))
    for (int s = 0; s < a.n_stages; ++s)
      fprintf(stderr, "block plan: M %d stage %d K-tiles %d tiles %d units %d  kr_len %d Sk %d per_range %d producers %d\n", a.M, s,
              a.st[s].k_tiles, a.st[s].total_tiles, a.st[s].total_v, a.st[s].kr_len, a.st[s].Sk, a.st[s].per_range, a.st[s].n_producers);
#endif
  a.t_lds_off = (int)((xs_max + 255) & ~(size_t)255);
  a.y_lds_off = a.t_lds_off + (int)t_bytes;
  size_t total = (size_t)a.y_lds_off + y_bytes;
  total = total > prod_need ? total : prod_need;
  if (total > kBlkLdsMax) return QERL_ERR_SHAPE;
  *lds_bytes = total;
  *partial_floats = part;
  *counter_words = ctrs;
  return QERL_OK;
}

template <int MR>
static int launch_block_t(const BlkArgs& a, size_t lds, hipStream_t st) {
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&block_kernel<MR>), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)kBlkLdsMax) != hipSuccess)
      return launch_status();
    attr_set = true;
  }
  block_kernel<MR><<<dim3(a.n_wgs), dim3(kBlkThreads), lds, st>>>(a);
  return launch_status();
}

int launch_block(const BlkArgs& a, size_t lds, int MR, hipStream_t st) {
  // every pointer the kernel dereferences and every bound its indexing assumes
  if (a.M < 1 || a.M > 16 || a.n_stages < 1 || a.n_stages > kBlkMaxStages || a.n_wgs < 2 || a.n_prod_max < 0 || a.n_prod_max >= a.n_wgs)
    return QERL_ERR_SHAPE;
  if (!a.ctl || !a.counters || !a.partial || !a.tpart) return QERL_ERR_NULL;
  if ((MR != 4 && MR != 8) || (a.M > 8 && MR != 8) || lds > kBlkLdsMax || a.t_lds_off < 0 || a.y_lds_off <= a.t_lds_off ||
      (size_t)a.y_lds_off + kBlkWaves * 16 * 32 * 2 > lds)
    return QERL_ERR_SHAPE;
  const int n_cons = a.n_wgs - a.n_prod_max;
  for (int s = 0; s < a.n_stages; ++s) {
    const BlkStage& S = a.st[s];
    if (!S.x || S.ldx < S.K || S.ldx % 8 != 0 || ((uintptr_t)S.x & 15) != 0 || S.K < 16 || S.K % 16 != 0) return QERL_ERR_ALIGN;
    if (S.k_tiles != (int)ceil_div(S.K, kPackTileK) || S.n_members < 1 || S.n_members > kMaxGroup) return QERL_ERR_SHAPE;
    if (S.kr_len < kBlkD || S.kr_len % kBlkD != 0 || S.Sk < 1 || (int64_t)S.Sk * S.kr_len < S.k_tiles || (int64_t)(S.Sk - 1) * S.kr_len >= S.k_tiles ||
        S.per_range < 1 || (int64_t)S.per_range * S.Sk > n_cons || (size_t)(a.M + 1) * (size_t)(S.kr_len * 256 + 16) > (size_t)a.t_lds_off)
      return QERL_ERR_SHAPE;
    if (S.gain && (((uintptr_t)S.gain & 15) != 0 || ((uintptr_t)S.noise & 15) != 0 || S.K % 8 != 0)) return QERL_ERR_ALIGN;
    int tiles = 0;
    for (int i = 0; i < S.n_members; ++i) {
      const BlkMember& m = S.mem[i];
      if (!m.packed || !m.tensor_scale || m.N < 1 || m.n_tiles != (int)ceil_div(m.N, kPackTileRows) || m.tile_begin != tiles) return QERL_ERR_SHAPE;
      if (!(S.pairs) && !m.y) return QERL_ERR_NULL;
      if (m.r < 0 || m.r > 64 || m.r % 8 != 0 || (m.r > 0 && (!m.A || !m.B || ((uintptr_t)m.A & 15) != 0 || ((uintptr_t)m.B & 15) != 0))) return QERL_ERR_SHAPE;
      tiles += m.n_tiles;
    }
    for (int i = S.n_members; i < kMaxGroup; ++i)
      if (S.mem[i].tile_begin != 0x7fffffff || S.mem[i].packed != S.mem[0].packed) return QERL_ERR_SHAPE;
    if (tiles != S.total_tiles) return QERL_ERR_SHAPE;
    if (S.pairs) {
      if (S.n_members != 2 || S.mem[0].N != S.mem[1].N || S.total_v != S.mem[0].n_tiles || !S.act || S.ld_act < S.mem[0].N) return QERL_ERR_SHAPE;
    } else if (S.total_v != S.total_tiles) {
      return QERL_ERR_SHAPE;
    }
    if (S.r_total > 0) {
      if (S.n_producers < 1 || S.n_producers > a.n_prod_max || S.n_producers > 16 || S.r_total > 256 || S.r_total % 8 != 0) return QERL_ERR_SHAPE;
      const size_t rows = (size_t)(S.r_total < 64 ? S.r_total : 64) + a.M + 1;
      if (S.prod_steps < 1 || S.prod_cb < 1 || S.prod_cb > kProdMaxSteps || (int64_t)S.prod_steps * S.n_producers < S.K / 16 ||
          rows * (size_t)(S.prod_cb * 32 + 16) > (size_t)S.prod_red_off ||
          (size_t)S.prod_red_off + lora_producer_red_bytes(kBlkWaves, MR) > lds)
        return QERL_ERR_SHAPE;
    } else if (S.n_producers != 0) {
      return QERL_ERR_SHAPE;
    }
  }
  return MR == 4 ? launch_block_t<4>(a, lds, st) : launch_block_t<8>(a, lds, st);
}

}  // namespace qerl

#ifdef QERL_TUNING_HOOKS   // built only for tuning sessions: they change process-wide state
extern "C" QERL_API void qerl_debug_force_block_kr(int kr) { qerl::g_blk_force_kr = kr; }
#endif
