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
// drain, the spread of its workgroups and the gap to the next launch each time; here, while a wave waits at a
// stage boundary for the other workgroups' outputs, the first tiles of its next unit are already on their way.
//
// Structure:
//   * One workgroup of eight waves per CU (two per SIMD, 256 registers each).  A unit of work is one row tile (32
//     output rows) over one K-range of a stage; a wave owns its units outright: it streams the unit's packed tiles
//     through a ring of kBlkD tiles in registers (refilled in place, across unit, phase and stage boundaries),
//     multiplies them -- bare E2M1 values into one v_mfma_f32_32x32x16_bf16 per 16-input scale block, then
//     acc += E4M3 scale * product, as in linear_stream.hip -- and finishes the unit itself: tensor scale, LoRA
//     up-projection (B rows requested one ring round ahead), bias, store.  There is no synchronisation inside the
//     streaming loop; eight independent streams per CU keep ~74 KB in flight (16.5 MB over the chip).
//   * The K-range's slice of the stage input lives in LDS, shared by the waves (rows 16 bytes apart in bank space;
//     MFMA rows beyond the tokens read a zero row); on a normalising stage each workgroup computes the row
//     statistics itself while it loads the rows and normalises the slice in place.  When all of K does not fit,
//     the stage either runs in phases (the next part of K is staged after a workgroup barrier, the accumulators
//     wait in LDS meanwhile) or K is split over ranges of workgroups: every range leaves fp32 partial tiles in the
//     workspace, counts itself in the tile's arrival word, and the wave that arrives last adds the partials in
//     range order, applies LoRA and bias and stores -- fixed order, so results do not depend on timing.
//   * A gate_proj / up_proj pair: waves 0..3 of a workgroup own gate tiles, waves 4..7 the up tiles of the same
//     rows and hand them over through LDS; or (K split over ranges) one wave walks both tiles and the last wave to
//     arrive for the rows finishes both.  act = bf16(bf16(SiLU(gate)) * up) goes out with write-through stores.
//   * t = x A^T of a stage comes from producer workgroups at the front of the grid (lora_producer.hpp): one per
//     (pair of rank tiles, run of K); the one that arrives last adds the partials in producer order and publishes
//     the finished t and a ready word.  The first wave of a consumer workgroup that needs a member's t loads it
//     (one round of loads) and leaves it in LDS as three bf16 terms (exact to 2^-24 relative) for the others.
//   * Stage boundary: every wave waits for its own stores, one thread per workgroup counts in and waits until all
//     workgroups have (bounded spin), one wave invalidates the CU's caches (what the next stage reads was written
//     through to memory), the next input is staged.
// Every wait on another workgroup is bounded; a wait that gives up sets the sticky error word of the workspace
// (qerl_workspace_status), poisons nothing silently, and the control words are then left as they are.
#include <stdio.h>
#include <stdlib.h>
#include "linear.hpp"
#include "lora_producer.hpp"

namespace qerl {

constexpr int kBlkThreads = kBlkWaves * 64;
#ifndef QERL_BLK_DEPTH
#define QERL_BLK_DEPTH 4
#endif
constexpr int kBlkD = QERL_BLK_DEPTH;           // ring depth in tiles; every K-range length is a multiple of it
constexpr uint32_t kBlkSpinLimit = 1u << 17;    // polls of a bounded wait (x s_sleep: tens of milliseconds)

// Optional timeline stamps for tuning (build with -DQERL_BLK_TRACE): 16 time stamps (100 MHz) per wave, read back with
// qerl_debug_read_block_trace().  Stamp 0 is the kernel entry; stage s uses 1 + 5 s ...: boundary passed, input
// staged, first unit multiplied, first unit finished, last unit finished; 15 is the exit.
#ifdef QERL_BLK_TRACE
__device__ unsigned long long g_blk_trace[256 * kBlkWaves * 16];
#define BSTAMP(p) do { if (lane == 0 && blockIdx.x < 256) g_blk_trace[((int)blockIdx.x * kBlkWaves + wave) * 16 + (p)] = wall_clock64(); } while (0)
#else
#define BSTAMP(p) do { } while (0)
#endif

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

// The eight x fragments (one per 16-input scale block) of a K-tile, from the LDS slice.  They are requested a whole
// tile ahead (right after the previous tile's arithmetic, with the weight refill), so that no matrix instruction
// ever waits for an LDS round trip.
struct BlkXFrag { u32x4 f[8]; };
__device__ __forceinline__ void blk_xload(BlkXFrag& x, const unsigned char* xk) {
#ifdef QERL_BLK_NOXLOAD   // timing experiment
  return;
#endif
#pragma unroll
  for (int j = 0; j < 8; ++j) x.f[j] = *reinterpret_cast<const u32x4*>(xk + j * 32);
}

// One packed tile (32 rows x 128 inputs = 8 scale blocks) times its x fragments.  The issue order is pinned block by
// block: the matrix instruction of block j + 1 goes out BEFORE the scale-and-add of block j (whose product was
// issued a whole block earlier and is complete by then: no wait states), and the conversions of block j + 2 fill
// the time the matrix unit needs.  Left to itself the scheduler puts each scale-and-add right behind its own
// matrix instruction and pads the gap with idle cycles.
template <int MR>
__device__ __forceinline__ void blk_consume(const BlkTile& t, const BlkXFrag& x, float (&acc)[MR]) {
#ifdef QERL_BLK_NOCOMPUTE   // timing experiment: the loads stay alive, the arithmetic is gone
  acc[0] += __uint_as_float((t.c0[0] ^ t.c0[3] ^ t.c1[0] ^ t.c1[3] ^ t.sc[0] ^ t.sc[1] ^ x.f[0][0] ^ x.f[7][3]) & 0x3fffffu);
  return;
#endif
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  f32x16 tmp[2];
  bf16x8 w = blk_e2m1x8(t.c0[0]);
  tmp[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, x.f[0]), w, zero, 0, 0, 0);
  w = blk_e2m1x8(t.c0[1]);
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    __builtin_amdgcn_sched_barrier(0);
    if (j + 1 < 8) tmp[(j + 1) & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, x.f[j + 1]), w, zero, 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    const float s = e4m3_byte_f32(t.sc[j >> 2], j & 3);
#pragma unroll
    for (int q = 0; q < MR; ++q) acc[q] = __builtin_fmaf(s, tmp[j & 1][q], acc[q]);
    if (j + 2 < 8) w = blk_e2m1x8(j + 2 < 4 ? t.c0[(j + 2) & 3] : t.c1[(j + 2) & 3]);
    // all 16 registers of the product stay reserved until here: handing the unused ones to other values would
    // make those writes wait for the matrix instruction that is still writing the block (a dozen idle cycles each)
    asm volatile("" :: "v"(tmp[j & 1]));
  }
}

// Workgroup barrier for data that went through LDS only: waits for this wave's LDS operations, not for its
// outstanding global loads (__syncthreads() would wait for the whole weight ring to come in).
__device__ __forceinline__ void blk_lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// Bounded wait until *word >= target (agent scope).  Returns false when it gave up.
__device__ __forceinline__ bool blk_wait_ge(const uint32_t* word, uint32_t target, int sleep, uint32_t limit = kBlkSpinLimit) {
  for (uint32_t spins = 0; spins < limit; ++spins) {
    if (__hip_atomic_load(word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= target) return true;
    if (sleep > 8) __builtin_amdgcn_s_sleep(32); else __builtin_amdgcn_s_sleep(2);
  }
  return false;
}

// One wave that waits, with the kernels' bounded wait cut to `polls` polls, for a hand-over word that nobody
// raises, gives up, records it in the sticky word as the kernels do, and exits: the error path, end to end, with
// nothing hanging.
__global__ void blk_wait_selftest_kernel(uint32_t* ctl, uint32_t polls) {
  if (threadIdx.x != 0) return;
  if (!blk_wait_ge(ctl + kBlkReady + kBlkMaxStages - 1, 0xffffffffu, 2, polls))
    __hip_atomic_fetch_or(ctl + kCtlErr, 2u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
int launch_block_wait_selftest(uint32_t* ctl, uint32_t polls, hipStream_t st) {
  blk_wait_selftest_kernel<<<1, 64, 0, st>>>(ctl, polls);
  return launch_status();
}

template <int MR>
__global__ __launch_bounds__(kBlkThreads) void block_kernel(const BlkArgs a) {
  // dynamic LDS: x slice [M + 1 rows][xs_stride], then the split t of up to four members, then one output tile
  // per wave.  256-byte alignment matters: 16-byte LDS accesses from a misaligned base run several times slower.
  extern __shared__ __attribute__((aligned(256))) unsigned char smem[];
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
  BSTAMP(0);
  uint32_t* const err_word = a.ctl + kCtlErr;
  unsigned char* const tarea = smem + a.t_lds_off;
  uint16_t* const ytile = reinterpret_cast<uint16_t*>(smem + a.y_lds_off) + wave * (16 * 32);

  // ---- stage boundary: everybody's outputs of the previous stage are complete and visible ----------------------
  // (What a later stage reads -- the gated activation -- is stored with agent-scope atomic stores, which go
  // through to memory, so no cache write-back is needed here: each wave waits for its own stores, one thread
  // counts the workgroup in and waits for the others, one wave invalidates the CU's caches.)
  auto stage_boundary = [&](int s) {
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's stores of the stage have completed
    __syncthreads();
    if (wave == 0) {
      if (lane == 0) {
        __hip_atomic_fetch_add(a.ctl + kBlkBarrier, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (!blk_wait_ge(a.ctl + kBlkBarrier, (uint32_t)(a.n_wgs * s), 1))
          __hip_atomic_fetch_or(err_word, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    }
    __syncthreads();
  };
  // ---- exit: the last workgroup to leave re-arms the control words, unless a wait gave up somewhere -------------
  auto leave = [&]() {
    __syncthreads();
    if (tid == 0) {
      const uint32_t old = __hip_atomic_fetch_add(a.ctl + kBlkExit, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (old == (uint32_t)(a.n_wgs - 1) &&
          __hip_atomic_load(err_word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u) {
        for (int s = 0; s < kBlkMaxStages; ++s) {
          __hip_atomic_store(a.ctl + kBlkArrive + s, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          __hip_atomic_store(a.ctl + kBlkReady + s, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
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
      BSTAMP(1 + 5 * s);
      if (wg >= S.n_producers) continue;
      const bool norm = S.gain != nullptr;
      if (norm) {                      // row statistics over all of K: wave w owns token rows w and w + 8
        const int chunks_row = (int)(S.K / 8);
#pragma unroll
        for (int r = 0; r < MT / 8; ++r) {
          const int t = wave + 8 * r;
          float ss = 0.f;
          for (int c0 = 0; c0 < chunks_row; c0 += 64 * 10) {
            u32x4 xq[10];
#pragma unroll
            for (int i = 0; i < 10; ++i) {
              const int c = c0 + lane + 64 * i;
              xq[i] = u32x4{0u, 0u, 0u, 0u};
              if (t < a.M && c < chunks_row) xq[i] = *reinterpret_cast<const u32x4*>(S.x + (int64_t)t * S.ldx + (int64_t)c * 8);
            }
#pragma unroll
            for (int i = 0; i < 10; ++i) ss += sumsq(xq[i]);
          }
          const float rstd = 1.0f / sqrtf(wave_sum(ss) / (float)S.K + S.eps);
          if (lane == 0 && t < a.M) s_rstd[t] = rstd;
        }
        __syncthreads();
      }
      LoraProducerArgs p;
      p.x = S.x; p.ldx = S.ldx; p.x2 = nullptr; p.ldx2 = 0;
      p.M = a.M; p.K = S.K; p.r_total = S.r_total; p.n_members = S.n_members;
#pragma unroll
      for (int i = 0; i < kMaxGroup; ++i) { p.A[i] = S.mem[i].A; p.t_off[i] = S.mem[i].t_off; }
      p.index = wg % S.prod_k; p.only_pair = wg / S.prod_k; p.n_arrivals = S.n_producers; p.n_k = S.prod_k;
      p.tfinal = a.tfinal + (int64_t)s * kBlkTfinalWords; p.ready = a.ctl + kBlkReady + s;
      p.prod_steps = S.prod_steps; p.prod_cb = S.prod_cb; p.prod_red_off = S.prod_red_off;
      p.tpart = a.tpart + (int64_t)s * kBlkTpartWords; p.arrive = a.ctl + kBlkArrive + s;
      p.gain = S.gain; p.noise = S.noise; p.rstd = s_rstd;
      BSTAMP(2 + 5 * s);
      if (norm) lora_producer<MR, 2, kBlkWaves>(p, smem);
      else lora_producer<MR, 0, kBlkWaves>(p, smem);
      BSTAMP(5 + 5 * s);
    }
    BSTAMP(15);
    leave();
    return;
  }

  // ---- which units are mine ----------------------------------------------------------------------------------
  // A stage's K-tiles are cut into Sk ranges (of workgroups) x `phases` (in time) x kr_len tiles.  A wave owns row
  // tiles outright: tile v = slot + j * slots_r of its range, j = 0 .. n_my - 1, and walks each of them once per
  // phase (the accumulators wait in LDS between phases, the workgroup re-stages its x slice at each phase).
  // Pairs (gate_proj / up_proj), pairs == 1: waves 0..3 of a workgroup take gate tiles, waves 4..7 the up tiles of the
  // same rows; wave w + 4 hands its finished tile to wave w, which forms SiLU(gate) (.) up and stores it.  pairs == 2
  // (K split over ranges of workgroups, one phase): a wave walks gate_proj's tile and then up_proj's tile of the same
  // rows over its K-range, leaves both shares in the workspace, and the wave that arrives last for the rows adds the
  // shares of both, applies LoRA and bias to each and stores SiLU(gate) (.) up.
  struct Geo { int range, slot, slots_r, n_my; };
  auto geo = [&](int s) {
    const BlkStage& S = a.st[s];
    Geo g;
    g.range = cons / S.per_range;
    const int ci = cons - g.range * S.per_range;
    if (S.pairs == 1) { g.slot = ci * (kBlkWaves / 2) + (wave & 3); g.slots_r = S.per_range * (kBlkWaves / 2); }
    else { g.slot = ci * kBlkWaves + wave; g.slots_r = S.per_range * kBlkWaves; }
    g.n_my = (g.range < S.Sk && g.slot < S.total_v) ? (S.total_v - g.slot + g.slots_r - 1) / g.slots_r : 0;
    return g;
  };
  auto seg_k0 = [&](const BlkStage& S, int range, int ph) { return (range * S.phases + ph) * S.kr_len; };
  struct Pass { int s, ph, j, sub; Geo g; };   // sub: pairs computed one after the other by one wave (pairs == 2): 0 gate_proj's tile, 1 up_proj's
  // row tile (within the stage's stacked members) of a pass
  auto pass_tile = [&](const Pass& p) {
    const BlkStage& S = a.st[p.s];
    const int v = p.g.slot + p.j * p.g.slots_r;
    return ((S.pairs == 1 && wave >= kBlkWaves / 2) || (S.pairs == 2 && p.sub)) ? S.mem[1].tile_begin + v : v;
  };
  auto member_of = [&](const BlkStage& S, int nt) {
    return (nt >= S.mem[1].tile_begin ? 1 : 0) + (nt >= S.mem[2].tile_begin ? 1 : 0) + (nt >= S.mem[3].tile_begin ? 1 : 0);
  };
  // address of the first tile of a pass, its K-tiles that exist, and the distance between successive K-tiles (the
  // members' tile order is given by two strides: row-tile-major as nvfp4_prepack writes it, or K-tile-major)
  auto pass_base = [&](const Pass& p, int64_t& kstride, int& nvalid) {
    const BlkStage& S = a.st[p.s];
    const int nt = pass_tile(p);
    int tb = 0;
    const uint8_t* mp = S.mem[0].packed;
    int64_t sk = S.mem[0].stride_k, sn = S.mem[0].stride_n;
    if (nt >= S.mem[1].tile_begin) { tb = S.mem[1].tile_begin; mp = S.mem[1].packed; sk = S.mem[1].stride_k; sn = S.mem[1].stride_n; }
    if (nt >= S.mem[2].tile_begin) { tb = S.mem[2].tile_begin; mp = S.mem[2].packed; sk = S.mem[2].stride_k; sn = S.mem[2].stride_n; }
    if (nt >= S.mem[3].tile_begin) { tb = S.mem[3].tile_begin; mp = S.mem[3].packed; sk = S.mem[3].stride_k; sn = S.mem[3].stride_n; }
    kstride = sk;
    const int k0 = seg_k0(S, p.g.range, p.ph);
    const int left = S.k_tiles - k0;
    nvalid = left < S.kr_len ? left : S.kr_len;
    return mp + (int64_t)(nt - tb) * sn + (int64_t)k0 * sk;
  };
  auto next_pass = [&](Pass& p) {     // false: there is none
    if (p.s >= 0 && a.st[p.s].pairs == 2 && p.sub == 0) { p.sub = 1; return true; }
    p.sub = 0;
    ++p.j;
    if (p.j < p.g.n_my) return true;
    p.j = 0;
    ++p.ph;
    if (p.g.n_my > 0 && p.ph < a.st[p.s].phases) return true;
    p.ph = 0;
    for (;;) {
      ++p.s;
      if (p.s >= a.n_stages) return false;
      p.g = geo(p.s);
      if (p.g.n_my > 0) return true;
    }
  };

  Pass cur;
  cur.s = -1; cur.ph = 0; cur.j = 0; cur.sub = 0; cur.g = Geo{0, 0, 1, 0};
  bool have_cur = next_pass(cur);
  const uint8_t* const park = a.st[0].mem[0].packed;   // where loads go that nobody needs: always valid memory
  BlkTile ring[D];
  auto issue_first_ring = [&]() {      // first D tiles of my first unit
    int64_t ks0 = 0;
    int nv = 1;
    const uint8_t* b0 = have_cur ? pass_base(cur, ks0, nv) : park;
    if (!have_cur) { ks0 = 0; nv = 1; }
#pragma unroll
    for (int d = 0; d < D; ++d) blk_issue(ring[d], b0 + (int64_t)(d < nv ? d : nv - 1) * ks0, lane, n32);
  };

  // ---- stage input: the K-tiles of (stage, range, phase) into LDS, normalised on the way if the stage normalises -----
  // Wave w owns token rows w and w + 8: it requests its rows' chunks (all of the row in the first phase of a
  // normalising stage, for the row statistics; the slice otherwise) in one round of loads, sums the squares, knows
  // rstd without asking anybody, and writes the slice to LDS; gain + noise of the slice go to LDS once (thread =
  // chunk) and the rows are normalised in place.  For the very first input the weight ring is requested right
  // behind the input's loads and before anything waits for them: a load issued behind the ring would wait for
  // ~70 KB per CU to come in first, and a ring issued after the staging would start microseconds late.
  constexpr int XB = MR == 4 ? 10 : 8;                      // chunks per lane and row in flight (registers: XB x rows x 4)
  constexpr int XR = MT / 8;                                // rows per wave
  auto stage_input = [&](int s, int ph, bool with_ring) {
    const BlkStage& S = a.st[s];
    const Geo g0 = geo(s);                                  // the range is the same for all waves of the workgroup
    const int xs_stride = S.kr_len * 256 + 16;
    const int chunks_row = (int)(S.K / 8);                  // 16-byte chunks of a row
    const int sl_chunks = S.kr_len * 16;                    // chunks of the slice (K-tiles padded)
    const int sl0 = seg_k0(S, g0.range, ph) * 16;
    const int sl_end = sl0 + sl_chunks < chunks_row ? sl0 + sl_chunks : chunks_row;
    const bool stage_slice = g0.range < S.Sk;
    const bool norm = S.gain != nullptr;
    const bool stats = norm && ph == 0;
    // gain + noise of the slice: thread = chunk, at most two chunks per thread
    u32x4 gv[2];
    f32x4 zv[2][2];
    if (norm && stage_slice) {
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        const int lc = tid + c * kBlkThreads, ch = sl0 + lc;
        gv[c] = u32x4{0u, 0u, 0u, 0u};
        zv[c][0] = f32x4{0.f, 0.f, 0.f, 0.f}; zv[c][1] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (lc < sl_chunks && ch < chunks_row) {
          gv[c] = *reinterpret_cast<const u32x4*>(S.gain + (int64_t)ch * 8);
          if (S.noise) {
            zv[c][0] = *reinterpret_cast<const f32x4*>(S.noise + (int64_t)ch * 8);
            zv[c][1] = *reinterpret_cast<const f32x4*>(S.noise + (int64_t)ch * 8 + 4);
          }
        }
      }
    }
    // my rows
    float ss[XR];
#pragma unroll
    for (int r = 0; r < XR; ++r) ss[r] = 0.f;
    const int cb = stats ? 0 : sl0, ce = stats ? chunks_row : sl_end;
    bool ring_pending = with_ring;
    if (stage_slice) {
      for (int c0 = cb; c0 < ce; c0 += 64 * XB) {
        u32x4 xq[XR][XB];
#pragma unroll
        for (int r = 0; r < XR; ++r) {
          const int t = wave + 8 * r;
#pragma unroll
          for (int i = 0; i < XB; ++i) {
            const int c = c0 + lane + 64 * i;
            xq[r][i] = u32x4{0u, 0u, 0u, 0u};
            if (t < a.M && c < ce) xq[r][i] = *reinterpret_cast<const u32x4*>(S.x + (int64_t)t * S.ldx + (int64_t)c * 8);
          }
        }
        if (ring_pending) { issue_first_ring(); ring_pending = false; }
#pragma unroll
        for (int r = 0; r < XR; ++r) {
          const int t = wave + 8 * r;
#pragma unroll
          for (int i = 0; i < XB; ++i) {
            const int c = c0 + lane + 64 * i;
            if (stats) ss[r] += sumsq(xq[r][i]);
            if (t < a.M && c >= sl0 && c < sl_end) *reinterpret_cast<u32x4*>(smem + t * xs_stride + (c - sl0) * 16) = xq[r][i];
          }
        }
      }
    }
    if (ring_pending) issue_first_ring();
    if (stage_slice) {
      // the zero row, and zeros where the slice is padded beyond K
      for (int lc = tid; lc < sl_chunks; lc += kBlkThreads) {
        *reinterpret_cast<u32x4*>(smem + a.M * xs_stride + lc * 16) = u32x4{0u, 0u, 0u, 0u};
        if (sl0 + lc >= chunks_row)
          for (int t = 0; t < a.M; ++t) *reinterpret_cast<u32x4*>(smem + t * xs_stride + lc * 16) = u32x4{0u, 0u, 0u, 0u};
      }
    }
    if (norm) {
      if (stats) {
#pragma unroll
        for (int r = 0; r < XR; ++r) {
          const int t = wave + 8 * r;
          const float rstd = 1.0f / sqrtf(wave_sum(ss[r]) / (float)S.K + S.eps);
          if (lane == 0 && t < a.M) s_rstd[t] = rstd;        // (kept for the later phases)
        }
      }
      blk_lds_barrier();             // the raw rows and every row's rstd are in LDS
      if (stage_slice) {
        // normalised in place, thread = chunk (all threads busy whatever the number of tokens); gain + noise are in registers
#pragma unroll
        for (int c = 0; c < 2; ++c) {
          const int lc = tid + c * kBlkThreads;
          if (lc < sl_chunks && sl0 + lc < chunks_row) {
            float g[8];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              g[2 * j] = bf16_bits_to_f32(gv[c][j] & 0xffffu) + zv[c][j >> 1][(2 * j) & 3];
              g[2 * j + 1] = bf16_bits_to_f32(gv[c][j] >> 16) + zv[c][j >> 1][(2 * j + 1) & 3];
            }
            u32x4 o[MT];
#pragma unroll
            for (int t = 0; t < MT; ++t)
              if (t < a.M) o[t] = *reinterpret_cast<const u32x4*>(smem + t * xs_stride + lc * 16);
#pragma unroll
            for (int t = 0; t < MT; ++t) {
              if (t < a.M) {
                const float rs = s_rstd[t];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                  const float lo = bf16_bits_to_f32(o[t][j] & 0xffffu), hi = bf16_bits_to_f32(o[t][j] >> 16);
                  o[t][j] = pack_bf16x2(g[2 * j] * (lo * rs), g[2 * j + 1] * (hi * rs));
                }
                *reinterpret_cast<u32x4*>(smem + t * xs_stride + lc * 16) = o[t];
              }
            }
          }
        }
      }
    }
    blk_lds_barrier();
  };

  float* const parkbuf = reinterpret_cast<float*>(smem + a.p_lds_off) + wave * a.park_units * 64 * MR;
  uint32_t* const xflag = reinterpret_cast<uint32_t*>(smem + a.e_lds_off);                    // [4] units handed over, [4] units taken
  float* const xbuf = reinterpret_cast<float*>(smem + a.e_lds_off + 64) + (wave & 3) * 64 * MR;  // the pair's up_proj tile
  if (tid < 8) xflag[tid] = 0u;
  if (tid < kMaxGroup) s_tstate[tid] = 0u;

  for (int s = 0; s < a.n_stages; ++s) {
    const BlkStage& S = a.st[s];
    const Geo g0 = geo(s);             // range and K-tiles are the same for all waves of the workgroup
    const int xs_stride = S.kr_len * 256 + 16;
    const int xrow = n32 < a.M ? n32 : a.M;
    const unsigned char* const xbase = smem + xrow * xs_stride + kg * 16;
    const bool pair_up = S.pairs == 1 && wave >= kBlkWaves / 2;   // this wave computes up_proj tiles and hands them over
    const bool seq_pairs = S.pairs == 2;
    for (int ph = 0; ph < S.phases; ++ph) {
      if (ph == 0) {
        if (s > 0) {
          stage_boundary(s);
          if (tid < kMaxGroup) s_tstate[tid] = 0u;
          if (tid < 8) xflag[tid] = 0u;
        }
      } else {
        blk_lds_barrier();             // every wave is done with the previous phase's x slice
      }
      stage_input(s, ph, s == 0 && ph == 0);
      BSTAMP(2 + 5 * s);
      bool first_pass = true;
      BlkXFrag xf;
      const bool last_phase = ph + 1 == S.phases;
      while (have_cur && cur.s == s && cur.ph == ph) {
        const int nt = pass_tile(cur);
        const int mi = member_of(S, nt);
        const BlkMember& mem = S.mem[mi];
        int64_t kstride = 0;
        int nvalid = 1;
        const uint8_t* const base = pass_base(cur, kstride, nvalid);
        float* const myslot = parkbuf + (cur.j * 64 + lane) * MR;
        float acc[MR];
        if (ph == 0) {
#pragma unroll
          for (int q = 0; q < MR; ++q) acc[q] = 0.f;
        } else {
#pragma unroll
          for (int q4 = 0; q4 < MR / 4; ++q4) {
            const f32x4 v = *reinterpret_cast<const f32x4*>(myslot + 4 * q4);
            acc[4 * q4] = v[0]; acc[4 * q4 + 1] = v[1]; acc[4 * q4 + 2] = v[2]; acc[4 * q4 + 3] = v[3];
          }
        }
        if (first_pass) blk_xload(xf, xbase);   // (later units: requested at the end of the unit before)
        int i0 = 0;
        for (; i0 + D < S.kr_len; i0 += D) {
#pragma unroll
          for (int d = 0; d < D; ++d) {
            if (i0 + d < nvalid) blk_consume<MR>(ring[d], xf, acc);
            // the refill stays below the last use of the slot (see linear_stream.hip): same registers, no copies
#pragma unroll
            for (int q = 0; q < MR; ++q) asm volatile("" : "+v"(acc[q]));
            __builtin_amdgcn_sched_barrier(0);
            const int nx = i0 + D + d;
            blk_issue(ring[d], base + (int64_t)(nx < nvalid ? nx : nvalid - 1) * kstride, lane, n32);
            blk_xload(xf, xbase + (i0 + d + 1) * 256);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
        // last ring round of the unit: what the epilogue reads from memory is requested now, then the refills go
        // to the next unit (of this or a later phase or stage)
        Pass nxt = cur;
        const bool have_next = next_pass(nxt);
        int64_t nkstride = 0;
        int nnv = 1;
        const uint8_t* const nbase = have_next ? pass_base(nxt, nkstride, nnv) : park;
        if (!have_next) { nkstride = 0; nnv = 1; }
        const bool lora = last_phase && mem.r > 0 && !seq_pairs;   // (with K split over ranges, the wave that adds the shares applies it)
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
          const bool live = last_phase && !seq_pairs && mem.bias && row0 + n32 < mem.N;
          const uint16_t* src = live ? mem.bias + row0 + n32 : reinterpret_cast<const uint16_t*>(park);
          bias_bits = *src;
          if (!live) bias_bits = 0;
        }
#pragma unroll
        for (int d = 0; d < D; ++d) {
          if (i0 + d < nvalid) blk_consume<MR>(ring[d], xf, acc);
#pragma unroll
          for (int q = 0; q < MR; ++q) asm volatile("" : "+v"(acc[q]));
          __builtin_amdgcn_sched_barrier(0);
          blk_issue(ring[d], nbase + (int64_t)(d < nnv ? d : nnv - 1) * nkstride, lane, n32);
          blk_xload(xf, xbase + (d + 1 < D ? i0 + d + 1 : 0) * 256);   // the unit's next tile, or the first tile of the next unit of this phase
          __builtin_amdgcn_sched_barrier(0);
        }
        if (first_pass) BSTAMP(3 + 5 * s);

        if (!last_phase) {
          // more K to come for this tile: the accumulators wait in LDS
#pragma unroll
          for (int q4 = 0; q4 < MR / 4; ++q4)
            *reinterpret_cast<f32x4*>(myslot + 4 * q4) = f32x4{acc[4 * q4], acc[4 * q4 + 1], acc[4 * q4 + 2], acc[4 * q4 + 3]};
        } else {
          // ---- epilogue of the unit ----------------------------------------------------------------------------------
          const float S32 = *mem.tensor_scale;
          float out[MR];
#pragma unroll
          for (int q = 0; q < MR; ++q) out[q] = acc[q] * S32;
          auto add_lora_bias = [&](float (&o)[MR], const int mi_, const bool lora_, const u32x4 (&bf_)[4], const uint32_t bias_bits_) {
            const BlkMember& mm = S.mem[mi_];
            if (lora_) {
              // t of this member in LDS as three bf16 terms; the first wave of the workgroup that needs it puts it there
              uint32_t ts = __hip_atomic_load(&s_tstate[mi_], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP);
              if (ts < 2u) {
                int won = 0;
                if (lane == 0) {
                  uint32_t expect = 0u;
                  won = __hip_atomic_compare_exchange_strong(&s_tstate[mi_], &expect, 1u, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                                             __HIP_MEMORY_SCOPE_WORKGROUP) ? 1 : 0;
                }
                won = __builtin_amdgcn_readfirstlane(won);
                if (won) {
                  const bool arrived = blk_wait_ge(a.ctl + kBlkReady + s, 1u, 2);
                  if (!arrived && lane == 0) __hip_atomic_fetch_or(err_word, 2u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
                  // the finished t of this member, M x r floats: one round of loads, split into three bf16 terms
                  const int r4 = mm.r >> 2, n4 = a.M * r4;
                  const float* src = a.tfinal + (int64_t)s * kBlkTfinalWords + mm.t_off;
                  uint16_t* th = reinterpret_cast<uint16_t*>(tarea) + (mi_ * 3) * MT * 64;
                  f32x4 tq[4];
#pragma unroll
                  for (int i = 0; i < 4; ++i) {
                    const int e = lane + 64 * i, tok = e / r4, j4 = e - tok * r4;
                    tq[i] = f32x4{0.f, 0.f, 0.f, 0.f};
                    if (e < n4) tq[i] = *reinterpret_cast<const f32x4*>(src + (int64_t)tok * S.r_total + 4 * j4);
                  }
#pragma unroll
                  for (int i = 0; i < 4; ++i) {
                    const int e = lane + 64 * i, tok = e / r4, j4 = e - tok * r4;
                    if (e < n4) {
                      f32x4 sum = tq[i];
                      if (!arrived) sum[0] = __uint_as_float(0x7fc00000u);   // the producers never came: make it visible
                      uint32_t hi[2], mid[2], lo[2];
#pragma unroll
                      for (int k = 0; k < 2; ++k) {
                        const float v0 = sum[2 * k], v1 = sum[2 * k + 1];
                        const uint32_t h = pack_bf16x2(v0, v1);
                        const float r0 = v0 - bf16_bits_to_f32(h & 0xffffu), r1 = v1 - __uint_as_float(h & 0xffff0000u);
                        const uint32_t m = pack_bf16x2(r0, r1);
                        const float q0 = r0 - bf16_bits_to_f32(m & 0xffffu), q1 = r1 - __uint_as_float(m & 0xffff0000u);
                        hi[k] = h; mid[k] = m; lo[k] = pack_bf16x2(q0, q1);
                      }
                      uint16_t* dst = th + tok * 64 + 4 * j4;
                      *reinterpret_cast<u32x2*>(dst) = u32x2{hi[0], hi[1]};
                      *reinterpret_cast<u32x2*>(dst + MT * 64) = u32x2{mid[0], mid[1]};
                      *reinterpret_cast<u32x2*>(dst + 2 * MT * 64) = u32x2{lo[0], lo[1]};
                    }
                  }
                  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                  if (lane == 0) __hip_atomic_store(&s_tstate[mi_], arrived ? 2u : 3u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
                } else {
                  uint32_t spins = 0;
                  while (__hip_atomic_load(&s_tstate[mi_], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) < 2u) {
                    if (++spins > 4 * kBlkSpinLimit) break;   // the loading wave itself gives up long before this
                    __builtin_amdgcn_s_sleep(8);
                  }
                }
              }
              f32x16 l;
#pragma unroll
              for (int i = 0; i < 16; ++i) l[i] = 0.f;
              const unsigned char* trow = tarea + ((mi_ * 3) * MT + (n32 < MT ? n32 : 0)) * 128 + kg * 16;
#pragma unroll
              for (int st = 0; st < 4; ++st) {
                if (16 * st < mm.r) {
                  const bf16x8 bf = __builtin_bit_cast(bf16x8, bf_[st]);
#pragma unroll
                  for (int term = 0; term < 3; ++term) {
                    u32x4 tv = *reinterpret_cast<const u32x4*>(trow + term * MT * 128 + st * 32);
                    if (n32 >= a.M || 16 * st + 8 * kg >= mm.r) tv = u32x4{0u, 0u, 0u, 0u};   // rows beyond the tokens, ranks beyond r: never written
                    l = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, tv), bf, l, 0, 0, 0);
                  }
                }
              }
#pragma unroll
              for (int q = 0; q < MR; ++q) o[q] += l[q] * mm.lora_scale;
            }
            {
              const float bias = bf16_bits_to_f32(bias_bits_);   // +0 without one
#pragma unroll
              for (int q = 0; q < MR; ++q) o[q] += bias;
            }
          };
          bool finish = true;            // this wave stores the tile
          float up[MR];                  // pairs: up_proj's finished tile
          bool have_up = false;
          if (seq_pairs && cur.sub == 0) {
            // gate_proj's share of the rows waits in LDS while the wave walks up_proj's tile
#pragma unroll
            for (int q4 = 0; q4 < MR / 4; ++q4)
              *reinterpret_cast<f32x4*>(parkbuf + lane * MR + 4 * q4) = f32x4{out[4 * q4], out[4 * q4 + 1], out[4 * q4 + 2], out[4 * q4 + 3]};
            finish = false;
          } else if (seq_pairs) {
            // `out` is up_proj's share; both shares go to the workspace, the last wave to arrive for these rows finishes both
            float og[MR];
#pragma unroll
            for (int q4 = 0; q4 < MR / 4; ++q4) {
              const f32x4 v = *reinterpret_cast<const f32x4*>(parkbuf + lane * MR + 4 * q4);
              og[4 * q4] = v[0]; og[4 * q4 + 1] = v[1]; og[4 * q4 + 2] = v[2]; og[4 * q4 + 3] = v[3];
            }
            const int vt = nt - S.mem[1].tile_begin;     // the pair's index = gate_proj's tile
            const int64_t stride = (int64_t)S.total_tiles * 64 * MR / 2;
            uint64_t* const pg = reinterpret_cast<uint64_t*>(a.partial + S.partial_off + ((int64_t)vt * 64 + lane) * MR);
            uint64_t* const pu = reinterpret_cast<uint64_t*>(a.partial + S.partial_off + ((int64_t)nt * 64 + lane) * MR);
            if (S.Sk > 1) {
#pragma unroll
              for (int q2 = 0; q2 < MR / 2; ++q2) {
                __hip_atomic_store(pg + (int64_t)cur.g.range * stride + q2, (uint64_t)__float_as_uint(og[2 * q2]) | ((uint64_t)__float_as_uint(og[2 * q2 + 1]) << 32),
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __hip_atomic_store(pu + (int64_t)cur.g.range * stride + q2, (uint64_t)__float_as_uint(out[2 * q2]) | ((uint64_t)__float_as_uint(out[2 * q2 + 1]) << 32),
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              }
              __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): the shares are in memory before the count
              uint32_t* ctr = a.counters + S.ctr_off + vt;
              uint32_t old = 0;
              if (lane == 0) old = __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              old = __builtin_amdgcn_readfirstlane(old);
              finish = old == (uint32_t)(S.Sk - 1);
              if (finish && lane == 0) __hip_atomic_store(ctr, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next call
            }
            if (finish) {
              // B rows and biases of both members, and the shares, in one round of loads
              u32x4 bg[4], bu[4];
              int64_t brow = row0 + n32;
              brow = brow < mem.N ? brow : mem.N - 1;
              const BlkMember& m0 = S.mem[0];
#pragma unroll
              for (int st = 0; st < 4; ++st) {
                const int j0 = 16 * st + 8 * kg;
                bg[st] = u32x4{0u, 0u, 0u, 0u}; bu[st] = u32x4{0u, 0u, 0u, 0u};
                if (j0 < m0.r) bg[st] = *reinterpret_cast<const u32x4*>(m0.B + brow * m0.r + j0);
                if (j0 < mem.r) bu[st] = *reinterpret_cast<const u32x4*>(mem.B + brow * mem.r + j0);
              }
              uint32_t bias_g = 0, bias_u = 0;
              if (m0.bias && row0 + n32 < m0.N) bias_g = m0.bias[row0 + n32];
              if (mem.bias && row0 + n32 < mem.N) bias_u = mem.bias[row0 + n32];
              if (S.Sk > 1) {
#pragma unroll
                for (int q = 0; q < MR; ++q) { og[q] = 0.f; out[q] = 0.f; }
                constexpr int ZB = 2;
                for (int z0 = 0; z0 < S.Sk; z0 += ZB) {
                  uint64_t wg_[ZB][MR / 2], wu_[ZB][MR / 2];
#pragma unroll
                  for (int b = 0; b < ZB; ++b)
#pragma unroll
                    for (int q2 = 0; q2 < MR / 2; ++q2) {
                      wg_[b][q2] = 0ull; wu_[b][q2] = 0ull;
                      if (z0 + b < S.Sk) {
                        wg_[b][q2] = __hip_atomic_load(pg + (int64_t)(z0 + b) * stride + q2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        wu_[b][q2] = __hip_atomic_load(pu + (int64_t)(z0 + b) * stride + q2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                      }
                    }
#pragma unroll
                  for (int b = 0; b < ZB; ++b)
#pragma unroll
                    for (int q2 = 0; q2 < MR / 2; ++q2) {
                      og[2 * q2] += __uint_as_float((uint32_t)wg_[b][q2]);
                      og[2 * q2 + 1] += __uint_as_float((uint32_t)(wg_[b][q2] >> 32));
                      out[2 * q2] += __uint_as_float((uint32_t)wu_[b][q2]);
                      out[2 * q2 + 1] += __uint_as_float((uint32_t)(wu_[b][q2] >> 32));
                    }
                }
              }
              add_lora_bias(og, 0, m0.r > 0, bg, bias_g);
              add_lora_bias(out, 1, mem.r > 0, bu, bias_u);
#pragma unroll
              for (int q = 0; q < MR; ++q) { up[q] = out[q]; out[q] = og[q]; }
              have_up = true;
            }
          } else {
          if (S.Sk == 1) add_lora_bias(out, mi, lora, bfrag, bias_bits);

          if (S.Sk > 1) {
            // K is split over ranges of workgroups: leave this range's share in the workspace and count; the wave that
            // arrives last adds the shares in range order (all requested in one round of loads).
            uint64_t* mine = reinterpret_cast<uint64_t*>(a.partial + S.partial_off + (((int64_t)cur.g.range * S.total_tiles + nt) * 64 + lane) * MR);
#pragma unroll
            for (int q2 = 0; q2 < MR / 2; ++q2) {
              const uint64_t v = (uint64_t)__float_as_uint(out[2 * q2]) | ((uint64_t)__float_as_uint(out[2 * q2 + 1]) << 32);
              __hip_atomic_store(mine + q2, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): the shares are in memory before the count
            uint32_t* ctr = a.counters + S.ctr_off + nt;
            uint32_t old = 0;
            if (lane == 0) old = __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            old = __builtin_amdgcn_readfirstlane(old);
            finish = old == (uint32_t)(S.Sk - 1);
            if (finish) {
              if (lane == 0) __hip_atomic_store(ctr, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next call
              const uint64_t* p = reinterpret_cast<const uint64_t*>(a.partial + S.partial_off + ((int64_t)nt * 64 + lane) * MR);
              const int64_t stride = (int64_t)S.total_tiles * 64 * MR / 2;
#pragma unroll
              for (int q = 0; q < MR; ++q) out[q] = 0.f;
              constexpr int ZB = MR == 4 ? 16 : 8;     // ranges in flight per round
              for (int z0 = 0; z0 < S.Sk; z0 += ZB) {
                uint64_t w[ZB][MR / 2];
#pragma unroll
                for (int b = 0; b < ZB; ++b)
#pragma unroll
                  for (int q2 = 0; q2 < MR / 2; ++q2) {
                    w[b][q2] = 0ull;   // +0.0f twice
                    if (z0 + b < S.Sk) w[b][q2] = __hip_atomic_load(p + (int64_t)(z0 + b) * stride + q2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                  }
#pragma unroll
                for (int b = 0; b < ZB; ++b)
#pragma unroll
                  for (int q2 = 0; q2 < MR / 2; ++q2) {
                    out[2 * q2] += __uint_as_float((uint32_t)w[b][q2]);
                    out[2 * q2 + 1] += __uint_as_float((uint32_t)(w[b][q2] >> 32));
                  }
              }
              add_lora_bias(out, mi, lora, bfrag, bias_bits);
            }
          }
          }

          if (finish && pair_up) {
            // hand the finished up_proj tile to the wave that holds gate_proj's tile of the same rows
            const int fi = wave & 3;
            uint32_t spins = 0;
            while (__hip_atomic_load(&xflag[4 + fi], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) < (uint32_t)cur.j) {
              if (++spins > 4 * kBlkSpinLimit) break;   // (the buffer is free once the unit before has been taken)
              __builtin_amdgcn_s_sleep(2);
            }
#pragma unroll
            for (int q4 = 0; q4 < MR / 4; ++q4)
              *reinterpret_cast<f32x4*>(xbuf + lane * MR + 4 * q4) = f32x4{out[4 * q4], out[4 * q4 + 1], out[4 * q4 + 2], out[4 * q4 + 3]};
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            if (lane == 0) __hip_atomic_store(&xflag[fi], (uint32_t)(cur.j + 1), __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
            finish = false;
          }

          if (finish) {
            uint32_t bits[MR];
            uint16_t* ybase; int64_t ldy, n0, nlim; bool vec;
            if (S.pairs) {
              // act = bf16(bf16(SiLU(gate)) * up) on the bf16-rounded projections: what a bf16 model evaluated
              // operator by operator gives.  up_proj's tile comes from the partner wave.
              if (!have_up) {
                const int fi = wave & 3;
                uint32_t spins = 0;
                bool got = true;
                while (__hip_atomic_load(&xflag[fi], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) < (uint32_t)(cur.j + 1)) {
                  if (++spins > 4 * kBlkSpinLimit) { got = false; break; }
                  __builtin_amdgcn_s_sleep(2);
                }
#pragma unroll
                for (int q4 = 0; q4 < MR / 4; ++q4) {
                  const f32x4 v = *reinterpret_cast<const f32x4*>(xbuf + lane * MR + 4 * q4);
                  up[4 * q4] = v[0]; up[4 * q4 + 1] = v[1]; up[4 * q4 + 2] = v[2]; up[4 * q4 + 3] = v[3];
                }
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                if (lane == 0) {
                  __hip_atomic_store(&xflag[4 + fi], (uint32_t)(cur.j + 1), __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
                  if (!got) __hip_atomic_fetch_or(err_word, 4u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
              }
#pragma unroll
              for (int q = 0; q < MR; q += 2) {
                const uint32_t gpk = pack_bf16x2(out[q], out[q + 1]), upk = pack_bf16x2(up[q], up[q + 1]);
                const uint32_t r = silu_mul2(gpk, upk);
                bits[q] = r & 0xffffu; bits[q + 1] = r >> 16;
              }
              ybase = S.act; ldy = S.ld_act; n0 = row0; nlim = S.mem[0].N; vec = S.act_vec != 0;
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
                uint16_t* dst = ybase + (int64_t)tok * ldy + n0 + part * 8;
                if (S.pairs) {   // read by the next stage of this launch, on other compute units: through to memory
                  __hip_atomic_store(reinterpret_cast<uint64_t*>(dst), (uint64_t)v[0] | ((uint64_t)v[1] << 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                  __hip_atomic_store(reinterpret_cast<uint64_t*>(dst) + 1, (uint64_t)v[2] | ((uint64_t)v[3] << 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                } else {
                  *reinterpret_cast<u32x4*>(dst) = v;
                }
              }
              asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // read before the next unit overwrites the tile
            } else {
#pragma unroll
              for (int q = 0; q < MR; ++q) {
                const int tok = 8 * (q >> 2) + 4 * kg + (q & 3);
                if (tok < a.M && n0 + n32 < nlim) {
                  if (S.pairs) __hip_atomic_store(ybase + (int64_t)tok * ldy + n0 + n32, (uint16_t)bits[q], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                  else ybase[(int64_t)tok * ldy + n0 + n32] = (uint16_t)bits[q];
                }
              }
            }
          }
        }
        if (first_pass) BSTAMP(4 + 5 * s);
        first_pass = false;
        cur = nxt;
        have_cur = have_next;
      }
    }
    BSTAMP(5 + 5 * s);
  }

  BSTAMP(15);
  leave();
}

// ---- host ------------------------------------------------------------------------------------------------------

constexpr size_t kBlkLdsMax = 160 * 1024 - 2048;   // the static words (row statistics, t states) take the first aligned slots of the CU's 160 KiB

static int g_blk_cus = 0;     // compute units of the device (one persistent workgroup each)
static int g_blk_force_kr = 0, g_blk_force_phases = 0;

constexpr int kBlkParkMax = 2;   // accumulator tiles a wave may park between K-phases

struct BlkLds { size_t x, g, t, y, park, exch; };
static BlkLds blk_lds(int M, int MR, int kr, bool norm, int park_units, bool pairs) {
  const int MT = MR == 4 ? 8 : 16;
  BlkLds l;
  l.x = ((size_t)(M + 1) * (size_t)(kr * 256 + 16) + 255) & ~(size_t)255;
  l.g = 0; (void)norm;
  l.t = (size_t)kMaxGroup * 3 * MT * 64 * 2;
  l.y = (size_t)kBlkWaves * 16 * 32 * 2;
  l.park = (size_t)kBlkWaves * (size_t)park_units * 64 * MR * sizeof(float);
  l.exch = pairs ? 256 + (size_t)4 * 64 * MR * sizeof(float) : 0;
  return l;
}
static size_t blk_lds_total(const BlkLds& l) { return l.x + l.g + l.t + l.y + l.park + l.exch; }

// Chooses how a stage's K is cut -- Sk ranges of workgroups x phases in time x kr_len tiles -- for n_cons consumer
// workgroups, and fills the stage's plan fields.  Model: a wave multiplies one tile in about t_tile us when nothing
// holds it up (two waves share a SIMD), the chip streams about 6 MB per us; a wave's units and phases run one after
// the other; splitting K over workgroups costs a trip through memory and the partial tiles' traffic, an extra phase
// costs a workgroup barrier and a re-staging of x.  
static int plan_block_stage(BlkStage& S, int M, int MR, int n_cons, size_t lds_floor_park_exch, int* park_units) {
  const int D = kBlkD;
  const bool norm = S.gain != nullptr, pairs = S.pairs != 0;
  const int kt_pad = (int)(ceil_div(S.k_tiles, D) * D);
  const int cpt_cap = 2 * kBlkThreads / 16;   // slice chunks whose gain + noise a workgroup stages in one round
  const double t_tile = MR == 4 ? 0.46 : 0.65, chip_rate = 6.0e6, wave_rate = kPackTileBytes / t_tile;   // bytes per us
  const double bytes = (double)S.total_tiles * S.k_tiles * kPackTileBytes;
  int best_kr = 0, best_ph = 0, best_park = 0, best_mode = 0;
  double best_cost = 0;
  for (int kr = D; kr <= kt_pad && kr <= cpt_cap; kr += D) {
    if (g_blk_force_kr > 0 && kr != g_blk_force_kr) continue;
    const int n_seg = (int)ceil_div(S.k_tiles, kr);
    for (int ph = 1; ph <= 4; ++ph) {
      if (n_seg % ph != 0) continue;
      if (g_blk_force_phases > 0 && ph != g_blk_force_phases) continue;
      const int Sk = n_seg / ph;
      if (Sk > n_cons) continue;
      // a gate / up pair: finished inside one workgroup by two waves (K in one range), or by one wave that walks
      // both tiles over its K-range, with the shares of the ranges meeting in the workspace (one phase)
      const int mode = !pairs ? 0 : (Sk == 1 ? 1 : 2);
      if (mode == 2 && ph != 1) continue;
      const int per_range = n_cons / Sk;
      const int64_t slots_r = (int64_t)per_range * (mode == 1 ? kBlkWaves / 2 : kBlkWaves);
      const int64_t rounds = ceil_div(S.total_v, slots_r);
      if (ph > 1 && rounds > kBlkParkMax) continue;
      const int park = ph > 1 ? (int)rounds : (mode == 2 ? 1 : 0);
      {
        // the launch's LDS layout is the union of its stages': the parked accumulators and the pairs' hand-over of
        // ANOTHER stage take their room here as well
        const BlkLds l = blk_lds(M, MR, kr, norm, park, mode == 1);
        const size_t pe = l.park + l.exch > lds_floor_park_exch ? l.park + l.exch : lds_floor_park_exch;
        if (l.x + l.g + l.t + l.y + pe > kBlkLdsMax) continue;
      }
      const int64_t active = (S.total_v < slots_r ? S.total_v : slots_r) * Sk * (mode == 1 ? 2 : 1);
      const double rate = active * wave_rate < chip_rate ? active * wave_rate : chip_rate;
      const double extra = Sk > 1 ? 1.5 * Sk * S.total_tiles * 64.0 * MR * 4 : 0.0;   // partial tiles out and back
      double cost = (bytes + extra) / rate;
      const double chain = (double)rounds * ph * kr * t_tile * (mode == 2 ? 2 : 1);
      cost = cost > chain ? cost : chain;
      // measured: a further round of units 2 us, the exchange of a K split 6 us and more (a pair's: two shares, two
      // adapters' t, behind the slowest of the ranges: 22 us against 11 us for a second phase on the 32B pair at 16
      // tokens), a further phase 10 us
      cost += 2.0 * (rounds - 1) + (Sk > 1 ? (mode == 2 ? 20.0 : 6.0) + 0.25 * Sk : 0.0) + 10.0 * (ph - 1);
      if (best_kr == 0 || cost < best_cost - 1e-9) { best_kr = kr; best_ph = ph; best_park = park; best_cost = cost; best_mode = mode; }
    }
  }
  if (best_kr == 0) return QERL_ERR_SHAPE;
  S.kr_len = best_kr;
  S.phases = best_ph;
  S.Sk = (int)ceil_div(S.k_tiles, best_kr) / best_ph;
  S.per_range = n_cons / S.Sk;
  S.pairs = best_mode;
  *park_units = best_park;
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
  const int MR = a.M <= 8 ? 4 : 8;
  *MR_out = MR;
  a.n_wgs = g_blk_cus;
  int pmax = 0;
  for (int s = 0; s < a.n_stages; ++s) {
    BlkStage& S = a.st[s];
    int rt = 0;
    for (int i = 0; i < S.n_members; ++i) if (S.mem[i].r > 0) { S.mem[i].t_off = rt; rt += S.mem[i].r; } else S.mem[i].t_off = 0x7fffffff;
    for (int i = S.n_members; i < kMaxGroup; ++i) S.mem[i].t_off = 0x7fffffff;
    S.r_total = rt;
    S.n_producers = 0; S.prod_k = 1;
    if (rt > 0) {
      // one producer workgroup per pair of rank tiles (64 stacked rows) and run of K: every producer makes one round of
      // loads; runs of about five K-tiles, as many as the producer budget allows
      const int n_pairs = (int)ceil_div(rt, 64);
      int64_t pk = ceil_div(S.k_tiles, 5);
      const int64_t pk_max = kBlkMaxProducers / n_pairs;
      pk = pk < 1 ? 1 : (pk > pk_max ? pk_max : pk);
      S.prod_k = (int)pk;
      S.n_producers = (int)pk * n_pairs;
    }
    pmax = S.n_producers > pmax ? S.n_producers : pmax;
  }
  a.n_prod_max = pmax;
  const int n_cons = a.n_wgs - pmax;
  if (n_cons < 1) return QERL_ERR_SHAPE;
  size_t part = 0, ctrs = 0, prod_need = 0;
  BlkLds mx{};
  int park_max = 0;
  // Stages are planned one by one; if the union of their LDS needs does not fit, they are planned once more with
  // the largest parked-accumulator + hand-over area of the first attempt taken as given by every stage.
  size_t floor_pe = 0;
  for (int attempt = 0; attempt < 2; ++attempt) {
  part = 0; ctrs = 0; prod_need = 0; mx = BlkLds{}; park_max = 0;
  for (int s = 0; s < a.n_stages; ++s) {
    BlkStage& S = a.st[s];
    int park = 0;
    const int rc = plan_block_stage(S, a.M, MR, n_cons, floor_pe, &park);
    if (rc != QERL_OK) return rc;
    park_max = park > park_max ? park : park_max;
    const BlkLds l = blk_lds(a.M, MR, S.kr_len, S.gain != nullptr, park, S.pairs == 1);
    mx.x = l.x > mx.x ? l.x : mx.x; mx.g = l.g > mx.g ? l.g : mx.g; mx.t = l.t; mx.y = l.y;
    mx.park = l.park > mx.park ? l.park : mx.park; mx.exch = l.exch > mx.exch ? l.exch : mx.exch;
    S.ctr_off = (int)ctrs; S.partial_off = (int64_t)part;
    if (S.Sk > 1) { ctrs += (size_t)S.total_tiles; part += (size_t)S.Sk * S.total_tiles * 64 * MR; }
    if (S.n_producers > 0) {
      const int64_t steps = S.K / 16;
      S.prod_steps = (int)ceil_div(steps, S.prod_k);
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
  if (mx.x + mx.g + mx.t + mx.y + mx.park + (mx.exch > 0 ? mx.exch : 256) <= kBlkLdsMax || attempt == 1) break;
  floor_pe = mx.park + (mx.exch > 0 ? mx.exch : 256);
  }
#ifdef QERL_TUNING_HOOKS
  if (getenv("QERL_BLK_TRACE"))
    for (int s = 0; s < a.n_stages; ++s)
      fprintf(stderr, "block plan: M %d stage %d K-tiles %d tiles %d units %d  kr_len %d phases %d Sk %d per_range %d producers %d pairs %d\n", a.M, s,
              a.st[s].k_tiles, a.st[s].total_tiles, a.st[s].total_v, a.st[s].kr_len, a.st[s].phases, a.st[s].Sk, a.st[s].per_range, a.st[s].n_producers, a.st[s].pairs);
#endif
  a.park_units = park_max > 0 ? park_max : 1;
  a.g_lds_off = (int)mx.x;
  a.t_lds_off = a.g_lds_off + (int)mx.g;
  a.y_lds_off = a.t_lds_off + (int)mx.t;
  a.p_lds_off = a.y_lds_off + (int)mx.y;
  a.e_lds_off = a.p_lds_off + (int)mx.park;
  size_t total = (size_t)a.e_lds_off + (mx.exch > 0 ? mx.exch : 256);
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

// Every pointer the kernel dereferences and every bound its indexing assumes; QERL_OK if the launch is safe.
int check_block(const BlkArgs& a, size_t lds, int MR) {
  if (a.M < 1 || a.M > 16 || a.n_stages < 1 || a.n_stages > kBlkMaxStages || a.n_wgs < 2 || a.n_prod_max < 0 || a.n_prod_max >= a.n_wgs)
    return QERL_ERR_SHAPE;
  if (!a.ctl || !a.counters || !a.partial || !a.tpart || !a.tfinal) return QERL_ERR_NULL;
  const int MT = MR == 4 ? 8 : 16;
  if ((MR != 4 && MR != 8) || (a.M > 8 && MR != 8) || lds > kBlkLdsMax || a.g_lds_off <= 0 || a.t_lds_off < a.g_lds_off ||
      (size_t)a.y_lds_off < (size_t)a.t_lds_off + (size_t)kMaxGroup * 3 * MT * 64 * 2 || (size_t)a.p_lds_off < (size_t)a.y_lds_off + kBlkWaves * 16 * 32 * 2 ||
      a.park_units < 1 || a.e_lds_off < a.p_lds_off || (size_t)a.e_lds_off + 256 > lds)
    return QERL_ERR_SHAPE;
  bool any_phases = false, any_pairs = false;
  const int n_cons = a.n_wgs - a.n_prod_max;
  for (int s = 0; s < a.n_stages; ++s) {
    const BlkStage& S = a.st[s];
    if (!S.x || S.ldx < S.K || S.ldx % 8 != 0 || ((uintptr_t)S.x & 15) != 0 || S.K < 16 || S.K % 16 != 0) return QERL_ERR_ALIGN;
    if (S.k_tiles != (int)ceil_div(S.K, kPackTileK) || S.n_members < 1 || S.n_members > kMaxGroup) return QERL_ERR_SHAPE;
    const int64_t n_seg = (int64_t)S.Sk * S.phases;
    if (S.kr_len < kBlkD || S.kr_len % kBlkD != 0 || S.Sk < 1 || S.phases < 1 || S.phases > 4 || n_seg * S.kr_len < S.k_tiles || (n_seg - 1) * S.kr_len >= S.k_tiles ||
        S.per_range < 1 || (int64_t)S.per_range * S.Sk > n_cons || S.kr_len * 16 > 2 * kBlkThreads || (size_t)(a.M + 1) * (size_t)(S.kr_len * 256 + 16) > (size_t)a.g_lds_off ||
        false)
      return QERL_ERR_SHAPE;
    {
      const int64_t slots_r = (int64_t)S.per_range * (S.pairs == 1 ? kBlkWaves / 2 : kBlkWaves);
      if (S.phases > 1 && ceil_div(S.total_v, slots_r) > a.park_units) return QERL_ERR_SHAPE;
      if (S.pairs < 0 || S.pairs > 2 || (S.pairs == 1 && S.Sk != 1) || (S.pairs == 2 && S.phases != 1)) return QERL_ERR_SHAPE;
    }
    any_phases |= S.phases > 1; any_pairs |= S.pairs == 1;
    if (S.gain && (((uintptr_t)S.gain & 15) != 0 || ((uintptr_t)S.noise & 15) != 0 || S.K % 8 != 0)) return QERL_ERR_ALIGN;
    int tiles = 0;
    for (int i = 0; i < S.n_members; ++i) {
      const BlkMember& m = S.mem[i];
      if (!m.packed || !m.tensor_scale || m.N < 1 || m.n_tiles != (int)ceil_div(m.N, kPackTileRows) || m.tile_begin != tiles) return QERL_ERR_SHAPE;
      const bool row_major = m.stride_k == kPackTileBytes && m.stride_n == (int64_t)S.k_tiles * kPackTileBytes;
      const bool k_major = m.stride_n == kPackTileBytes && m.stride_k == (int64_t)m.n_tiles * kPackTileBytes;
#ifndef QERL_TUNING_HOOKS
      if (!row_major && !k_major) return QERL_ERR_SHAPE;
#else
      (void)row_major; (void)k_major;
#endif
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
      if (S.n_producers < 1 || S.n_producers > a.n_prod_max || S.n_producers > kBlkMaxProducers || S.r_total > 256 || S.r_total % 8 != 0 ||
          S.prod_k < 1 || S.n_producers != S.prod_k * (int)ceil_div(S.r_total, 64))
        return QERL_ERR_SHAPE;
      const size_t rows = (size_t)(S.r_total < 64 ? S.r_total : 64) + a.M + 1;
      if (S.prod_steps < 1 || S.prod_cb < 1 || S.prod_cb > kProdMaxSteps || (int64_t)S.prod_steps * S.prod_k < S.K / 16 ||
          rows * (size_t)(S.prod_cb * 32 + 16) > (size_t)S.prod_red_off ||
          (size_t)S.prod_red_off + lora_producer_red_bytes(kBlkWaves, MR) > lds)
        return QERL_ERR_SHAPE;
    } else if (S.n_producers != 0) {
      return QERL_ERR_SHAPE;
    }
  }
  if (any_phases && (size_t)a.p_lds_off + (size_t)kBlkWaves * a.park_units * 64 * MR * sizeof(float) > (size_t)a.e_lds_off) return QERL_ERR_SHAPE;
  if (any_pairs && (size_t)a.e_lds_off + 256 + (size_t)4 * 64 * MR * sizeof(float) > lds) return QERL_ERR_SHAPE;
  return QERL_OK;
}

int launch_block(const BlkArgs& a, size_t lds, int MR, hipStream_t st) {
  const int rc = check_block(a, lds, MR);
  if (rc != QERL_OK) return rc;
  return MR == 4 ? launch_block_t<4>(a, lds, st) : launch_block_t<8>(a, lds, st);
}

}  // namespace qerl

#ifdef QERL_TUNING_HOOKS   // built only for tuning sessions: they change process-wide state
extern "C" QERL_API void qerl_debug_force_block_kr(int kr, int phases) { qerl::g_blk_force_kr = kr; qerl::g_blk_force_phases = phases; }
#endif
#ifdef QERL_BLK_TRACE
extern "C" QERL_API int qerl_debug_read_block_trace(void* dst, size_t bytes) {
  return (int)hipMemcpyFromSymbol(dst, HIP_SYMBOL(qerl::g_blk_trace), bytes, 0, hipMemcpyDeviceToHost);
}
#endif
