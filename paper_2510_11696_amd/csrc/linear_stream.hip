// Streaming decode kernel (M <= 16 tokens) for one linear or a group of linears that share x
// (q/k/v, gate/up) on tile-packed NVFP4 weights, LoRA included, one launch.
//
//   y_g[m,n] = S32_g * sum_b s_g[n,b] * ( sum_{k in block b} x[m,k] * e_g[n,k] )           (Eq. 6)
//            + lora_scale_g * sum_j t_g[m,j] * B_g[n,j],      t_g = x A_g^T                 (Eq. 2)
//
// The op is bound by streaming 0.5625 B per weight from HBM once; at decode sizes the enemy
// is latency, not arithmetic.  So the kernel is persistent and keeps memory busy from the
// first cycle to the last:
//   * ~one workgroup per CU walks a list of units; a unit is one row-tile (32 output rows) over
//     the workgroup's K-range.  Seven "main" waves split the K-tiles of that range and stream
//     them through a ring of D tiles in registers that is refilled as it is consumed -- across
//     unit boundaries, so the next unit's weights are already in flight while this one is
//     being multiplied.  Nothing in their loop waits on anything but weight data and one
//     barrier per unit.
//   * The x slice of the K-range lives in LDS for the whole launch (rows padded by 32 bytes so
//     that the MFMA operand reads of 8..16 tokens hit distinct banks; tokens >= M read a zero
//     row), so any wave can work on any K-tile without holding x in registers.
//   * Arithmetic per 16-input scale block as in linear_decode.hip: bare E2M1 values into one
//     v_mfma_f32_32x32x16_bf16, then acc += E4M3 scale * product (one FMA per live token row).
//   * The eighth wave is the epilogue wave and runs one unit behind: it computes the LoRA
//     up-projection of the unit (B rows prefetched, fp32 t split into three bf16 terms, MFMAs
//     over j), and after the unit's barrier adds the seven partial tiles from LDS, applies S32,
//     and either stores y or -- when K is split over several workgroups because x does not fit
//     in LDS -- exchanges partial tiles through the workspace (agent-scope atomics, last one to
//     arrive adds them in range order).  Its stores and waits never stall the streaming waves.
//   * t = x A^T for all members comes from producer workgroups at the front of the grid, as in
//     linear_decode.hip (ready word, bounded wait, NaN on time-out).
// Results are bit-identical from call to call: every sum has a fixed order.
#include "linear.hpp"
#include "lora_producer.hpp"

namespace qerl {

constexpr int kStreamWaves = 8;             // 7 main + 1 epilogue
constexpr int kMainWaves = kStreamWaves - 1;
constexpr int kCtlArrive = 0, kCtlDone = 2;   // producers that have stored their partial t; consumers that have read it
constexpr uint32_t kStreamSpinLimit = 1u << 14;

__device__ __forceinline__ bf16x8 stream_e2m1x8(uint32_t codes) {
  const bf16x2 p0 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(codes, 1.0f, 0);
  const bf16x2 p1 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(codes, 1.0f, 1);
  const bf16x2 p2 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(codes, 1.0f, 2);
  const bf16x2 p3 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(codes, 1.0f, 3);
  u32x4 o = {__builtin_bit_cast(uint32_t, p0), __builtin_bit_cast(uint32_t, p1),
             __builtin_bit_cast(uint32_t, p2), __builtin_bit_cast(uint32_t, p3)};
  return __builtin_bit_cast(bf16x8, o);
}
// Optional timeline stamps for tuning (build with -DQERL_STREAM_TRACE): eight 100 MHz time stamps per wave
// of the first 512 workgroups, read back with qerl_debug_read_trace().
#ifdef QERL_STREAM_TRACE
__device__ unsigned long long g_trace[512 * 8 * 8];
#define QSTAMP(p) do { if (lane == 0 && blockIdx.x < 512) g_trace[((int)blockIdx.x * 8 + wave) * 8 + (p)] = wall_clock64(); } while (0)
#if QERL_STREAM_TRACE == 2   // start-up detail instead of the per-unit view
#define QTRACE(p) do { } while (0)
#define QSTART(p) QSTAMP(p)
#else
#define QTRACE(p) QSTAMP(p)
#define QSTART(p) do { } while (0)
#endif
#else
#define QTRACE(p) do { } while (0)
#define QSTART(p) do { } while (0)
#endif

// ---- producers: t = x Astack^T for the stacked A of all members (lora_producer.hpp) ------------------
template <int MR, bool GATED>
__device__ __forceinline__ void stream_producer(const StreamArgs& a, unsigned char* smem) {
  LoraProducerArgs p;
  p.x = a.x; p.ldx = a.ldx; p.x2 = a.x2; p.ldx2 = a.ldx2;
  p.M = a.M; p.K = a.K; p.r_total = a.r_total; p.n_members = a.n_members;
#pragma unroll
  for (int i = 0; i < kMaxGroup; ++i) { p.A[i] = a.mem[i].A; p.t_off[i] = a.mem[i].t_off; }
  p.index = (int)blockIdx.x; p.only_pair = -1; p.n_arrivals = 0; p.n_k = 0; p.tfinal = nullptr; p.ready = nullptr;
  p.prod_steps = a.prod_steps; p.prod_cb = a.prod_cb; p.prod_red_off = a.prod_red_off;
  p.tpart = a.tpart; p.arrive = a.lora_ctl + kCtlArrive;
  p.gain = nullptr; p.noise = nullptr; p.rstd = nullptr;
  lora_producer<MR, GATED ? 1 : 0, kStreamWaves>(p, smem);
}

struct StreamTile { u32x4 c0, c1; u32x2 sc; };

constexpr int kRedBufs = 4;                // partial-tile buffers between the main waves and the epilogue wave (at most; 2 when LDS is short)
constexpr int kLoraSteps = 4;               // 16-wide j steps of the up-projection (r <= 64)
constexpr int kMaxPending = 4;              // units an epilogue wave can park while t is not ready (at most; 2 when LDS is short)

// TIGHT: two reduction buffers and parking slots instead of four, B fragments parked for the adapters' actual
// rank only (the LDS budget of 16 tokens with K = 3584 in one range)
template <int MR, int D, bool TIGHT, bool GATED>
__global__ __launch_bounds__(kStreamWaves * 64) void stream_kernel(const StreamArgs a) {
  // x slice [M (+ 1 zero) rows][xs_stride bytes], red[red_bufs][7][64][MR] floats, parked units, t of a member.  The alignment matters:
  // 16-byte LDS accesses from a misaligned base run several times slower.
  extern __shared__ __attribute__((aligned(256))) unsigned char smem[];
  __shared__ StreamMember s_mem[kMaxGroup];
  __shared__ int s_prod[kRedBufs], s_cons; // per buffer: main waves that have written their partial tile; units taken over by the epilogue wave
  float* red = reinterpret_cast<float*>(smem + a.red_off);
  // grid: the producers, then the consumers range by range: exactly the workgroups that have work, so that
  // all of them are resident from the start (one per CU)
  if ((int)blockIdx.x < a.n_producers) {
    stream_producer<MR, GATED>(a, smem);
    return;
  }
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps everything derived from it in SGPRs
  const int n32 = lane & 31, kg = lane >> 5;
  QTRACE(0);
  QSTART(0);
  // units u0 .. u0 + n_units - 1 of K-range `range` are this workgroup's
  const int cid = (int)blockIdx.x - a.n_producers;
  const int range = cid / a.per_range, ci = cid - range * a.per_range;
  const int n_units = a.units_base + (ci < a.units_rem ? 1 : 0);
  const int u0 = ci * a.units_base + (ci < a.units_rem ? ci : a.units_rem);   // consecutive row-tiles: mostly one member per workgroup
  const int kr_len = a.kr_len;            // K-tiles per range
  const int kr0 = range * kr_len, kr1 = (kr0 + kr_len < a.k_tiles) ? kr0 + kr_len : a.k_tiles;
  // unused entries of the member table start at INT_MAX
  auto member_index = [&](int nt) { return (nt >= a.tb1 ? 1 : 0) + (nt >= a.tb2 ? 1 : 0) + (nt >= a.tb3 ? 1 : 0); };

  // ---- staging of the x slice of this K-range into LDS, all eight waves: thread -> 16-byte chunk column,
  // all tokens of a column loaded before any is stored
  constexpr int MT = MR == 4 ? 8 : 16;
  constexpr int kThreads = kStreamWaves * 64;
  const int chunks_per_row = (kr1 - kr0) * 16;
  auto xload = [&](int ch, u32x4 (&xv)[MT]) {
    const int64_t k = (int64_t)kr0 * 128 + ch * 8;
#pragma unroll
    for (int tok = 0; tok < MT; ++tok) {
      xv[tok] = u32x4{0u, 0u, 0u, 0u};
      if (tok < a.M && ch < chunks_per_row && k < a.K) xv[tok] = *reinterpret_cast<const u32x4*>(a.x + (int64_t)tok * a.ldx + k);
    }
    if constexpr (GATED) {               // gated input: the second operand, then the product in place
      u32x4 uv[MT];
#pragma unroll
      for (int tok = 0; tok < MT; ++tok) {
        uv[tok] = u32x4{0u, 0u, 0u, 0u};
        if (tok < a.M && ch < chunks_per_row && k < a.K) uv[tok] = *reinterpret_cast<const u32x4*>(a.x2 + (int64_t)tok * a.ldx2 + k);
      }
#pragma unroll
      for (int tok = 0; tok < MT; ++tok) xv[tok] = silu_mul8(xv[tok], uv[tok]);
    }
  };
  auto xstore = [&](int ch, const u32x4 (&xv)[MT]) {
    if (ch < chunks_per_row) {
#pragma unroll
      for (int tok = 0; tok < MT; ++tok)
        if (tok < a.M) *reinterpret_cast<u32x4*>(smem + tok * a.xs_stride + ch * 16) = xv[tok];
      if (!TIGHT) *reinterpret_cast<u32x4*>(smem + a.M * a.xs_stride + ch * 16) = u32x4{0u, 0u, 0u, 0u};   // the zero row
    }
  };
  u32x4 xv[MT];
  int ch0 = 0;
  for (; chunks_per_row - ch0 > kThreads; ch0 += kThreads) {   // K-ranges beyond 4096 inputs: all but the last batch
    xload(ch0 + tid, xv);
    xstore(ch0 + tid, xv);
  }
  QSTART(1);
  xload(ch0 + tid, xv);
  QSTART(2);
  if (tid < kRedBufs) s_prod[tid] = 0;
  if (tid == 0) s_cons = 0;

  // ---- what the epilogue wave reads from memory: requested ahead, because a load of that wave queues behind
  // the whole weight ring of its CU, a latency it must never wait out between one barrier and the next.
  constexpr int red_bufs = TIGHT ? 2 : kRedBufs, max_pending = TIGHT ? 2 : kMaxPending;
  const int pend_steps = TIGHT ? a.pend_steps : kLoraSteps;
  const bool lora_range = range == 0 && a.any_lora != 0;   // only the first K-range adds the LoRA branch
  const bool bias_range = range == 0 && a.any_bias != 0;   // ... and the bias
  // B rows (32 rows x r of the unit's member): one unit ahead, parked with the unit's sums
  u32x4 bnext[kLoraSteps];
  auto request_b = [&](int u) {
#pragma unroll
    for (int s = 0; s < kLoraSteps; ++s) bnext[s] = u32x4{0u, 0u, 0u, 0u};
    if (u < n_units && lora_range) {
      const int nt = u0 + u;
      const StreamMember mem = s_mem[member_index(nt)];
      if (mem.r > 0) {
        int64_t brow = (int64_t)(nt - mem.tile_begin) * 32 + n32;
        brow = brow < mem.N ? brow : mem.N - 1;
#pragma unroll
        for (int s = 0; s < kLoraSteps; ++s) {
          const int j0 = 16 * s + 8 * kg;
          if (j0 < mem.r) bnext[s] = *reinterpret_cast<const u32x4*>(mem.B + brow * mem.r + j0);
        }
      }
    }
  };
  // partial sums of t: the first eight parts of 64 groups of four ranks (all there is for 8 tokens x rank 32)
  f32x4 tq[8];
  int tq_member = -1;
  auto request_t = [&](int mi, int e0, int p0) {
    const StreamMember mem = s_mem[mi];
    const int r = mem.r, r4 = r >> 2, n4 = a.M * r4;
    const float* src = mem.t_ext ? mem.t_ext : reinterpret_cast<const float*>(a.tpart) + mem.t_off;
    const int n_parts = mem.t_ext ? QERL_T_PARTS : a.n_producers;
    const int64_t row_stride = mem.t_ext ? r : a.r_total;
    const int64_t part_stride = mem.t_ext ? (int64_t)a.M * r : (int64_t)kTpartTokens * a.r_total;
    const int e = e0 + lane, tok = e / r4, j4 = e - tok * r4;
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      tq[b] = f32x4{0.f, 0.f, 0.f, 0.f};
      if (e < n4 && p0 + b < n_parts)
        tq[b] = *reinterpret_cast<const f32x4*>(src + (p0 + b) * part_stride + tok * row_stride + 4 * j4);
    }
  };
  // Every wave of this CU has queued its x loads before any weight load is queued behind them: without
  // this, x for the last waves would arrive after the whole first ring of all waves.
  __builtin_amdgcn_s_barrier();
  QSTART(3);

  if (wave < kMainWaves) {
    // ---- main wave: my K-tiles of every unit
    const int lw = (kr1 - kr0 + kMainWaves - 1) / kMainWaves;
    const int kt0 = kr0 + wave * lw;
    int kt1 = kt0 + lw;
    kt1 = kt1 < kr1 ? kt1 : kr1;
    const bool have = kt0 < kt1;
    StreamTile ring[D];
    int lu = 0, lk = kt0;                 // load cursor (unit, K-tile)
    // Address of the load cursor's unit (its K-tile 0), looked up once per unit, not per tile.  Past the end
    // of this wave's sequence the cursor parks on the first tile of the group: every call of issue() still
    // issues exactly three loads (cache hits that are never used), so that with a fixed number of loads in
    // flight the wait before a slot is consumed covers that slot only, not the whole ring.
    const uint8_t* ubase;
    int kmul;
    auto set_unit = [&]() {
      const bool live = have && lu < n_units;
      const int nt = live ? u0 + lu : 0;
      int tb = 0;
      const uint8_t* mp = a.mp0;
      if (nt >= a.tb1) { tb = a.tb1; mp = a.mp1; }
      if (nt >= a.tb2) { tb = a.tb2; mp = a.mp2; }
      if (nt >= a.tb3) { tb = a.tb3; mp = a.mp3; }
      ubase = mp + (live ? (int64_t)(nt - tb) * a.k_tiles * kPackTileBytes : 0);
      kmul = live ? kPackTileBytes : 0;
    };
    set_unit();
    auto issue = [&](StreamTile& t) {
      const uint8_t* base = ubase + (int64_t)lk * kmul;
      t.c0 = *reinterpret_cast<const u32x4*>(base + lane * 16);
      t.c1 = *reinterpret_cast<const u32x4*>(base + 1024 + lane * 16);
      t.sc = *reinterpret_cast<const u32x2*>(base + 2048 + n32 * 8);
      if (++lk == kt1) { lk = kt0; ++lu; set_unit(); }
    };
#pragma unroll
    for (int d = 0; d < D; ++d) issue(ring[d]);
    QSTART(4);
    xstore(ch0 + tid, xv);                // waits for x only: the ring stays in flight
    QSTART(5);
    __syncthreads();
    QSTART(6);
    QTRACE(1);

    // MFMA rows beyond the tokens read a zero row (all-zero operand rows also keep the matrix unit's power
    // down: measurably faster than feeding it copies of a real row).  Where LDS is short there is none and
    // they read the last token's row: an output row depends on its own input row only, and rows >= M are
    // never stored, so any data will do there.
    const int xrow = n32 < a.M ? n32 : (TIGHT ? a.M - 1 : a.M);
    const unsigned char* xbase = smem + xrow * a.xs_stride + kg * 16;
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    float acc[MR];
#pragma unroll
    for (int q = 0; q < MR; ++q) acc[q] = 0.f;
    int cu = 0, ck = kt0;                 // compute cursor
    // (a wave without K-tiles in this range has nothing to add: the epilogue wave counts the live ones only)
    // Ring slot d always holds tiles d, d + D, d + 2D, ... of this wave's sequence, so every slot is a fixed
    // set of registers.  Past the end of the sequence only the arithmetic is skipped: the refill still runs,
    // which keeps the number of loads in flight the same on every path.
    const int n_seq = have ? n_units * (kt1 - kt0) : 0;
    for (int i0 = 0; i0 < n_seq; i0 += D) {
#pragma unroll
      for (int d = 0; d < D; ++d) {
        if (i0 + d < n_seq) {
        const StreamTile& t = ring[d];
        const unsigned char* xk = xbase + (ck - kr0) * 256;
        f32x16 tmp[2];
        tmp[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(xk)),
                                                         stream_e2m1x8(t.c0[0]), zero, 0, 0, 0);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          // the product of the next scale block is on its way while this one is scaled and added
          if (j + 1 < 8) {
            const bf16x8 xa = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>(xk + (j + 1) * 32));
            const bf16x8 w = stream_e2m1x8(j + 1 < 4 ? t.c0[(j + 1) & 3] : t.c1[(j + 1) & 3]);
            tmp[(j + 1) & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa, w, zero, 0, 0, 0);
          }
          const float s = e4m3_byte_f32(t.sc[j >> 2], j & 3);
#pragma unroll
          for (int q = 0; q < MR; ++q) acc[q] = __builtin_fmaf(s, tmp[j & 1][q], acc[q]);
        }
        // The refill must stay below the last use of the slot: otherwise the incoming data needs other
        // registers, and moving them back at the loop end costs a wait for everything in flight.  The empty
        // asm pins the accumulators (and with them every use of the slot) above this point.
#pragma unroll
        for (int q = 0; q < MR; ++q) asm volatile("" : "+v"(acc[q]));
        }
        __builtin_amdgcn_sched_barrier(0);
        issue(ring[d]);                   // refill the slot in place (same registers), D tiles ahead
        if (i0 + d < n_seq && ++ck == kt1) {
          if (cu < n_units) {
            // Unit finished: hand the partial tile to the epilogue wave through one of kRedBufs buffers and
            // go on.  No barrier: the waves of a workgroup drift apart freely, and only a buffer that the
            // epilogue wave has not taken over yet (it is kRedBufs units behind) makes this wave wait.
            if (cu >= red_bufs) {
              while (__hip_atomic_load(&s_cons, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) < cu - red_bufs + 1)
                __builtin_amdgcn_s_sleep(1);
            }
            float* slot = red + (((cu % red_bufs) * kMainWaves + wave) * 64 + lane) * MR;
#pragma unroll
            for (int q = 0; q < MR; q += 4) {
              *reinterpret_cast<f32x4*>(slot + q) = f32x4{acc[q], acc[q + 1], acc[q + 2], acc[q + 3]};
              acc[q] = 0.f; acc[q + 1] = 0.f; acc[q + 2] = 0.f; acc[q + 3] = 0.f;
            }
            QTRACE(2 + (cu < 4 ? cu : 4));
            if (lane == 0) __hip_atomic_fetch_add(&s_prod[cu % red_bufs], 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
            ++cu;
          }
          ck = kt0;
        }
      }
    }
    QTRACE(7);
    return;
  }

  // ---- epilogue wave -----------------------------------------------------------------------------
  // It looks members up by a computed index.  Indexing the kernel arguments that way would be a vector load
  // from memory per field and unit, each waiting for its turn behind the weight ring; so the table is copied
  // to LDS once (constant indices: scalar loads) and read from there.
  if (lane == 0) {
#pragma unroll
    for (int i = 0; i < kMaxGroup; ++i) s_mem[i] = a.mem[i];
  }
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  // first requests while the main waves are still queueing their ring: B of the first unit, and t if it was
  // computed before the launch
  request_b(0);
  if (n_units > 0 && lora_range) {
    const int m0 = member_index(u0);
    if (s_mem[m0].r > 0 && s_mem[m0].t_ext) { request_t(m0, 0, 0); tq_member = m0; }
  }
  // Two steps per unit, each written once: receive (barrier, add the seven partial tiles, park the sums and
  // the unit's B fragments in LDS) and finalize (LoRA up-projection, K-range exchange, store).  Finalizing
  // trails receiving by up to kMaxPending units, which is how the wave rides out the time until t is ready
  // without holding up the streaming waves.
  xstore(ch0 + tid, xv);
  __syncthreads();
  QTRACE(1);
  // This wave shares its SIMD with a streaming wave whose conversion arithmetic would otherwise take every
  // other issue slot: its work per unit is small, and whatever it has not finished when the streaming waves
  // are done is the tail of the launch.
  __builtin_amdgcn_s_setprio(3);

  // tensor scales of all members up front: no memory round trip between a unit's barrier and its stores
  float S32m[kMaxGroup];
#pragma unroll
  for (int i = 0; i < kMaxGroup; ++i) S32m[i] = i < a.n_members ? *a.mem[i].tensor_scale : 0.f;

  const int lw_e = (kr1 - kr0 + kMainWaves - 1) / kMainWaves;
  const int n_live = lw_e > 0 ? (kr1 - kr0 + lw_e - 1) / lw_e : 0;   // main waves that have K-tiles in this range
  u32x4 th[kLoraSteps], tm[kLoraSteps], tl[kLoraSteps];
  int t_member = -1;                      // member whose split t is in th/tm/tl
  bool poisoned = false, t_ready = a.n_producers == 0;
  float* pend_base = reinterpret_cast<float*>(smem + a.pend_off);          // [max_pending][MR][64]
  u32x4* pend_b = reinterpret_cast<u32x4*>(smem + a.pend_off + max_pending * MR * 64 * 4);   // [max_pending][pend_steps][64]
  int u_recv = 0, u_done = 0;             // units received / finalized so far
  int b_wanted = -1;                      // unit whose B rows are to be requested next
  // t of member mi: its partial sums (QERL_T_PARTS slices of K computed before the launch, or the producers'
  // partials of this launch) are fetched by the whole wave in one round of loads -- element groups of four,
  // all parts of a group in flight together -- added in part order, and left in LDS as [token][rank]; from
  // there each lane takes its MFMA operand rows and splits the fp32 values into three bf16 terms (exact to
  // 2^-24 relative).  The partials were written through to memory before this wave looks (kernel boundary, or
  // the producers' count followed by an agent-scope acquire fence): ordinary loads suffice.
  float* tsum = reinterpret_cast<float*>(smem + a.tsum_off);               // [M][r] of the current member
  uint16_t* ytile = reinterpret_cast<uint16_t*>(smem + a.tsum_off + 16 * 64 * 4);   // [16 tokens][32 rows] bf16, output staging
  auto load_t = [&](int mi) {
    const StreamMember mem = s_mem[mi];
    const int r = mem.r, r4 = r >> 2, n4 = a.M * r4;                        // groups of four ranks
    const int n_parts = mem.t_ext ? QERL_T_PARTS : a.n_producers;
    for (int e0 = 0; e0 < n4; e0 += 64) {                                   // one group per lane and round
      f32x4 sum = {0.f, 0.f, 0.f, 0.f};
      for (int p0 = 0; p0 < n_parts; p0 += 8) {
        if (!(tq_member == mi && e0 == 0 && p0 == 0)) request_t(mi, e0, p0);   // else: requested at kernel start
        tq_member = -1;
#pragma unroll
        for (int b = 0; b < 8; ++b) sum += tq[b];
      }
      if (e0 + lane < n4) *reinterpret_cast<f32x4*>(tsum + 4 * (e0 + lane)) = sum;
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // this wave's LDS writes are done before it reads them back
#pragma unroll
    for (int s = 0; s < kLoraSteps; ++s) {
      const int j0 = 16 * s + 8 * kg;
      float tv[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) tv[i] = 0.f;
      if (n32 < a.M && j0 < r) {
        const f32x4 t0 = *reinterpret_cast<const f32x4*>(tsum + n32 * r + j0);
        const f32x4 t1 = *reinterpret_cast<const f32x4*>(tsum + n32 * r + j0 + 4);
        tv[0] = t0[0]; tv[1] = t0[1]; tv[2] = t0[2]; tv[3] = t0[3];
        tv[4] = t1[0]; tv[5] = t1[1]; tv[6] = t1[2]; tv[7] = t1[3];
        if (poisoned) tv[0] = __uint_as_float(0x7fc00000u);   // the hand-over timed out: make it visible
      }
      split3_bf16(tv, th[s], tm[s], tl[s]);
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // ... and read before the next member overwrites them
    t_member = mi;
  };

  while (u_done < n_units) {
    if (b_wanted >= 0) { request_b(b_wanted); b_wanted = -1; }
    if (u_recv < n_units && u_recv - u_done < max_pending) {
      // ---- receive unit u_recv
      const int u = u_recv, slot = u % max_pending;
      const int nt = u0 + u;
      const int mi = member_index(nt);
      QTRACE(2 + (u < 4 ? u : 4));
      const int rb = u % red_bufs;
      while (__hip_atomic_load(&s_prod[rb], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) < n_live)
        __builtin_amdgcn_s_sleep(1);      // the live waves' partial tiles of unit u are in red[u % red_bufs]
      if (lora_range) {
#pragma unroll
        for (int s = 0; s < kLoraSteps; ++s)
          if (s < pend_steps) pend_b[(slot * pend_steps + s) * 64 + lane] = bnext[s];
        b_wanted = u + 1;                 // requested at the end of this round: nothing finalize waits for may queue behind it
      }
      float S32 = S32m[0];
#pragma unroll
      for (int i = 1; i < kMaxGroup; ++i) S32 = mi == i ? S32m[i] : S32;
      {
        f32x4 part[kMainWaves][MR / 4];
#pragma unroll
        for (int w = 0; w < kMainWaves; ++w)
#pragma unroll
          for (int q4 = 0; q4 < MR / 4; ++q4) {
            part[w][q4] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (w < n_live) part[w][q4] = *reinterpret_cast<const f32x4*>(red + ((rb * kMainWaves + w) * 64 + lane) * MR + 4 * q4);
          }
#pragma unroll
        for (int q = 0; q < MR; ++q) {
          float sum = 0.f;
#pragma unroll
          for (int w = 0; w < kMainWaves; ++w) sum += part[w][q >> 2][q & 3];
          pend_base[(slot * MR + q) * 64 + lane] = sum * S32;
        }
      }
      // the buffer may be written again (its reads above have returned: the sums were formed from them);
      // its counter goes back to zero before the main waves are told
      if (lane == 0) {
        __hip_atomic_store(&s_prod[rb], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        __hip_atomic_store(&s_cons, u + 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
      }
      ++u_recv;
    }
    // ---- finalize the oldest received unit, if it can be
    const int u = u_done, slot = u % max_pending;
    const int nt = u0 + u;
    const int mi = member_index(nt);
    const StreamMember mem = s_mem[mi];
    const bool needs_lora = lora_range && mem.r > 0;
    if (needs_lora && !t_ready && !mem.t_ext) {
      const bool can_receive_more = u_recv < n_units && u_recv - u_done < max_pending;
      uint32_t spins = 0;
      for (;;) {
        if (__hip_atomic_load(a.lora_ctl + kCtlArrive, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == (uint32_t)a.n_producers) {
          t_ready = true;
          break;
        }
        if (can_receive_more) break;      // one look per unit while there is streaming to attend to
        if (++spins > kStreamSpinLimit) {   // bounded: poison the output and leave word in the workspace
          poisoned = true; t_ready = true;
          if (lane == 0) __hip_atomic_fetch_or(a.lora_ctl + kCtlErr, 4u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          break;
        }
        __builtin_amdgcn_s_sleep(32);
      }
      if (!t_ready) continue;
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");   // the producers' partials were written by other workgroups: once per launch
      QTRACE(6);
    }
    // the bias of this lane's output row, requested before the LoRA arithmetic that hides its latency; the
    // first K-range carries it
    uint16_t bias_bits = 0;
    if (bias_range) {
      const int64_t nb_row = (int64_t)(nt - mem.tile_begin) * 32 + n32;
      if (mem.bias && nb_row < mem.N) bias_bits = mem.bias[nb_row];
    }
    float out[MR];
#pragma unroll
    for (int q = 0; q < MR; ++q) out[q] = pend_base[(slot * MR + q) * 64 + lane];
    if (needs_lora) {
      if (t_member != mi) load_t(mi);
      f32x16 lh, lm, ll;                  // one chain per bf16 term of t: independent MFMAs back to back
#pragma unroll
      for (int i = 0; i < 16; ++i) { lh[i] = 0.f; lm[i] = 0.f; ll[i] = 0.f; }
#pragma unroll
      for (int s = 0; s < kLoraSteps; ++s) {
        if (16 * s < mem.r) {
          const bf16x8 bf = __builtin_bit_cast(bf16x8, pend_b[(slot * pend_steps + s) * 64 + lane]);
          lh = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, th[s]), bf, lh, 0, 0, 0);
          lm = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, tm[s]), bf, lm, 0, 0, 0);
          ll = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, tl[s]), bf, ll, 0, 0, 0);
        }
      }
#pragma unroll
      for (int q = 0; q < MR; ++q) out[q] += ((lh[q] + lm[q]) + ll[q]) * mem.lora_scale;
    }
    if (bias_range) {
      const float bias = bf16_bits_to_f32(bias_bits);   // +0 for a member without one
#pragma unroll
      for (int q = 0; q < MR; ++q) out[q] += bias;
    }
    ++u_done;
    // out = this range's share of tile nt.  With several K-ranges it goes to the workspace as it is
    // ([range][tile][lane][MR] fp32) and stream_reduce_kernel, launched behind this kernel, adds the ranges in
    // order and stores y: no workgroup ever waits for another one's range.
    if (a.Sk > 1) {
      float* mine = reinterpret_cast<float*>(a.partial) + (((int64_t)range * a.total_tiles + nt) * 64 + lane) * MR;
#pragma unroll
      for (int q4 = 0; q4 < MR / 4; ++q4)
        *reinterpret_cast<f32x4*>(mine + 4 * q4) = f32x4{out[4 * q4], out[4 * q4 + 1], out[4 * q4 + 2], out[4 * q4 + 3]};
      continue;
    }
    const int64_t n0 = (int64_t)(nt - mem.tile_begin) * 32;
    if (mem.y_vec && n0 + 32 <= mem.N) {
      // Whole tile, 16-byte aligned rows: transpose through LDS so that the tile leaves in ONE store
      // instruction (16 bytes per lane) -- every vector memory instruction of this wave waits for its turn
      // behind the main waves' weight loads.
#pragma unroll
      for (int q = 0; q < MR; ++q) {
        const int tok = 8 * (q >> 2) + 4 * kg + (q & 3);
        ytile[tok * 32 + n32] = (uint16_t)f32_to_bf16_bits(out[q]);
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      const int tok = lane >> 2, part = lane & 3;
      if (tok < a.M) {
        const u32x4 v = *reinterpret_cast<const u32x4*>(ytile + tok * 32 + part * 8);
        *reinterpret_cast<u32x4*>(mem.y + (int64_t)tok * mem.ldy + n0 + part * 8) = v;
      }
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // read before the next unit overwrites the tile
    } else {
#pragma unroll
      for (int q = 0; q < MR; ++q) {
        const int tok = 8 * (q >> 2) + 4 * kg + (q & 3);
        if (tok < a.M && n0 + n32 < mem.N) mem.y[(int64_t)tok * mem.ldy + n0 + n32] = (uint16_t)f32_to_bf16_bits(out[q]);
      }
    }
  }
  QTRACE(7);
  // every first-range workgroup reports in once all producers have been counted; the last one re-arms the
  // control words
  if (a.n_producers > 0 && range == 0 && lane == 0) {
    if (!t_ready) {   // a workgroup without LoRA units still has to count, after the hand-over is complete
      uint32_t spins = 0;
      while (__hip_atomic_load(a.lora_ctl + kCtlArrive, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != (uint32_t)a.n_producers) {
        if (++spins > kStreamSpinLimit) { __hip_atomic_fetch_or(a.lora_ctl + kCtlErr, 4u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); break; }
        __builtin_amdgcn_s_sleep(32);
      }
    }
    // (after a wait that gave up the words stay as they are: a late producer may still count, and the sticky word
    // tells the host that the workspace has to be initialised again)
    const uint32_t old = __hip_atomic_fetch_add(a.lora_ctl + kCtlDone, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (old == (uint32_t)(a.per_range - 1) && __hip_atomic_load(a.lora_ctl + kCtlErr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u) {
      __hip_atomic_store(a.lora_ctl + kCtlArrive, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(a.lora_ctl + kCtlDone, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

// Second kernel of a launch with several K-ranges: y tile = sum over ranges, in range order, of the
// partial tiles the epilogue waves left in the workspace.  One wave per row-tile.
struct ReduceMember { uint16_t* y; int64_t ldy; int64_t N; int tile_begin; };
struct ReduceArgs { const float* partial; int M, Sk, total_tiles; ReduceMember mem[kMaxGroup]; };

template <int MR>
__global__ __launch_bounds__(256) void stream_reduce_kernel(const ReduceArgs a) {
  const int lane = threadIdx.x & 63;
  const int nt = blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  if (nt >= a.total_tiles) return;
  int mi = 0;
#pragma unroll
  for (int i = 1; i < kMaxGroup; ++i) mi = nt >= a.mem[i].tile_begin ? i : mi;
  const float* p = a.partial + ((int64_t)nt * 64 + lane) * MR;
  const int64_t stride = (int64_t)a.total_tiles * 64 * MR;
  f32x4 acc[MR / 4];
#pragma unroll
  for (int q4 = 0; q4 < MR / 4; ++q4) acc[q4] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int z0 = 0; z0 < a.Sk; z0 += 4) {      // four ranges in flight, added in range order
    f32x4 v[4][MR / 4];
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int q4 = 0; q4 < MR / 4; ++q4) {
        v[b][q4] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (z0 + b < a.Sk) v[b][q4] = *reinterpret_cast<const f32x4*>(p + (int64_t)(z0 + b) * stride + 4 * q4);
      }
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
      for (int q4 = 0; q4 < MR / 4; ++q4) acc[q4] += v[b][q4];
  }
  uint16_t* y = a.mem[0].y; int64_t ldy = a.mem[0].ldy, N = a.mem[0].N; int tb = a.mem[0].tile_begin;
#pragma unroll
  for (int i = 1; i < kMaxGroup; ++i)
    if (mi == i) { y = a.mem[i].y; ldy = a.mem[i].ldy; N = a.mem[i].N; tb = a.mem[i].tile_begin; }
  const int n32 = lane & 31, kg = lane >> 5;
  const int64_t n = (int64_t)(nt - tb) * 32 + n32;
#pragma unroll
  for (int q = 0; q < MR; ++q) {
    const int tok = 8 * (q >> 2) + 4 * kg + (q & 3);
    if (tok < a.M && n < N) y[(int64_t)tok * ldy + n] = (uint16_t)f32_to_bf16_bits(acc[q >> 2][q & 3]);
  }
}

// ---- host ------------------------------------------------------------------------------------------

static int g_force_ranges = 0;
static int g_force_depth = 0;

// LDS layout for M tokens of a K-range of kr_len K-tiles: x slice, reduction buffers, the parking area of
// the epilogue wave (sums always; B fragments for `steps` 16-rank steps with LoRA), t of a member.  `roomy`:
// four reduction buffers and four parking slots; otherwise two of each (the main waves and the epilogue wave
// are then coupled more tightly), which is what lets 16 tokens of K = 3584 fit without splitting K.
struct StreamLds { int kr_len, xs_stride, red_off, pend_off, tsum_off, red_bufs, max_pending, pend_steps; size_t total; };
static StreamLds stream_lds(int M, int kr_len, int MR, int steps, bool roomy) {
  StreamLds l{};
  l.kr_len = kr_len;
  l.red_bufs = roomy ? kRedBufs : 2; l.max_pending = roomy ? kMaxPending : 2;
  l.pend_steps = roomy ? (steps > 0 ? kLoraSteps : 0) : steps;
  steps = l.pend_steps;
  l.xs_stride = kr_len * 256 + 16;   // rows 16 bytes apart in bank space: the token rows read conflict-free
  const size_t xs = (size_t)(M + (roomy ? 1 : 0)) * (size_t)l.xs_stride;   // + the zero row
  l.red_off = (int)((xs + 255) & ~(size_t)255);
  const size_t red_consumer = (size_t)l.red_bufs * kMainWaves * MR * 64 * sizeof(float);
  l.pend_off = l.red_off + (int)red_consumer;
  const size_t pend = (size_t)l.max_pending * (MR * 64 * sizeof(float) + (size_t)steps * 64 * 16);
  l.tsum_off = l.pend_off + (int)pend;
  const size_t tsum = (size_t)16 * 64 * sizeof(float) + 16 * 32 * 2;               // t of one member (up to 16 tokens x 64 ranks); output tile staging
  l.total = l.tsum_off + tsum;
  return l;
}

constexpr size_t kStreamLdsMax = 160 * 1024 - 512;   // the static flag word takes one aligned slot of the CU's 160 KiB

int plan_stream(StreamArgs& a, size_t* lds_bytes, int* MR_out) {
  const int MR = a.M <= 8 ? 4 : 8;
  *MR_out = MR;
  int r_max = 0;
  for (int i = 0; i < a.n_members; ++i) r_max = a.mem[i].r > r_max ? a.mem[i].r : r_max;
  const int steps = (int)ceil_div(r_max, 16);             // B fragments parked per unit: 16 ranks each
  const size_t lds_cap = kStreamLdsMax - 2048;
  auto layout = [&](int kr_len) {                          // the roomy layout if it fits
    const StreamLds l = stream_lds(a.M, kr_len, MR, steps, true);
    return l.total <= lds_cap ? l : stream_lds(a.M, kr_len, MR, steps, false);
  };
  // Number of K-ranges: at least what makes the x slice fit, and beyond that whatever gives the shortest
  // critical path -- tiles a main wave multiplies one after the other (about half a microsecond each), plus
  // the second launch that adds the ranges' partial tiles once K is split at all.  A unit cannot take less
  // than the epilogue wave needs to collect it.  Never more
  // ranges than K-tiles / 7: the workspace is sized for that, and a range should feed seven waves.
  const int sk_limit = (int)ceil_div(a.k_tiles, kMainWaves);
  const int cus = 256 - a.n_producers;   // one workgroup per CU (the register use allows no second one), producers included
  const double epilogue_us = MR == 4 ? 0.6 : 1.0;
  int best = 0;
  double best_cost = 0;
  for (int Sk = 1; Sk <= sk_limit; ++Sk) {
    const int kr_len = (int)ceil_div(a.k_tiles, Sk);
    if (layout(kr_len).total > lds_cap) continue;
    if (g_force_ranges > 0 && Sk != g_force_ranges) continue;
    int64_t per_range = cus / Sk;
    if (per_range < 1) break;
    if (per_range > a.total_tiles) per_range = a.total_tiles;
    const int64_t units = ceil_div(a.total_tiles, per_range), lw = ceil_div(kr_len, kMainWaves);
    const double per_unit = 0.5 * (double)lw > epilogue_us ? 0.5 * (double)lw : epilogue_us;
    const double cost = (double)units * per_unit + (Sk > 1 ? 4.0 : 0.0);
    if (best == 0 || cost < best_cost) { best = Sk; best_cost = cost; }
    if (Sk >= 8 && best != 0) break;
  }
  if (best == 0) return QERL_ERR_SHAPE;
  const int Sk = best;
  const StreamLds l = layout((int)ceil_div(a.k_tiles, Sk));
  size_t total = l.total;
  a.red_bufs = l.red_bufs; a.max_pending = l.max_pending; a.pend_steps = l.pend_steps;
  if (a.n_producers > 0) {
    // producers: column blocks of their K share as large as LDS allows (one block = one round of loads)
    const int64_t steps = a.K / 16;
    a.prod_steps = (int)ceil_div(steps, a.n_producers);
    const size_t rows = (size_t)(a.r_total < 64 ? a.r_total : 64) + a.M + 1;
    const size_t red_producer = (size_t)kStreamWaves * 2 * MR * 64 * sizeof(float);
    int64_t cb = ((int64_t)((lds_cap - red_producer - 256) / rows) - 16) / 32;
    cb = cb < a.prod_steps ? cb : a.prod_steps;
    cb = cb < kProdMaxSteps ? cb : kProdMaxSteps;
    if (cb < 1) return QERL_ERR_SHAPE;
    a.prod_cb = (int)cb;
    a.prod_red_off = (int)((rows * (size_t)(cb * 32 + 16) + 255) & ~(size_t)255);
    const size_t need = a.prod_red_off + red_producer;
    if (need > total) total = need;
  }
  *lds_bytes = total;
  a.Sk = Sk; a.xs_stride = l.xs_stride; a.red_off = l.red_off; a.pend_off = l.pend_off; a.tsum_off = l.tsum_off;
  int64_t per_range = cus / Sk;
  if (per_range > a.total_tiles) per_range = a.total_tiles;
  if (per_range < 1) per_range = 1;
  // As many workgroups as give every one the same number of units (+- 1 only where the tiles do not divide):
  // the launch ends with its slowest workgroup, and the memory system is shared, so 237 workgroups of five
  // units finish before 160 of five beside 96 of four do.
  per_range = ceil_div(a.total_tiles, ceil_div(a.total_tiles, per_range));
  a.per_range = (int)per_range; a.kr_len = l.kr_len;
  a.units_base = a.total_tiles / a.per_range; a.units_rem = a.total_tiles % a.per_range;
  return QERL_OK;
}

template <int MR, int D, bool TIGHT, bool GATED = false>
static int launch_stream_t(const StreamArgs& a, size_t lds, hipStream_t st) {
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&stream_kernel<MR, D, TIGHT, GATED>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)kStreamLdsMax) != hipSuccess)
      return launch_status();
    attr_set = true;
  }
  stream_kernel<MR, D, TIGHT, GATED><<<dim3(a.n_producers + a.per_range * a.Sk), dim3(kStreamWaves * 64), lds, st>>>(a);
  if (a.Sk > 1) {
    const int rc = launch_status();
    if (rc != QERL_OK) return rc;
    ReduceArgs ra{};
    ra.partial = reinterpret_cast<const float*>(a.partial); ra.M = a.M; ra.Sk = a.Sk; ra.total_tiles = a.total_tiles;
    for (int i = 0; i < kMaxGroup; ++i) ra.mem[i] = ReduceMember{a.mem[i].y, a.mem[i].ldy, a.mem[i].N, a.mem[i].tile_begin};
    stream_reduce_kernel<MR><<<dim3((unsigned)ceil_div(a.total_tiles, 4)), dim3(256), 0, st>>>(ra);
  }
  return launch_status();
}

int launch_stream(const StreamArgs& a, size_t lds, int MR, hipStream_t st) {
  // every pointer the kernel dereferences must be set by the caller
  if (!a.x || !a.counters || !a.partial || a.n_members < 1 || a.n_members > kMaxGroup) return QERL_ERR_NULL;
  if (a.x2 && (a.ldx2 < a.K || a.ldx2 % 8 != 0 || ((uintptr_t)a.x2 & 15) != 0)) return QERL_ERR_ALIGN;
  for (int i = 0; i < a.n_members; ++i) {
    const StreamMember& m = a.mem[i];
    if (!m.packed || !m.tensor_scale || !m.y || m.N < 1 || m.n_tiles < 1) return QERL_ERR_NULL;
    if (m.r > 0 && (!m.A || !m.B || m.r > 64 || m.r % 8 != 0)) return QERL_ERR_SHAPE;
  }
  if (a.r_total > 0 && (a.n_producers < 1 || a.n_producers > 16 || !a.lora_ctl || !a.tpart)) return QERL_ERR_NULL;
  if (a.r_total == 0 && a.n_producers != 0) return QERL_ERR_SHAPE;
  if (a.n_producers > 0) {
    const size_t rows = (size_t)(a.r_total < 64 ? a.r_total : 64) + a.M + 1;
    if (a.prod_steps < 1 || a.prod_cb < 1 || a.prod_cb > kProdMaxSteps || (int64_t)a.prod_steps * a.n_producers < a.K / 16 ||
        rows * (size_t)(a.prod_cb * 32 + 16) > (size_t)a.prod_red_off ||
        (size_t)a.prod_red_off + (size_t)kStreamWaves * 2 * MR * 64 * sizeof(float) > lds)
      return QERL_ERR_SHAPE;
  }
  if (a.r_total < 0 || a.r_total > 256 || a.r_total % 8 != 0) return QERL_ERR_SHAPE;
  if (a.mp0 != a.mem[0].packed || a.mp1 != a.mem[1].packed || a.mp2 != a.mem[2].packed || a.mp3 != a.mem[3].packed ||
      a.tb1 != a.mem[1].tile_begin || a.tb2 != a.mem[2].tile_begin || a.tb3 != a.mem[3].tile_begin)
    return QERL_ERR_SHAPE;
  if (a.M < 1 || a.M > 16 || a.K < 16 || a.k_tiles < 1 || a.Sk < 1 || a.per_range < 1 || a.kr_len < 1 || (int64_t)a.kr_len * a.Sk < a.k_tiles ||
      a.units_base * a.per_range + a.units_rem != a.total_tiles ||
      a.total_tiles < 1 || lds > kStreamLdsMax || a.red_off <= 0 || a.pend_off < a.red_off ||
      a.red_bufs < 2 || a.red_bufs > kRedBufs || a.max_pending < 2 || a.max_pending > kMaxPending || a.pend_steps < 0 ||
      a.pend_steps > kLoraSteps || (size_t)a.red_off < (size_t)(a.M + (a.red_bufs == 2 ? 0 : 1)) * (size_t)a.xs_stride ||
      (size_t)(a.pend_off - a.red_off) < (size_t)a.red_bufs * kMainWaves * MR * 64 * sizeof(float) ||
      (size_t)(a.tsum_off - a.pend_off) < (size_t)a.max_pending * (MR * 64 * sizeof(float) + (size_t)a.pend_steps * 64 * 16) ||
      (size_t)a.tsum_off + 16 * 64 * sizeof(float) + 16 * 32 * 2 > lds)
    return QERL_ERR_SHAPE;
  const bool tight = a.red_bufs == 2;
  if (tight != (a.max_pending == 2) || (!tight && (a.red_bufs != kRedBufs || a.max_pending != kMaxPending ||
                                                   (a.pend_steps != kLoraSteps && a.pend_steps != 0))))
    return QERL_ERR_SHAPE;
  if (a.x2) {   // the variants that form SiLU(x) (.) x2 while staging (kept apart: the code costs the plain ones 2 %)
    if (MR == 4) return tight ? launch_stream_t<4, 4, true, true>(a, lds, st) : launch_stream_t<4, 4, false, true>(a, lds, st);
    return tight ? launch_stream_t<8, 4, true, true>(a, lds, st) : launch_stream_t<8, 4, false, true>(a, lds, st);
  }
  if (MR == 4 && tight) return launch_stream_t<4, 4, true>(a, lds, st);
  if (MR == 4 && g_force_depth == 3) return launch_stream_t<4, 3, false>(a, lds, st);
  if (MR == 4 && g_force_depth == 6) return launch_stream_t<4, 6, false>(a, lds, st);
  if (MR == 4) return launch_stream_t<4, 4, false>(a, lds, st);
  if (tight) return launch_stream_t<8, 4, true>(a, lds, st);
  return launch_stream_t<8, 4, false>(a, lds, st);
}

}  // namespace qerl

// Tuning hooks for experiments (not part of the public header): number of K-ranges and ring depth; 0 = automatic.
#ifdef QERL_TUNING_HOOKS   // built only for tuning sessions: they change process-wide state
extern "C" QERL_API void qerl_debug_force_stream(int ranges) { qerl::g_force_ranges = ranges; }
extern "C" QERL_API void qerl_debug_force_stream_depth(int d) { qerl::g_force_depth = d; }
#endif  // QERL_TUNING_HOOKS
#ifdef QERL_STREAM_TRACE
extern "C" QERL_API int qerl_debug_read_trace(void* dst, size_t bytes) {
  return (int)hipMemcpyFromSymbol(dst, HIP_SYMBOL(qerl::g_trace), bytes, 0, hipMemcpyDeviceToHost);
}
#endif
