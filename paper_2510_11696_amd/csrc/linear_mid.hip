// NVFP4 + LoRA linear for 17..128 tokens: too many for the accumulator-side scaling of the decode
// kernels (its cost grows with the token count), too few for the prefill GEMM to fill the chip (one
// block of token rows, so only N / 256 workgroups, each waiting for one 64-input stage at a time).
//
//   y[m,n] = S32 * sum_k x[m,k] * (s[n,k/16] * e[n,k]) + lora_scale * sum_j t[m,j] * B[n,j]
//                                                                    (Eq. 6, Eq. 2)
// Here the layer is bound by streaming the packed weights (up to ~64 tokens) or by the MFMA rate
// (128 tokens), and in both cases by memory latency unless enough loads are in flight.  So:
//
//   * A workgroup of W waves owns W adjacent row-tiles (32 output rows each, one per wave) for ALL
//     tokens (BM = 32*MT >= M) and walks K in stages of one packed K-tile (128 inputs, 2304 bytes per
//     wave).  Every weight is dequantised once: codes -> (cvt, * block scale, pack) -> bf16 MFMA B
//     operand; s * e has at most 6 significant bits, exact in bf16.
//   * Weights go global -> registers through a ring of kRing stages per wave (seven K-tiles requested
//     ahead of the one in use); nothing of the weight stream touches LDS.
//   * x is the shared operand: the BM x 128 slab of a stage is requested kXAhead stages ahead into
//     registers, written to one of two LDS buffers a stage before it is used (16-byte chunks
//     XOR-swizzled by row: the A-operand reads of 16 rows at one column hit 16 distinct bank groups),
//     one barrier per stage.
//   * K can be split over S workgroups per row-tile group when N alone gives too few workgroups; each
//     split writes its fp32 partial [M, N] to the workspace and mid_reduce_kernel adds the splits in
//     order.  No workgroup waits for another.
//   * LoRA: ts = [hi | mid | lo] (three bf16 terms of (lora_scale / S32) * x A^T, produced by the
//     prefill path's down-projection kernel) enters as 3r more input columns against [B ; B ; B]; the
//     accumulators are multiplied by S32 once at the end (split 0 carries the LoRA columns).
//
// Operand layouts and the packed tile format are described in linear_decode.hip.
#include "linear.hpp"
#include "lora_down.hpp"

namespace qerl {

constexpr int kRing = 8;      // weight stages per wave: one in use, seven requested
constexpr uint32_t kMidSpinLimit = 1u << 16;   // polls (of ~0.5 us) a consumer spends on the producers of its launch before it gives up

struct MidTile { u32x4 c0, c1; u32x2 sc; };   // one wave's share of a packed tile: 2 x 4 steps x 8 codes, 8 scale bytes

template <int MT, int W>
__global__ __launch_bounds__(W * 64) void mid_kernel(const MidArgs a) {
  constexpr int BM = MT * 32;
  constexpr int kThreads = W * 64;
  constexpr int kXAhead = MT == 4 ? 2 : 4;         // x slabs in registers (they are shared reads, usually L2 hits; 128 tokens leave room for two)
  constexpr int kChunks = BM * 16;                 // 16-byte chunks of one x slab (BM x 128)
  constexpr int XL = kChunks / kThreads;           // chunks per thread
  static_assert(kChunks % kThreads == 0 && kRing % kXAhead == 0 && kRing % 2 == 0, "ring sizes");
  // x slab [2][BM][16 chunks]; chunk c of row r sits at r*16 + (c ^ (r & 15))
  extern __shared__ __attribute__((aligned(256))) u32x4 xs[];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n32 = lane & 31, kg = lane >> 5;
  // Workgroup ids go round-robin to the 8 XCDs: the splits and token blocks of one row-tile group get ids
  // that are equal mod 8, i.e. they share an L2.
  if ((int)blockIdx.x < a.n_prod) {
    // ---- a LoRA producer: one (token block, rank tile, K-part) of the down-projections; dispatched before
    // every consumer, waits for nothing but its own loads
    const int id = (int)blockIdx.x;
    if (id >= a.p_tbs * a.p_tiles * a.p_parts) return;
    const int bx = id % a.p_tbs, by = (id / a.p_tbs) % a.p_tiles, bz = id / (a.p_tbs * a.p_tiles);
    lora_down_block<1, W>(a.dn, bx, by, bz, a.p_parts, a.p_tbs, a.p_tiles, reinterpret_cast<float*>(xs));
    return;
  }
  const int bid = (int)blockIdx.x - a.n_prod;
  const int inner_n = a.m_chunks * a.S;
  const int xcd = bid & 7, rest = bid >> 3;
  const int inner = rest % inner_n;
  const int nb = (rest / inner_n) * 8 + xcd;
  if (nb >= a.n_blocks) return;                    // padding of the last group of eight (uniform)
  const int chunk = inner / a.S, split = inner % a.S;
  const int64_t m0 = (int64_t)chunk * BM;
  // the linear of the group this column block belongs to (one member: always the first)
  int mi = 0;
#pragma unroll
  for (int i = 1; i < kMaxGroup; ++i) mi = nb >= a.mem[i].block_begin ? i : mi;
  const MidMember& mem = a.mem[__builtin_amdgcn_readfirstlane(mi)];   // uniform index: scalar loads from the kernel arguments
  const int nt = (nb - mem.block_begin) * W + wave;   // row-tile within the member
  const int nt_ld = nt < mem.n_tiles ? nt : mem.n_tiles - 1;
  const int kt0 = split * a.kt_per_split;
  const int kt1 = kt0 + a.kt_per_split < a.k_tiles ? kt0 + a.kt_per_split : a.k_tiles;
  const int n = kt1 - kt0;                         // >= 1 (host)

  f32x16 acc[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[mt][i] = 0.f;

  // ---- loaders (stage kt covers columns [128 kt, 128 kt + 128) of the row-major bf16 matrix `src`)
  auto gload_x = [&](u32x4 (&r)[XL], const uint16_t* src, int64_t ld, int64_t cols, int kt) {
#pragma unroll
    for (int i = 0; i < XL; ++i) {
      const int idx = tid + i * kThreads;
      const int row = idx >> 4, c = idx & 15;
      int64_t gr = m0 + row;
      gr = gr < a.M ? gr : a.M - 1;
      int64_t k = (int64_t)kt * 128 + c * 8;
      k = k < cols ? k : cols - 8;      // past the end the other operand is zero; any finite value will do
      r[i] = *reinterpret_cast<const u32x4*>(src + gr * ld + k);
    }
  };
  auto swrite_x = [&](int buf, const u32x4 (&r)[XL]) {
#pragma unroll
    for (int i = 0; i < XL; ++i) {
      const int idx = tid + i * kThreads;
      const int row = idx >> 4, c = idx & 15;
      xs[buf * kChunks + row * 16 + (c ^ (row & 15))] = r[i];
    }
  };
  const uint8_t* wbase = mem.packed + (int64_t)nt_ld * a.k_tiles * kPackTileBytes;
  auto gload_w = [&](MidTile& t, int kt) {
    const uint8_t* base = wbase + (int64_t)kt * kPackTileBytes;
    t.c0 = *reinterpret_cast<const u32x4*>(base + lane * 16);
    t.c1 = *reinterpret_cast<const u32x4*>(base + 1024 + lane * 16);
    t.sc = *reinterpret_cast<const u32x2*>(base + 2048 + n32 * 8);
  };
  auto mma_step = [&](const u32x4* xst, int j, bf16x8 wf) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int row = mt * 32 + n32;
      const bf16x8 af = __builtin_bit_cast(bf16x8, xst[row * 16 + ((2 * j + kg) ^ (row & 15))]);
      acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, wf, acc[mt], 0, 0, 0);
    }
  };
  // One stage, software-pipelined by hand (a SIMD holds one or two of these waves, so what a wave does not
  // overlap itself stays exposed): on entry `wf` holds the dequantised weights of the stage's first step;
  // the conversions of step j + 1 (of the next stage's first step, from `tn`, at the end) are written
  // between the MFMAs of step j, and every x fragment is re-requested from LDS right after the MFMA that
  // used it.
  auto dequant_step = [&](const MidTile& t, int j) {
    const uint32_t codes = j < 4 ? t.c0[j & 3] : t.c1[j & 3];
    return dequant8_bf16(codes, e4m3_byte_f32(j < 4 ? t.sc[0] : t.sc[1], j & 3));
  };
  bf16x8 wf;
  auto compute = [&](int buf, const MidTile& t, const MidTile& tn) {
    const u32x4* xst = xs + buf * kChunks;
    if constexpr (MT > 2) {   // four token blocks: the MFMAs of a step already cover its conversions; keep the registers
#pragma unroll
      for (int j = 0; j < 8; ++j) mma_step(xst, j, dequant_step(t, j));
      return;
    }
    bf16x8 af[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int row = mt * 32 + n32;
      af[mt] = __builtin_bit_cast(bf16x8, xst[row * 16 + (kg ^ (row & 15))]);
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const bf16x8 wfn = j < 7 ? dequant_step(t, j + 1) : dequant_step(tn, 0);
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mt], wf, acc[mt], 0, 0, 0);
        if (j < 7) {
          const int row = mt * 32 + n32;
          af[mt] = __builtin_bit_cast(bf16x8, xst[row * 16 + ((2 * (j + 1) + kg) ^ (row & 15))]);
        }
      }
      wf = wfn;
    }
  };

  MidTile wr[kRing];
  u32x4 xr[kXAhead][XL];
  // ---- prologue: the first slabs and weight stages are requested, slab 0 goes to LDS.  Requests past the
  // end of the range are not skipped but redirected to its last stage (a few redundant loads that hit in
  // L2): with no branches around the loads the compiler's wait counts stay exact, and a wave never waits for
  // more than the stage it needs.
  const int kt_last = kt1 - 1;
  auto clamp_kt = [&](int kt) { return kt < kt_last ? kt : kt_last; };
#pragma unroll
  for (int p = 0; p < kXAhead; ++p) gload_x(xr[p], a.x, a.ldx, a.K, clamp_kt(kt0 + p));
#pragma unroll
  for (int d = 0; d < kRing - 1; ++d) gload_w(wr[d], clamp_kt(kt0 + d));
  swrite_x(0, xr[0]);
  wf = dequant_step(wr[0], 0);
  __syncthreads();
  // ---- main loop, unrolled over the ring so that every register array index is a constant: whole rounds of
  // the ring without a branch inside, then the remaining stages as straight-line code with forward exits only
  auto stage = [&](int i, int u) {
    gload_x(xr[u % kXAhead], a.x, a.ldx, a.K, clamp_kt(kt0 + i + kXAhead));
    gload_w(wr[(u + kRing - 1) % kRing], clamp_kt(kt0 + i + kRing - 1));
    compute(u & 1, wr[u], wr[(u + 1) % kRing]);
    swrite_x((u + 1) & 1, xr[(u + 1) % kXAhead]);
    __syncthreads();
  };
  int i0 = 0;
  for (; i0 + kRing <= n; i0 += kRing) {
#pragma unroll
    for (int u = 0; u < kRing; ++u) stage(i0 + u, u);
  }
#pragma unroll
  for (int u = 0; u < kRing - 1; ++u) {
    if (i0 + u >= n) goto main_done;
    stage(i0 + u, u);
  }
main_done:

  // ---- LoRA up-projection: 3r extra columns [hi | mid | lo] . [B ; B ; B]^T.  ts already carries the
  // factor lora_scale / S32, so one multiplication by S32 at the end scales both branches.
  bool poisoned = false;
  if (split == 0 && mem.ext_stages > 0 && a.n_prod > 0) {
    // ts comes from the producers of this launch: wait (bounded) until all of them have published it
    uint32_t spins = 0;
    while (__hip_atomic_load(a.ready, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < (uint32_t)(a.p_tbs * a.p_tiles)) {
      if (++spins > kMidSpinLimit) {   // never reached unless a producer died or was kept off the chip: make it visible
        poisoned = true;
        if (tid == 0) __hip_atomic_fetch_or(a.ready + kCtlErr, 4u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        break;
      }
      __builtin_amdgcn_s_sleep(32);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
  }
  if (split == 0) {
    for (int e = 0; e < mem.ext_stages; ++e) {
      gload_x(xr[0], mem.ts, mem.ts_ld, mem.ts_ld, e);
      swrite_x(0, xr[0]);
      __syncthreads();
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        int64_t row = (int64_t)nt * 32 + n32;
        row = row < mem.N ? row : mem.N - 1;
        const int c = e * 128 + 16 * j + 8 * kg;
        u32x4 b = {0u, 0u, 0u, 0u};
        if (c < 3 * mem.r) b = *reinterpret_cast<const u32x4*>(mem.B + row * mem.r + (c % mem.r));
        mma_step(xs, j, __builtin_bit_cast(bf16x8, b));
      }
      __syncthreads();
    }
  }
  if (a.n_prod > 0 && tid == 0) {
    // the last consumer to leave re-arms the hand-over words (every waiting workgroup has passed its wait by then)
    const uint32_t old = __hip_atomic_fetch_add(a.done, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (old == (uint32_t)(a.n_consumers - 1) && __hip_atomic_load(a.ready + kCtlErr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u) {   // (not after a wait that gave up)
      __hip_atomic_store(a.ready, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(a.done, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
  const float S32 = poisoned ? __uint_as_float(0x7fc00000u) : *mem.tensor_scale;
  const int64_t nn = (int64_t)nt * 32 + n32;
  if (nt >= mem.n_tiles || nn >= mem.N) return;
  const float bias = (mem.bias && split == 0) ? bf16_bits_to_f32(mem.bias[nn]) : 0.f;   // split 0 carries it, like the LoRA columns
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int64_t m = m0 + mt * 32 + 8 * (i >> 2) + 4 * kg + (i & 3);
      if (m < a.M) {
        const float v = acc[mt][i] * S32 + bias;
        if (a.S == 1) mem.y[m * mem.ldy + nn] = (uint16_t)f32_to_bf16_bits(v);
        else a.partial[mem.partial_off + ((int64_t)split * a.M + m) * mem.N + nn] = v;
      }
    }
}

// y = sum over the K-splits, in split order, of the fp32 partial outputs [S][M][N] of every member.
// Grid: (max N / 256, M, members).
struct MidReduceArgs { const float* partial; int S; int64_t M; int64_t N[kMaxGroup]; int64_t off[kMaxGroup]; uint16_t* y[kMaxGroup]; int64_t ldy[kMaxGroup]; };
__global__ __launch_bounds__(256) void mid_reduce_kernel(const MidReduceArgs a) {
  const int mi = blockIdx.z;
  const int64_t N = a.N[mi];
  const int64_t n = (int64_t)blockIdx.x * 256 + threadIdx.x, m = blockIdx.y;
  if (n >= N) return;
  const float* p = a.partial + a.off[mi] + m * N + n;
  float v[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) v[s] = s < a.S ? p[(int64_t)s * a.M * N] : 0.f;
  float sum = 0.f;
#pragma unroll
  for (int s = 0; s < 8; ++s) sum += v[s];
  a.y[mi][m * a.ldy[mi] + n] = (uint16_t)f32_to_bf16_bits(sum);
}

// ---- host ------------------------------------------------------------------------------------------

static int g_force_w = 0, g_force_s = 0;
int g_mid_max_tokens = 128;   // token counts above this go to the prefill GEMM

template <int MT, int W>
static int launch_mid_t(const MidArgs& a, hipStream_t st) {
  constexpr size_t lds_tiles = 2 * (size_t)MT * 32 * 16 * sizeof(u32x4);
  const size_t lds = (a.n_prod > 0 && kLoraDownLdsBytes(1, W) > lds_tiles) ? kLoraDownLdsBytes(1, W) : lds_tiles;
  const int64_t groups = ceil_div(a.n_blocks, 8);
  mid_kernel<MT, W><<<dim3((unsigned)(a.n_prod + groups * 8 * a.m_chunks * a.S)), dim3(W * 64), lds, st>>>(a);
  return launch_status();
}

int plan_mid(MidArgs& a, size_t partial_cap_bytes) {
  if (a.M < 1 || a.M > g_mid_max_tokens || a.n_members < 1 || a.n_members > kMaxGroup || a.k_tiles < 1) return QERL_ERR_SHAPE;
  const int MT = a.M <= 32 ? 1 : a.M <= 64 ? 2 : 4;
  a.MT = MT; a.m_chunks = (int)ceil_div(a.M, 32 * MT);
  int64_t n_sum = 0;
  for (int i = 0; i < a.n_members; ++i) n_sum += a.mem[i].N;
  // Waves per workgroup and K-splits: the pair with the shortest estimated time.  A wave spends about
  // 650 + 350 MT cycles on a stage (dequantisation plus MT x 8 MFMAs); workgroups spread evenly over the 256
  // CUs, their waves over the CU's four SIMDs.  A split costs a second launch and the partial sums' traffic.
  // the first wins ties: four waves measured equal or better than two at equal estimates, except for a group of
  // few row tiles (q + k + v at 7B: 144) at up to 32 tokens, which then has too few workgroups
  int64_t tiles_sum = 0;
  for (int i = 0; i < a.n_members; ++i) tiles_sum += a.mem[i].n_tiles;
  const bool small_group = MT == 1 && a.n_members > 1 && tiles_sum < 256;
  const int w_opts[2] = {MT == 4 || !small_group ? 4 : 2, MT == 4 ? 8 : (small_group ? 4 : 2)};
  const double cyc = 650.0 + 350.0 * MT;
  double best = 0;
  a.W = 0;
  for (int wi = 0; wi < 2; ++wi) {
    const int W = w_opts[wi];
    if (g_force_w > 0 && W != g_force_w) continue;
    int64_t blocks = 0;
    for (int i = 0; i < a.n_members; ++i) blocks += ceil_div(a.mem[i].n_tiles, W);
    for (int S = 1; S <= 8; ++S) {
      if (g_force_s > 0 && S != g_force_s) continue;
      if (S > 1 && ((size_t)S * a.M * n_sum * sizeof(float) > partial_cap_bytes || a.k_tiles / S < 4)) continue;
      const int64_t per = ceil_div(a.k_tiles, S), S_eff = ceil_div(a.k_tiles, per);
      if (S_eff != S) continue;
      const int64_t wgs = blocks * a.m_chunks * S;
      const int64_t on_cu = ceil_div(wgs, 256), per_simd = ceil_div(on_cu * W, 4);
      double us = (double)(per_simd * per) * cyc / 2400.0;
      if (S > 1) us += 4.0 + 2.0 * (double)S * a.M * n_sum * sizeof(float) / 4.0e6;
      if (a.W == 0 || us < best) { best = us; a.W = W; a.S = S; a.kt_per_split = (int)per; }
    }
  }
  if (a.W == 0) return QERL_ERR_SHAPE;
  int blocks = 0;
  int64_t poff = 0;
  for (int i = 0; i < kMaxGroup; ++i) {
    if (i < a.n_members) {
      a.mem[i].block_begin = blocks; a.mem[i].partial_off = poff;
      blocks += (int)ceil_div(a.mem[i].n_tiles, a.W);
      poff += (int64_t)a.S * a.M * a.mem[i].N;
    } else {
      a.mem[i] = a.mem[0];
      a.mem[i].block_begin = 0x7fffffff;
    }
  }
  a.n_blocks = blocks;
  return QERL_OK;
}

int launch_mid(const MidArgs& a, hipStream_t st) {
  // every pointer the kernel dereferences must be set by the caller
  if (!a.x || a.n_members < 1 || a.n_members > kMaxGroup || (a.S > 1 && !a.partial)) return QERL_ERR_NULL;
  if (a.M < 1 || a.M > g_mid_max_tokens || a.K < 16 || a.k_tiles < 1 || a.S < 1 || a.S > 8 || a.kt_per_split < 1 ||
      (int64_t)a.kt_per_split * a.S < a.k_tiles || (int64_t)a.kt_per_split * (a.S - 1) >= a.k_tiles ||
      (int64_t)a.m_chunks * a.MT * 32 < a.M)
    return QERL_ERR_SHAPE;
  int blocks = 0;
  for (int i = 0; i < a.n_members; ++i) {
    const MidMember& m = a.mem[i];
    if (!m.packed || !m.tensor_scale || !m.y || (m.r > 0 && (!m.ts || !m.B))) return QERL_ERR_NULL;
    if (m.N < 1 || m.n_tiles < 1 || m.block_begin != blocks ||
        (m.r > 0 && (m.ts_ld < 3 * m.r || m.ts_ld != (int64_t)m.ext_stages * 128)) || (m.r == 0 && m.ext_stages != 0))
      return QERL_ERR_SHAPE;
    blocks += (int)ceil_div(m.n_tiles, a.W);
  }
  if (blocks != a.n_blocks) return QERL_ERR_SHAPE;
  if (a.n_prod != 0) {   // the producers' description, checked as the stand-alone launch checks it
    const GemmArgs& d = a.dn;
    if (a.n_prod < 0 || a.n_prod % 8 != 0 || a.p_tbs < 1 || a.p_tiles < 1 || a.p_parts < 1 || a.p_parts > kDownMaxParts ||
        (int64_t)a.p_tbs * a.p_tiles * a.p_parts > a.n_prod || (int64_t)a.p_tbs * 32 < a.M ||
        a.n_consumers != a.n_blocks * a.m_chunks * a.S || d.g_n < 1 || d.g_n > kMaxGroup || d.M != a.M || d.K != a.K)
      return QERL_ERR_SHAPE;
    if (!a.ready || !a.done || d.ready != a.ready || d.x != a.x || (a.p_parts > 1 && (!d.tpart || !d.counters))) return QERL_ERR_NULL;
    int tiles = 0;
    for (int i = 0; i < d.g_n; ++i) {
      if (!d.g_A[i] || !d.g_ts[i] || !d.g_tensor_scale[i]) return QERL_ERR_NULL;
      if (d.g_r[i] < 1 || d.g_ts_ld[i] < 3 * d.g_r[i] || d.g_tile0[i] != tiles) return QERL_ERR_SHAPE;
      tiles += (int)ceil_div(d.g_r[i], 32);
    }
    if (d.g_tile0[d.g_n] != tiles || tiles != a.p_tiles) return QERL_ERR_SHAPE;
  }
  int rc = QERL_ERR_SHAPE;
  if (a.MT == 1 && a.W == 2) rc = launch_mid_t<1, 2>(a, st);
  else if (a.MT == 1 && a.W == 4) rc = launch_mid_t<1, 4>(a, st);
  else if (a.MT == 2 && a.W == 2) rc = launch_mid_t<2, 2>(a, st);
  else if (a.MT == 2 && a.W == 4) rc = launch_mid_t<2, 4>(a, st);
  else if (a.MT == 4 && a.W == 4) rc = launch_mid_t<4, 4>(a, st);
  else if (a.MT == 4 && a.W == 8) rc = launch_mid_t<4, 8>(a, st);
  if (rc != QERL_OK || a.S == 1) return rc;
  MidReduceArgs ra{};
  ra.partial = a.partial; ra.S = a.S; ra.M = a.M;
  int64_t n_max = 0;
  for (int i = 0; i < a.n_members; ++i) {
    const MidMember& m = a.mem[i];
    ra.N[i] = m.N; ra.off[i] = m.partial_off; ra.y[i] = m.y; ra.ldy[i] = m.ldy;
    n_max = n_max > m.N ? n_max : m.N;
  }
  mid_reduce_kernel<<<dim3((unsigned)ceil_div(n_max, 256), (unsigned)a.M, (unsigned)a.n_members), dim3(256), 0, st>>>(ra);
  return launch_status();
}

}  // namespace qerl

// Tuning hook for experiments (not part of the public header): waves per workgroup and K-splits, 0 = automatic.
#ifdef QERL_TUNING_HOOKS   // built only for tuning sessions: they change process-wide state
extern "C" QERL_API void qerl_debug_force_mid(int waves, int splits) { qerl::g_force_w = waves; qerl::g_force_s = splits; }
extern "C" QERL_API void qerl_debug_mid_max_tokens(int m) { qerl::g_mid_max_tokens = m; }
#endif  // QERL_TUNING_HOOKS
