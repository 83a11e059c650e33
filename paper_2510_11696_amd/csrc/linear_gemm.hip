// Prefill-sized NVFP4 + LoRA linear (M > 16 tokens): a bf16 MFMA GEMM that
// dequantises the tile-packed weights in registers.
//
//   y[m,n] = S32 * sum_k x[m,k] * (s[n,k/16] * e[n,k]) + lora_scale * sum_j t[m,j] * B[n,j]
//                                                                    (Eq. 6, Eq. 2)
// Compute bound (2*M*N*K flop against 0.5625*N*K bytes), so the target is the
// bf16 MFMA rate.  s * e has at most 6 significant bits and is exact in bf16;
// products are exact in the fp32 accumulator; S32 multiplies the sum once.
//
//   * Workgroup tile: BM = 32*MT tokens x BN = 32*NT*W output rows, W waves.
//     Every wave owns its own NT column tiles for all BM tokens, so no weight
//     is dequantised twice in a workgroup: packed bytes go global -> registers
//     -> (cvt, scale, pack: ~20 VALU ops per 8 weights) -> MFMA B operand.
//   * x is the shared operand: a BM x 128 slab per K-tile is staged in LDS,
//     double buffered through registers, 16-byte chunks XOR-swizzled by row so
//     that the A-operand reads (32 rows at one column) hit distinct banks.
//   * v_mfma_f32_32x32x16_bf16, A = x (row = token), B = weights (col = n);
//     MT*NT accumulator tiles of 16 registers per lane.
//   * LoRA: a first launch of the same kernel over the dense bf16 matrix A
//     (split along K, partial tiles added in slice order by the last workgroup
//     to arrive) produces  ts = [hi | mid | lo]  with hi + mid + lo =
//     lora_scale * x A^T up to 2^-27, three bf16 terms per value.  The main
//     launch then treats the up-projection as 3r more input columns:
//     [x | ts] . [S32 * W_hat ; B ; B ; B]^T, i.e. the accumulators are scaled by
//     S32 after the weight stages and the extra stages multiply ts by B.
//
// Operand layouts and the packed tile format are described in linear_decode.hip.
#include "linear.hpp"
#include "lora_down.hpp"

namespace qerl {

constexpr uint32_t kGemmSpinLimit = 1u << 16;   // polls (of ~0.5 us) a workgroup spends on the producers of its launch before it gives up
constexpr int kGemmRing = 4;    // stages of weights in registers per wave (even)
constexpr int kGemmXAhead = 2;  // x slabs in registers (divides kGemmRing)

template <int NT>
struct WeightRegs {      // one stage = 64 inputs (4 MFMA steps) of NT column tiles
  u32x4 c[NT];           // 4 steps x 8 codes
  uint32_t sc[NT];       // 4 scale bytes
};

// TR: the packed operand is in the transposed tile order (nvfp4_prepack_t): the contraction runs over the rows
// of W, so the eight weights of a lane and MFMA step carry eight different block scales; the scale bytes of a
// stage (128 per column tile) ride along with the x slab through LDS.  Used by the backward pass
// (dX = dY W_hat); everything around the dequantisation step is shared with the forward kernel.
// SK: the forward launch of few tokens -- K split over workgroups and / or the LoRA down-projections as its first
// workgroups; a variant of its own so that the prefill kernel carries none of it.
template <int MT, int NT, int W, bool TR = false, bool SK = false>
__global__ __launch_bounds__(W * 64) void gemm32_kernel(const GemmArgs a) {
  static_assert(!(TR && SK), "the backward launch has no K split");
  constexpr int BM = MT * 32;
  constexpr int kThreads = W * 64;
  constexpr int kChunks = BM * 8;                          // 16-byte chunks of one x slab (BM x 64)
  constexpr int XL = (kChunks + kThreads - 1) / kThreads;  // chunks per thread
  // x slab [2][BM][8 chunks]; chunk c of row r sits at r*8 + (c ^ ((r >> 1) & 7)): rows r, r+1 use
  // different bank halves, so 16 consecutive rows at one column touch 16 distinct 16-byte bank groups.
  extern __shared__ u32x4 xs[];
  constexpr int kScBytes = W * NT * 128;                   // TR: scale bytes of one stage, all column tiles of the workgroup
  uint8_t* ssc = reinterpret_cast<uint8_t*>(xs + 2 * kChunks);   // TR: [2][kScBytes] behind the x slabs

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keeps everything derived from it in SGPRs
  const int n32 = lane & 31, kg = lane >> 5;
  // Workgroup -> tile map, XCD aware: consecutive workgroup ids go round-robin to the 8 XCDs (each with
  // its own L2), so XCD x = id % 8 gets a contiguous eighth of the column blocks and walks them fastest:
  // the ~32 workgroups an XCD runs at a time then share a few x slabs and each weight stripe stays in
  // one L2 instead of eight.
  int bid = (int)blockIdx.x;
  if constexpr (SK && W <= 8) {
    if (bid < a.n_prod) {
      // ---- a LoRA producer: one (token block, rank tile, K-part) of the down-projections; dispatched before
      // every consumer, waits for nothing but its own loads
      if (bid >= a.p_tbs * a.p_tiles * a.p_parts) return;
      const int bx = bid % a.p_tbs, by = (bid / a.p_tbs) % a.p_tiles, bz = bid / (a.p_tbs * a.p_tiles);
      lora_down_block<1, W>(a, bx, by, bz, a.p_parts, a.p_tbs, a.p_tiles, reinterpret_cast<float*>(xs));
      return;
    }
    bid -= a.n_prod;
  }
  const int xcd = bid & 7, local = bid >> 3;
  const int nb_local = local % a.nblk_per_xcd, mb_all = local / a.nblk_per_xcd;
  const int nb = xcd * a.nblk_per_xcd + nb_local;
  if (nb >= a.n_blocks) return;          // padding of the last XCD's share (uniform per workgroup)
  // K split over workgroups (forward only): part ks of a.ksplit, token block mb
  int mb = mb_all, ks = 0;
  if constexpr (SK) {
    if (a.ksplit > 1) { ks = mb_all / a.m_blocks; mb = mb_all - ks * a.m_blocks; }
  }
  const int64_t m0 = (int64_t)mb * BM;
  // the member of the group this column block belongs to: a uniform index into the kernel arguments, so
  // its fields arrive by scalar loads
  int mi = 0;
#pragma unroll
  for (int i = 1; i < kMaxGroup; ++i) mi = (i < a.m_n && nb >= a.m[i].block_begin) ? i : mi;
  const GemmMember& mem = a.m[__builtin_amdgcn_readfirstlane(mi)];
  const int nt0 = ((nb - mem.block_begin) * W + wave) * NT;
  // The contraction's source: the launch's x and the member's tiles, or (TR) one segment after the other
  const uint16_t* sx = a.x;
  int64_t sldx = a.ldx, sK = a.K, skt = a.k_tiles;
  const uint8_t* spk = mem.packed;
  const uint16_t* sts = mem.ts;
  int64_t sts_ld = mem.ts_ld;
  int sext = mem.ext_stages, sr = mem.r;
  const uint16_t* sB = mem.B;
  const float* sscale = mem.tensor_scale;

  bool poisoned = false;   // a bounded wait gave up: the outputs become NaN
  f32x16 acc[MT][NT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
      for (int i = 0; i < 16; ++i) acc[mt][nt][i] = 0.f;

  // ---- loaders (stage s covers columns [64 s, 64 s + 64) of the row-major bf16 matrix `src`)
  auto gload_x = [&](u32x4 (&xr)[XL], const uint16_t* src, int64_t ld, int64_t cols, int64_t s) {
#pragma unroll
    for (int i = 0; i < XL; ++i) {
      const int idx = tid + i * kThreads;
      const int row = idx >> 3, chunk = idx & 7;
      int64_t gr = m0 + row;
      gr = gr < a.M ? gr : a.M - 1;
      int64_t k = s * 64 + chunk * 8;
      k = k < cols ? k : cols - 8;      // past the end the other operand is zero; any finite value will do
      xr[i] = u32x4{0u, 0u, 0u, 0u};
      if (idx < kChunks) xr[i] = *reinterpret_cast<const u32x4*>(src + gr * ld + k);
    }
  };
  auto swrite_x = [&](int buf, const u32x4 (&xr)[XL]) {
#pragma unroll
    for (int i = 0; i < XL; ++i) {
      const int idx = tid + i * kThreads;
      const int row = idx >> 3, chunk = idx & 7;
      if (idx < kChunks) xs[buf * kChunks + row * 8 + (chunk ^ ((row >> 1) & 7))] = xr[i];
    }
  };
  auto gload_w = [&](WeightRegs<NT>& wr, int64_t s) {
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      int tile = nt0 + nt;
      tile = tile < mem.n_tiles ? tile : mem.n_tiles - 1;
      const uint8_t* base = spk + ((int64_t)tile * skt + (s >> 1)) * kPackTileBytes;
      const int plane = (int)(s & 1);
      wr.c[nt] = *reinterpret_cast<const u32x4*>(base + plane * 1024 + lane * 16);
      wr.sc[nt] = 0u;
      if constexpr (!TR) wr.sc[nt] = *reinterpret_cast<const uint32_t*>(base + 2048 + n32 * 8 + plane * 4);
    }
  };
  // TR: thread t < 8 W NT fetches 16 of the 128 scale bytes of column tile t / 8 for stage s
  const int sc_tl = tid >> 3, sc_part = tid & 7;
  auto gload_sc = [&](u32x4& r, int64_t s) {
    r = u32x4{0u, 0u, 0u, 0u};
    if (tid < W * NT * 8) {
      int tile = (nb - mem.block_begin) * W * NT + sc_tl;
      tile = tile < mem.n_tiles ? tile : mem.n_tiles - 1;
      const uint8_t* base = spk + ((int64_t)tile * skt + (s >> 1)) * kPackTileBytes;
      r = *reinterpret_cast<const u32x4*>(base + 2048 + (int)(s & 1) * 128 + sc_part * 16);
    }
  };
  auto swrite_sc = [&](int buf, const u32x4& r) {
    if (tid < W * NT * 8) *reinterpret_cast<u32x4*>(ssc + buf * kScBytes + sc_tl * 128 + sc_part * 16) = r;
  };
  auto mma_step = [&](const u32x4* xst, int j, const bf16x8 (&wf)[NT]) {
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int row = mt * 32 + n32;
      const bf16x8 af = __builtin_bit_cast(bf16x8, xst[row * 8 + ((2 * j + kg) ^ ((row >> 1) & 7))]);
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, wf[nt], acc[mt][nt], 0, 0, 0);
    }
  };
  // One stage, software-pipelined by hand: on entry `wf` holds the dequantised weights of the stage's first
  // step.  The MFMAs of step j are interleaved with the dequantisation of step j + 1 (of the next stage's
  // first step, from `wn`, at the end), and every x fragment register is re-requested from LDS right after
  // the MFMAs that used it, so neither the LDS latency nor the conversions stand between two MFMAs.
  bf16x8 wf[NT];
  auto compute = [&](int buf, const WeightRegs<NT>& wr, const WeightRegs<NT>& wn) {
    const u32x4* xst = xs + buf * kChunks;
    bf16x8 af[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int row = mt * 32 + n32;
      af[mt] = __builtin_bit_cast(bf16x8, xst[row * 8 + (kg ^ ((row >> 1) & 7))]);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      bf16x8 wfn[NT];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        wfn[nt] = j < 3 ? dequant8_bf16(wr.c[nt][(j + 1) & 3], e4m3_byte_f32(wr.sc[nt], (j + 1) & 3))
                        : dequant8_bf16(wn.c[nt][0], e4m3_byte_f32(wn.sc[nt], 0));
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
          acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mt], wf[nt], acc[mt][nt], 0, 0, 0);
        if (j < 3) {
          const int row = mt * 32 + n32;
          af[mt] = __builtin_bit_cast(bf16x8, xst[row * 8 + ((2 * (j + 1) + kg) ^ ((row >> 1) & 7))]);
        }
      }
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) wf[nt] = wfn[nt];
    }
  };

  // TR: no pipelining across steps -- each step's weights are dequantised right before its MFMAs, with the
  // eight scale bytes of the lane's (input block, 8 rows) read from LDS
  auto compute_tr = [&](int buf, const WeightRegs<NT>& wr) {
    const u32x4* xst = xs + buf * kChunks;
    const uint8_t* sst = ssc + buf * kScBytes + wave * NT * 128 + (n32 >> 4) * 64 + 8 * kg;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      bf16x8 wt[NT];
#pragma unroll
      for (int nt = 0; nt < NT; ++nt)
        wt[nt] = dequant8_t_bf16(wr.c[nt][j], *reinterpret_cast<const u32x2*>(sst + nt * 128 + 16 * j));
      mma_step(xst, j, wt);
    }
  };

  // ---- main loop over 64-input stages.  Weights are requested kGemmRing - 1 stages ahead into a ring of
  // registers, x slabs kGemmXAhead stages ahead (shared between workgroups, so usually an L2 hit; they pass through LDS: written a stage before use, one barrier
  // per stage): a stage lasts a few hundred nanoseconds, a memory round trip several times that.  The loop is
  // unrolled over the ring so that every register index is a constant; requests past the end are redirected to
  // the last stage rather than branched around, which keeps the compiler's wait counts exact.
  const int n_seg = TR ? a.seg_n : 1;
  for (int sg = 0; sg < n_seg; ++sg) {
  if constexpr (TR) {
    const GemmSeg& g = a.seg[sg];                           // uniform index: scalar loads
    sx = g.x; sldx = g.ldx; sK = g.K; skt = g.k_tiles; spk = g.packed;
    sts = g.ts; sts_ld = g.ts_ld; sext = g.ext_stages; sr = g.r; sB = g.B; sscale = g.tensor_scale;
  }
  int64_t s_begin = 0, s_end = ceil_div_dev(sK, 64);
  if constexpr (SK) {
    if (a.ksplit > 1) {                                     // the launcher leaves no part empty
      const int64_t per = ceil_div_dev(s_end, a.ksplit);
      s_begin = ks * per;
      s_end = s_begin + per < s_end ? s_begin + per : s_end;
    }
  }
  if (s_begin < s_end) {
    constexpr int R = kGemmRing, PX = kGemmXAhead;
    WeightRegs<NT> wring[R];
    u32x4 xring[PX][XL];
    u32x4 scring[PX];
    const int64_t s_last = s_end - 1;
    auto clamp_s = [&](int64_t s) { return s < s_last ? s : s_last; };
#pragma unroll
    for (int p = 0; p < PX; ++p) {
      gload_x(xring[p], sx, sldx, sK, clamp_s(s_begin + p));
      if constexpr (TR) gload_sc(scring[p], clamp_s(s_begin + p));
    }
#pragma unroll
    for (int d = 0; d < R - 1; ++d) gload_w(wring[d], clamp_s(s_begin + d));
    swrite_x(0, xring[0]);
    if constexpr (TR) swrite_sc(0, scring[0]);
    if constexpr (!TR) {
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) wf[nt] = dequant8_bf16(wring[0].c[nt][0], e4m3_byte_f32(wring[0].sc[nt], 0));
    }
    __syncthreads();
    auto stage = [&](int64_t s, int u) {
      gload_x(xring[u % PX], sx, sldx, sK, clamp_s(s + PX));
      if constexpr (TR) gload_sc(scring[u % PX], clamp_s(s + PX));
      gload_w(wring[(u + R - 1) % R], clamp_s(s + R - 1));
      if constexpr (TR) compute_tr(u & 1, wring[u]);
      else compute(u & 1, wring[u], wring[(u + 1) % R]);
      swrite_x((u + 1) & 1, xring[(u + 1) % PX]);
      if constexpr (TR) swrite_sc((u + 1) & 1, scring[(u + 1) % PX]);
      __syncthreads();
    };
    int64_t s = s_begin;
    for (; s + R <= s_end; s += R) {
#pragma unroll
      for (int u = 0; u < R; ++u) stage(s + u, u);
    }
#pragma unroll
    for (int u = 0; u < R - 1; ++u) {
      if (s + u >= s_end) goto main_done;
      stage(s + u, u);
    }
  }
main_done:

  {
    // ---- LoRA up-projection: 3r extra columns  [hi | mid | lo] . [B ; B ; B]^T.  ts already carries
    // the factor lora_scale / S32, so one multiplication by S32 at the end scales both branches.
    const int n_ext = (!SK || ks == 0) ? sext : 0;         // the LoRA columns belong to the first K-part
    if constexpr (SK && W <= 8) {
      if (a.n_prod > 0 && n_ext > 0) {
        // ts comes from the producers of this launch: wait (bounded) until all of them have published it
        uint32_t spins = 0;
        while (__hip_atomic_load(a.ready, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < (uint32_t)(a.p_tbs * a.p_tiles)) {
          if (++spins > kGemmSpinLimit) {   // never reached unless a producer died or was kept off the chip: make it visible
            poisoned = true;
            if (tid == 0) __hip_atomic_fetch_or(a.ready + kCtlErr, 4u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            break;
          }
          __builtin_amdgcn_s_sleep(32);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
      }
    }
    for (int e = 0; e < n_ext; ++e) {
      u32x4 xe[XL];
      gload_x(xe, sts, sts_ld, sts_ld, e);
      swrite_x(0, xe);
      __syncthreads();
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        bf16x8 wf[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
          int64_t row = (int64_t)(nt0 + nt) * 32 + n32;
          row = row < mem.N ? row : mem.N - 1;
          const int c = e * 64 + 16 * j + 8 * kg;
          u32x4 b = {0u, 0u, 0u, 0u};
          if (c < 3 * sr) b = *reinterpret_cast<const u32x4*>(sB + row * sr + (c % sr));
          wf[nt] = __builtin_bit_cast(bf16x8, b);
        }
        mma_step(xs, j, wf);
      }
      __syncthreads();
    }
    if constexpr (TR) {
      // the sums so far are in units of this segment's tensor scale: put them into the next segment's
      if (sg + 1 < n_seg) {
        const float f = *sscale / *a.seg[sg + 1].tensor_scale;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
          for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[mt][nt][i] *= f;
      }
    }
  }
  }   // segments
  if constexpr (SK && W <= 8) {
    if (a.n_prod > 0 && tid == 0) {
      // the last consumer to leave re-arms the hand-over words (every waiting workgroup has passed its wait by then)
      const uint32_t old = __hip_atomic_fetch_add(a.done, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (old == (uint32_t)(a.n_consumers - 1) && __hip_atomic_load(a.ready + kCtlErr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u) {   // (not after a wait that gave up)
        __hip_atomic_store(a.ready, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(a.done, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
  }
  {
    const float S32 = (SK && poisoned) ? __uint_as_float(0x7fc00000u) : *sscale;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const int64_t n = (int64_t)(nt0 + nt) * 32 + n32;
        if constexpr (SK) {
          if (a.ksplit > 1) {                               // this part's sums; gemm_split_reduce_kernel adds the parts and the bias
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              const int64_t m = m0 + mt * 32 + 8 * (i >> 2) + 4 * kg + (i & 3);
              if (m < a.M && n < mem.N) a.kpartial[((int64_t)ks * a.M + m) * a.kp_ld + mem.col0 + n] = acc[mt][nt][i] * S32;
            }
            continue;
          }
        }
        const float bias = (mem.bias && n < mem.N) ? bf16_bits_to_f32(mem.bias[n]) : 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int64_t m = m0 + mt * 32 + 8 * (i >> 2) + 4 * kg + (i & 3);
          if (m < a.M && n < mem.N) mem.y[m * mem.ldy + n] = (uint16_t)f32_to_bf16_bits(acc[mt][nt][i] * S32 + bias);
        }
      }
  }
}

// ---- LoRA down-projection for many tokens: ts = three bf16 terms of (lora_scale / S32) * x A^T --------
// A skinny GEMM (32 output columns per block) that is bound by reading x once.  One workgroup owns 32 tokens and
// one rank tile; its eight waves take the 64-column slabs of its K-part in turn (lora_down_block) and are summed
// through LDS.
__global__ __launch_bounds__(512) void lora_down32_kernel(const GemmArgs a) {
  __shared__ __attribute__((aligned(16))) float red[kLoraDownLdsBytes(1, 8) / sizeof(float)];
  lora_down_block<1, 8>(a, (int)blockIdx.x, (int)blockIdx.y, (int)blockIdx.z, (int)gridDim.z, (int)gridDim.x, (int)gridDim.y, red);
}

// ---- the same product for a few hundred tokens and more ----------------------------------------------
// lora_down32_kernel fetches both operands in MFMA operand layout (one row per lane, 32 bytes of a row per
// instruction), which the memory pipeline serves at a fraction of its rate.  Here a workgroup of four waves owns
// 64 tokens, all rank tiles of all adapters of the launch and K-part blockIdx.y: x and A slabs of 64 columns are
// fetched row-contiguously (eight lanes per 128-byte row segment), three or four slabs ahead through a register ring, and
// handed to the MFMA operand layout through LDS (double buffered, one barrier per slab, the row-XOR swizzle of the
// GEMM above).  Wave w owns token half w & 1 and the rank tiles (w >> 1), (w >> 1) + 2, ...: no sums across waves.
// K-parts meet in the workspace as in lora_down_block: the workgroup that arrives last adds them in part order.
// The adapters come in the group form of GemmArgs (g_*); ts as lora_down_block writes it.
template <int TPW>   // rank tiles per wave
__global__ __launch_bounds__(256) void lora_down64_kernel(const GemmArgs a, const int n_tiles, const int P) {
  constexpr int T = 2 * TPW;                      // rank tiles held in LDS (the last one a repeat when n_tiles is odd)
  constexpr int kXChunks = 64 * 8, kAChunks = T * 32 * 8;
  extern __shared__ u32x4 lds64[];                // [2][x slab | A slab]
  __shared__ uint32_t s_old;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n32 = lane & 31, kg = lane >> 5;
  const int mt = wave & 1, t_first = wave >> 1;
  const int tb = blockIdx.x, bz = blockIdx.y;
  const int64_t m0 = (int64_t)tb * 64;
  const int64_t part_cols = ceil_div_dev(ceil_div_dev(a.K, 64), P) * 64;
  const int64_t k_lo = (int64_t)bz * part_cols;
  const int64_t k_hi = k_lo + part_cols < a.K ? k_lo + part_cols : a.K;
  const int n_slabs = k_hi > k_lo ? (int)ceil_div_dev(k_hi - k_lo, 64) : 0;

  // the adapter that owns rank tile t (uniform), and the tile's index inside it
  auto member_of = [&](int t) {
    int mi = 0;
#pragma unroll
    for (int i = 1; i < kMaxGroup; ++i) mi = (i < a.g_n && t >= a.g_tile0[i]) ? i : mi;
    return mi;
  };
  // ---- loaders: thread tid fetches chunk tid & 7 of row tid >> 3 (+ 32 per further request)
  const int lrow = tid >> 3, lchunk = tid & 7;
  const uint16_t* xsrc[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    int64_t m = m0 + lrow + 32 * i;
    m = m < a.M ? m : a.M - 1;
    xsrc[i] = a.x + m * a.ldx;
  }
  const uint16_t* asrc[T];
#pragma unroll
  for (int i = 0; i < T; ++i) {
    const int t = i < n_tiles ? i : n_tiles - 1;
    int mi = member_of(t);
    const uint16_t* A = a.g_A[0];
    int rN = a.g_r[0], t0 = a.g_tile0[0];
#pragma unroll
    for (int j = 1; j < kMaxGroup; ++j)
      if (mi == j) { A = a.g_A[j]; rN = a.g_r[j]; t0 = a.g_tile0[j]; }
    int row = (t - t0) * 32 + lrow;
    row = row < rN ? row : rN - 1;
    asrc[i] = A + (int64_t)row * a.K;
  }
  struct Slab { u32x4 x[2]; u32x4 w[T]; bool in; };
  // slabs past the part's end contribute nothing: their x is zeroed on its way to LDS (the address is redirected
  // into the row; nothing here touches the loaded value, which would wait for it)
  auto load = [&](Slab& sl, int s) {
    int64_t k = k_lo + (int64_t)s * 64 + lchunk * 8;
    sl.in = k < k_hi;
    k = k < a.K - 8 ? k : a.K - 8;
#pragma unroll
    for (int i = 0; i < 2; ++i) sl.x[i] = *reinterpret_cast<const u32x4*>(xsrc[i] + k);
#pragma unroll
    for (int i = 0; i < T; ++i) sl.w[i] = *reinterpret_cast<const u32x4*>(asrc[i] + k);
  };
  auto to_lds = [&](int buf, const Slab& sl) {
    u32x4* base = lds64 + buf * (kXChunks + kAChunks);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int row = lrow + 32 * i;
      base[row * 8 + (lchunk ^ ((row >> 1) & 7))] = sl.in ? sl.x[i] : u32x4{0u, 0u, 0u, 0u};
    }
#pragma unroll
    for (int i = 0; i < T; ++i) {
      const int row = lrow + 32 * i;
      base[kXChunks + row * 8 + (lchunk ^ ((row >> 1) & 7))] = sl.w[i];
    }
  };
  f32x16 acc[TPW];
#pragma unroll
  for (int i = 0; i < TPW; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
  auto compute = [&](int buf) {
    const u32x4* base = lds64 + buf * (kXChunks + kAChunks);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int xrow = mt * 32 + n32;
      const bf16x8 xf = __builtin_bit_cast(bf16x8, base[xrow * 8 + ((2 * j + kg) ^ ((xrow >> 1) & 7))]);
#pragma unroll
      for (int i = 0; i < TPW; ++i) {
        const int arow = (t_first + 2 * i) * 32 + n32;
        const bf16x8 af = __builtin_bit_cast(bf16x8, base[kXChunks + arow * 8 + ((2 * j + kg) ^ ((arow >> 1) & 7))]);
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xf, af, acc[i], 0, 0, 0);
      }
    }
  };

  // ---- main loop: whole rounds of the ring, the last one padded with empty slabs
  {
    constexpr int D = TPW == 4 ? 3 : 4;   // slabs in flight per thread (registers)
    Slab ring[D];
#pragma unroll
    for (int d = 0; d < D; ++d) load(ring[d], d);
    for (int s0 = 0; s0 < n_slabs; s0 += D) {
#pragma unroll
      for (int u = 0; u < D; ++u) {
        const int buf = (s0 + u) & 1;   // consecutive slabs alternate (D may be odd)
        to_lds(buf, ring[u]);
        __builtin_amdgcn_sched_barrier(0);   // the requests stay here, D slabs ahead of their use
        load(ring[u], s0 + u + D);
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        compute(buf);
      }
    }
  }

  // ---- K-parts: every part leaves its sums in the workspace (written through to memory before the workgroup's
  // arrival is counted); the workgroup that arrives last adds all parts in part order and goes on.
  if (P > 1) {
    constexpr int kWgFloats = 4 * TPW * 16 * 64;
    const int64_t part_stride = (int64_t)gridDim.x * kWgFloats;
    uint32_t* mine = a.tpart + (int64_t)bz * part_stride + (int64_t)tb * kWgFloats + wave * (TPW * 16 * 64) + lane;
#pragma unroll
    for (int i = 0; i < TPW; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e)
        __hip_atomic_store(mine + (i * 16 + e) * 64, __float_as_uint(acc[i][e]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    __syncthreads();
    if (tid == 0) s_old = __hip_atomic_fetch_add(a.counters + tb, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (s_old != (uint32_t)(P - 1)) return;
    const uint32_t* all = a.tpart + (int64_t)tb * kWgFloats + wave * (TPW * 16 * 64) + lane;
#pragma unroll
    for (int i = 0; i < TPW; ++i) {
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
      for (int z0 = 0; z0 < P; z0 += kDownMaxParts) {   // in part order, eight parts requested together
        uint32_t v[kDownMaxParts][16];
#pragma unroll
        for (int z = 0; z < kDownMaxParts; ++z)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            v[z][e] = 0u;
            if (z0 + z < P) v[z][e] = __hip_atomic_load(all + (int64_t)(z0 + z) * part_stride + (i * 16 + e) * 64, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          }
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          float sum = acc[i][e];
#pragma unroll
          for (int z = 0; z < kDownMaxParts; ++z) sum += __uint_as_float(v[z][e]);
          acc[i][e] = sum;
        }
        __builtin_amdgcn_sched_barrier(0);   // one tile's 128 values at a time in registers
      }
    }
    if (tid == 0) __hip_atomic_store(a.counters + tb, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next call
  }

  // ---- ts = three bf16 terms of (lora_scale / S32) * sum, per adapter
#pragma unroll
  for (int i = 0; i < TPW; ++i) {
    const int t = t_first + 2 * i;
    if (t >= n_tiles) continue;
    const int mi = member_of(t);
    uint16_t* ts = const_cast<uint16_t*>(a.g_ts[0]);
    int64_t ts_ld = a.g_ts_ld[0];
    int rN = a.g_r[0], t0 = a.g_tile0[0];
    float lora_scale = a.g_lora_scale[0];
    const float* tensor_scale = a.g_tensor_scale[0];
#pragma unroll
    for (int j = 1; j < kMaxGroup; ++j)
      if (mi == j) {
        ts = const_cast<uint16_t*>(a.g_ts[j]); ts_ld = a.g_ts_ld[j]; rN = a.g_r[j]; t0 = a.g_tile0[j];
        lora_scale = a.g_lora_scale[j]; tensor_scale = a.g_tensor_scale[j];
      }
    const float t_mult = lora_scale / *tensor_scale;   // undone by the final * S32 of the main launch
    const int n = (t - t0) * 32 + n32;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int64_t m = m0 + mt * 32 + 8 * (e >> 2) + 4 * kg + (e & 3);
      if (m < a.M && n < rN) {
        const float v = acc[i][e] * t_mult;
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
    if (t == t0) {   // the adapter's first tile: zero the padding columns [3 r, ts_ld) of this wave's 32 tokens
      const int pad = (int)(ts_ld - 3 * rN);
      for (int idx = lane; idx < 32 * pad; idx += 64) {
        const int64_t m = m0 + mt * 32 + idx / pad;
        if (m < a.M) ts[m * ts_ld + 3 * rN + idx % pad] = 0;
      }
    }
  }
}

// ---- K split over workgroups: y = bf16(sum over parts, in part order, + bias) ------------------------------
struct GemmReduceArgs {
  const float* partial; int S; int64_t M, ld; int n;
  int64_t col0[kMaxGroup], N[kMaxGroup], ldy[kMaxGroup]; uint16_t* y[kMaxGroup]; const uint16_t* bias[kMaxGroup];
};
// one thread per four consecutive columns of a row (every member's columns start at a multiple of four)
__global__ __launch_bounds__(256) void gemm_split_reduce_kernel(const GemmReduceArgs a) {
  const int64_t quads = a.ld / 4, total = a.M * quads;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int64_t m = i / quads, c = (i - m * quads) * 4;
    int mi = 0;
#pragma unroll
    for (int j = 1; j < kMaxGroup; ++j) mi = (j < a.n && c >= a.col0[j]) ? j : mi;
    f32x4 sum = {0.f, 0.f, 0.f, 0.f};
    for (int z = 0; z < a.S; ++z) {
      const f32x4 v = *reinterpret_cast<const f32x4*>(a.partial + ((int64_t)z * a.M + m) * a.ld + c);
      sum[0] += v[0]; sum[1] += v[1]; sum[2] += v[2]; sum[3] += v[3];
    }
    int64_t col0 = a.col0[0], N = a.N[0], ldy = a.ldy[0];
    uint16_t* y = a.y[0];
    const uint16_t* bias = a.bias[0];
#pragma unroll
    for (int j = 1; j < kMaxGroup; ++j)
      if (mi == j) { col0 = a.col0[j]; N = a.N[j]; ldy = a.ldy[j]; y = a.y[j]; bias = a.bias[j]; }
    const int64_t n0 = c - col0;
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (n0 + e < N) y[m * ldy + n0 + e] = (uint16_t)f32_to_bf16_bits(sum[e] + (bias ? bf16_bits_to_f32(bias[n0 + e]) : 0.f));
  }
}

// ---- host ------------------------------------------------------------------------------------------

struct GemmConfig { int MT, NT, W, wg_per_cu; float quality, quality_shared, quality_rounds; };
// wg_per_cu: workgroups of this shape that fit one CU (register use).  Relative speeds at equal useful work,
// measured on 7B / 14B / 32B-shaped layers at 192..4096 tokens: quality when every workgroup has a CU of its own
// (at most 256 of them), quality_shared when a single round puts two on a CU, quality_rounds when the launch takes
// several rounds.  The one-tile-per-wave shapes hide the conversions behind more waves but re-read x more often.
static const GemmConfig kConfigs[] = {
    {4, 2, 4, 1, 0.72f, 0.72f, 0.72f}, {4, 2, 5, 1, 0.75f, 0.75f, 0.75f}, {4, 2, 8, 1, 1.00f, 1.00f, 1.00f},
    {4, 1, 4, 2, 0.95f, 0.84f, 0.85f}, {4, 1, 8, 2, 0.95f, 0.93f, 0.95f},
    {4, 1, 10, 1, 0.90f, 0.90f, 0.86f},   // 320 output rows per workgroup, ten waves: N = 5120 in one full round
};
static int g_force_cfg = -1;
static bool g_split = true;   // whole rounds and remainder as two launches when that is estimated faster
static int g_force_ksplit = 0;   // tuning: K-parts of the forward launch (0 = automatic, 1 = never)
static int g_fuse_max_tokens = 512;   // up to here the LoRA down-projections run inside the forward launch
static int g_fuse_wgs = 256;          // producer workgroups aimed at (K-parts until there are that many)
constexpr int kGemmMaxKsplit = 8;
constexpr int kGemmMinSplitStages = 8;   // a K-part is at least 512 inputs

// The partial outputs' row length: every member's columns padded to a multiple of four
static int64_t split_ld(const GemmMember* m, int n) {
  int64_t ld = 0;
  for (int i = 0; i < n; ++i) ld += (m[i].N + 3) / 4 * 4;
  return ld;
}
// Shapes worth a K split: fewer than two rounds of 128 x 128 tiles.  The bound covers any member count's padding.
size_t gemm_split_bytes(int64_t M, int64_t N_total) {
  if (M < 1 || N_total < 1 || ceil_div(M, 128) * ceil_div(N_total, 128) >= 512) return 0;
  const size_t b = (size_t)kGemmMaxKsplit * (size_t)M * (size_t)(N_total + 4 * kMaxGroup) * sizeof(float);
  return b < kGemmSplitCap ? (b + 255) & ~(size_t)255 : kGemmSplitCap;
}

template <int MT, int NT, int W, bool TR = false>
static int launch_cfg(const GemmArgs& a, hipStream_t st) {
  constexpr size_t lds_tiles = 2 * (size_t)MT * 32 * 8 * sizeof(u32x4) + (TR ? 2 * (size_t)W * NT * 128 : 0);
  constexpr size_t lds_prod = (TR || W > 8) ? 0 : kLoraDownLdsBytes(1, W);   // what a producer workgroup of the few-token variant needs
  const size_t lds = (a.n_prod > 0 && lds_prod > lds_tiles) ? lds_prod : lds_tiles;
  GemmArgs b = a;
  b.n_blocks = 0;
  for (int i = 0; i < b.m_n; ++i) {
    b.m[i].block_begin = b.n_blocks;
    b.n_blocks += (int)ceil_div(b.m[i].n_tiles, W * NT);
  }
  b.nblk_per_xcd = (int)ceil_div(b.n_blocks, 8);
  const int64_t m_blocks = ceil_div(a.M, MT * 32);
  b.m_blocks = (int)m_blocks;
  if (TR || b.ksplit < 2) b.ksplit = 1;
  if (TR || W > 8) b.n_prod = 0;   // (launch_gemm has run the down-projection by itself then)
  b.n_consumers = (int)(b.n_blocks * m_blocks * b.ksplit);
  const dim3 grid((unsigned)(b.n_prod + 8 * b.nblk_per_xcd * m_blocks * b.ksplit));
  if constexpr (!TR) {
    if (b.ksplit > 1 || b.n_prod > 0) gemm32_kernel<MT, NT, W, false, true><<<grid, W * 64, lds, st>>>(b);
    else gemm32_kernel<MT, NT, W, false, false><<<grid, W * 64, lds, st>>>(b);
  } else {
    gemm32_kernel<MT, NT, W, true, false><<<grid, W * 64, lds, st>>>(b);
  }
  int rc = launch_status();
  if (rc != QERL_OK || b.ksplit == 1) return rc;
  GemmReduceArgs r{};
  r.partial = b.kpartial; r.S = b.ksplit; r.M = b.M; r.ld = b.kp_ld; r.n = b.m_n;
  for (int i = 0; i < b.m_n; ++i) {
    r.col0[i] = b.m[i].col0; r.N[i] = b.m[i].N; r.ldy[i] = b.m[i].ldy; r.y[i] = b.m[i].y; r.bias[i] = b.m[i].bias;
  }
  int64_t blocks = ceil_div(b.M * (b.kp_ld / 4), 256);
  blocks = blocks > 4096 ? 4096 : blocks;
  gemm_split_reduce_kernel<<<dim3((unsigned)blocks), 256, 0, st>>>(r);
  return launch_status();
}

int launch_gemm(const GemmArgs& a0, hipStream_t st) {
  GemmArgs a = a0;
  if (a.m_n == 0) {   // a single linear, described by the top-level fields
    a.m_n = 1;
    a.m[0] = GemmMember{a.packed, a.tensor_scale, a.N, a.n_tiles, a.ts, a.ts_ld, a.ext_stages, a.B, a.r, a.bias, a.y, a.ldy, 0};
  }
  // every pointer the kernel dereferences must be set by the caller
  if (!a.x || a.m_n < 1 || a.m_n > kMaxGroup || a.M < 1 || a.K < (a.transposed ? 8 : 16) || a.k_tiles < 1) return QERL_ERR_SHAPE;
  for (int i = 0; i < a.m_n; ++i) {
    const GemmMember& m = a.m[i];
    if (!m.packed || !m.tensor_scale || !m.y || (m.r > 0 && (!m.ts || !m.B))) return QERL_ERR_NULL;
    if (m.N < 1 || m.n_tiles < 1 || m.ldy < m.N || m.r < 0 || (m.r > 0 && m.ts_ld < 3 * m.r) ||
        m.ext_stages * 64 < 3 * m.r || (int64_t)m.ext_stages * 64 > (m.r > 0 ? m.ts_ld : 0))
      return QERL_ERR_SHAPE;
  }
  // Estimated time of every eligible shape, in units of one output element's K-loop on a fully used chip at
  // quality 1: rounds x slots x tile area / quality.
  const int n_cfg = (int)(sizeof(kConfigs) / sizeof(kConfigs[0]));
  // The LoRA down-projections of the launch (a.n_prod < 0: described by the g_* fields, not run yet): with few tokens
  // they ride as the first workgroups of the main launch, hidden behind its K-loop; otherwise, and for the shape
  // of ten waves, they get their launch here.
  int64_t prod_wgs = 0;
  const bool fuse_wanted = a.n_prod < 0 && !a.transposed && a.g_n > 0 && a.ready && a.done && a.M <= g_fuse_max_tokens;
  if (fuse_wanted) {
    a.p_tbs = (int)ceil_div(a.M, 32); a.p_tiles = a.g_tile0[a.g_n];
    const int64_t base_wgs = (int64_t)a.p_tbs * a.p_tiles;
    int64_t P = (a.tpart && a.counters && base_wgs < g_fuse_wgs) ? g_fuse_wgs / base_wgs : 1;
    const int64_t p_max = ceil_div(a.K, 512);
    P = P < p_max ? P : p_max;
    P = P > kDownMaxPartsWide ? kDownMaxPartsWide : (P < 1 ? 1 : P);
    a.p_parts = (int)P;
    prod_wgs = ceil_div(base_wgs * P, 8) * 8;
  }
  auto cfg_time = [&](int c, const GemmMember* m, int n, int S = 1) {
    const GemmConfig& g = kConfigs[c];
    const int64_t bm = g.MT * 32, bn = (int64_t)g.W * g.NT * 32;
    int64_t col_blocks = 0;
    for (int i = 0; i < n; ++i) col_blocks += ceil_div(m[i].N, bn);
    const int64_t wgs = ceil_div(a.M, bm) * col_blocks * S + prod_wgs;     // S K-parts: S times the workgroups, each 1 / S of the K-loop
    const bool alone = wgs <= 256;                              // every workgroup gets a CU of its own
    const int64_t slots = alone ? 256 : 256 * g.wg_per_cu;
    const int64_t rounds = ceil_div(wgs, slots);
    const float q = rounds > 1 ? g.quality_rounds : alone ? g.quality : g.quality_shared;
    return (double)rounds * (double)slots * (double)bm * (double)bn / q / (double)S;
  };
  auto best_cfg = [&](const GemmMember* m, int n, double& t_best) {
    int best = -1;
    for (int c = 0; c < n_cfg; ++c) {
      if (a.transposed && c != 2 && c != 5) continue;   // the backward pass is instantiated for two shapes
      if (fuse_wanted && kConfigs[c].W > 8) continue;    // the producers' reduction needs LDS per wave
      const double t = cfg_time(c, m, n);
      if (best < 0 || t < t_best) { t_best = t; best = c; }
    }
    return best;
  };
  double t_single = 0;
  int best = best_cfg(a.m, a.m_n, t_single);
  if (a.transposed) {
    if (a.m_n != 1 || a.seg_n < 0 || a.seg_n > kMaxGroup) return QERL_ERR_SHAPE;
    if (a.seg_n == 0) {   // one segment: the launch's x and the member's tiles
      const GemmMember& m = a.m[0];
      a.seg_n = 1;
      a.seg[0] = GemmSeg{a.x, a.ldx, a.K, m.packed, a.k_tiles, m.tensor_scale, m.ts, m.ts_ld, m.ext_stages, m.B, m.r};
    }
    for (int i = 0; i < a.seg_n; ++i) {
      const GemmSeg& g = a.seg[i];
      if (!g.x || !g.packed || !g.tensor_scale || (g.r > 0 && (!g.ts || !g.B))) return QERL_ERR_NULL;
      if (g.K < 8 || g.ldx < g.K || g.k_tiles < 1 || g.r < 0 || (g.r > 0 && g.ts_ld < 3 * g.r) || g.ext_stages * 64 < 3 * g.r ||
          (int64_t)g.ext_stages * 64 > (g.r > 0 ? g.ts_ld : 0))
        return QERL_ERR_SHAPE;
    }
  }
  if (a.transposed) return best == 5 ? launch_cfg<4, 1, 10, true>(a, st) : launch_cfg<4, 2, 8, true>(a, st);
  if (g_force_cfg >= 0) best = g_force_cfg;
  // K split over workgroups when the tiles alone leave most of the chip idle.  In the units above one microsecond is
  // about 5.6e8 / K; a split costs every workgroup its pipeline fill once more per part, and the second launch.
  a.ksplit = 1;
  if (a.kpartial && g_force_ksplit != 1) {
    const int64_t ld = split_ld(a.m, a.m_n), n_stages = ceil_div(a.K, 64);
    const double us = 5.6e8 / (double)a.K;
    double t_best = t_single;
    for (int c = 0; c < n_cfg; ++c) {
      if (g_force_cfg >= 0 && c != g_force_cfg) continue;
      if (fuse_wanted && kConfigs[c].W > 8) continue;
      for (int S = 2; S <= kGemmMaxKsplit; ++S) {
        if (g_force_ksplit > 1 && S != g_force_ksplit) continue;
        const int64_t per = ceil_div(n_stages, S);
        if (per < kGemmMinSplitStages || per * (S - 1) >= n_stages) continue;       // parts too short, or an empty last part
        const size_t bytes = (size_t)S * (size_t)a.M * (size_t)ld * sizeof(float);
        if (bytes > a.kpartial_bytes) continue;
        const double t = cfg_time(c, a.m, a.m_n, S) + (4.0 + (double)bytes / 3.0e6) * us +      // the second launch: its gap, S reads and one write
                         2.0 * us * (double)(S - 1) / (double)S;
        if (t < t_best || (g_force_ksplit > 1 && a.ksplit == 1)) { t_best = t; best = c; a.ksplit = S; }
      }
    }
    if (a.ksplit > 1) {
      a.kp_ld = ld;
      int64_t col = 0;
      for (int i = 0; i < a.m_n; ++i) { a.m[i].col0 = col; col += (a.m[i].N + 3) / 4 * 4; }
    }
  }
  if (a.n_prod < 0) {
    // measured on 32B shapes at 128 and 256 tokens: worth it where K is split because the tiles alone leave the chip
    // idle (q + k + v 69 -> 49 us, o 45 -> 37, down 92 -> 82 at 128 tokens); a launch that fills the chip by itself
    // (gate + up) only loses its first slots to the producers (193 -> 240 us at 256 tokens)
    bool fuse = fuse_wanted && kConfigs[best].W <= 8 && a.ksplit > 1;
    if (fuse) {   // everything resident at once: the consumers wait for the producers
      const GemmConfig& g = kConfigs[best];
      int64_t col_blocks = 0;
      for (int i = 0; i < a.m_n; ++i) col_blocks += ceil_div(a.m[i].N, (int64_t)g.W * g.NT * 32);
      fuse = ceil_div(a.M, g.MT * 32) * col_blocks * a.ksplit + prod_wgs <= 256 * (int64_t)g.wg_per_cu;
    }
    if (fuse) {
      a.n_prod = (int)prod_wgs;
    } else {
      GemmArgs dn = a;
      dn.ready = nullptr;
      const int rc = launch_lora_down_gemm(dn, st);
      if (rc != QERL_OK) return rc;
      a.n_prod = 0;
    }
  }
  auto launch_one = [&](int c, const GemmArgs& b) -> int {
#define QERL_GEMM_CASE(idx, mt, nt, w) \
    if (c == idx) return launch_cfg<mt, nt, w>(b, st);
    QERL_GEMM_CASE(0, 4, 2, 4) QERL_GEMM_CASE(1, 4, 2, 5) QERL_GEMM_CASE(2, 4, 2, 8)
    QERL_GEMM_CASE(3, 4, 1, 4) QERL_GEMM_CASE(4, 4, 1, 8) QERL_GEMM_CASE(5, 4, 1, 10)
#undef QERL_GEMM_CASE
    return QERL_ERR_SHAPE;
  };
  // A launch of several rounds whose last round is partly empty: the whole rounds go out in one shape,
  // the remaining columns as a launch of their own in whatever shape suits them (smaller tiles fill the chip
  // where a part round of large ones would leave CUs idle).  A member cut by the boundary appears in both
  // launches; the second sees it from a row-tile offset on (the packed tiles of 32 rows are contiguous per row tile).
  if (g_split && g_force_cfg < 0 && a.ksplit == 1 && a.n_prod == 0) {
    // ~15 us in the units above: the gap between the launches, the second one's fill and drain
    const double overhead = 8.4e9 / (double)a.K;
    double t_split = 0.97 * t_single;   // what a pair of launches has to beat
    int c_main = -1, c_rem = -1;
    GemmArgs main_args, rem_args;
    for (int c1 = 0; c1 < n_cfg; ++c1) {
      const GemmConfig& g = kConfigs[c1];
      const int64_t bm = g.MT * 32, bn = (int64_t)g.W * g.NT * 32, tiles_per_block = (int64_t)g.W * g.NT;
      int64_t col_blocks = 0;
      for (int i = 0; i < a.m_n; ++i) col_blocks += ceil_div(a.m[i].N, bn);
      const int64_t m_blocks = ceil_div(a.M, bm), wgs = m_blocks * col_blocks, slots = 256 * (int64_t)g.wg_per_cu;
      const int64_t whole = wgs / slots;
      int64_t c_blocks = whole * slots / m_blocks;             // column blocks of the whole rounds
      if (whole < 1 || wgs % slots == 0 || c_blocks < 1 || c_blocks >= col_blocks) continue;
      GemmArgs ma = a, ra = a;
      ma.m_n = ra.m_n = 0;
      for (int i = 0; i < a.m_n; ++i) {
        const GemmMember& m = a.m[i];
        const int64_t cb = ceil_div(m.N, bn);
        const int64_t take = c_blocks < cb ? c_blocks : cb;    // this member's column blocks in the first launch
        c_blocks -= take;
        if (take > 0) {
          GemmMember& d = ma.m[ma.m_n++];
          d = m;
          if (take < cb) { d.N = take * bn; d.n_tiles = (int)(take * tiles_per_block); }
        }
        if (take < cb) {
          GemmMember& d = ra.m[ra.m_n++];
          d = m;
          const int64_t t0 = take * tiles_per_block, row0 = t0 * 32;
          d.packed = m.packed + t0 * a.k_tiles * kPackTileBytes;
          d.N = m.N - row0; d.n_tiles = m.n_tiles - (int)t0;
          if (m.B) d.B = m.B + row0 * m.r;
          if (m.bias) d.bias = m.bias + row0;
          d.y = m.y + row0;
        }
      }
      double t_rem = 0;
      const int cr = best_cfg(ra.m, ra.m_n, t_rem);
      const double t = cfg_time(c1, ma.m, ma.m_n) + t_rem + overhead;
      if (t < t_split) { t_split = t; c_main = c1; c_rem = cr; main_args = ma; rem_args = ra; }
    }
    if (c_main >= 0) {
      const int rc = launch_one(c_main, main_args);
      return rc != QERL_OK ? rc : launch_one(c_rem, rem_args);
    }
  }
  return launch_one(best, a);
}

// ts = three-term bf16 split of (lora_scale / S32) * x A^T, [M, ts_ld]; a.N = r rows of A.
// Token counts from which the 64-token kernel takes over
static int g_down64_min_tokens = 256;
static int g_down64_parts = 0;   // tuning: force the number of K-parts (0 = automatic)

template <int TPW>
static int launch_down64_t(const GemmArgs& a, int n_tiles, int P, dim3 grid, hipStream_t st) {
  constexpr size_t lds = 2 * ((size_t)64 * 8 + (size_t)2 * TPW * 32 * 8) * sizeof(u32x4);   // up to 80 KB
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&lora_down64_kernel<TPW>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
      return launch_status();
    attr_set = true;
  }
  lora_down64_kernel<TPW><<<grid, 256, lds, st>>>(a, n_tiles, P);
  return launch_status();
}

static int launch_lora_down64(const GemmArgs& a0, hipStream_t st) {
  GemmArgs a = a0;
  if (a.g_n == 0) {   // a single adapter, put into the group form
    a.g_n = 1;
    a.g_tile0[0] = 0; a.g_tile0[1] = (int)ceil_div(a.N, 32);
    a.g_A[0] = a.wbf16; a.g_ts[0] = a.ts; a.g_ts_ld[0] = a.ts_ld; a.g_r[0] = (int)a.N;
    a.g_lora_scale[0] = a.lora_scale; a.g_tensor_scale[0] = a.tensor_scale;
  }
  const int n_tiles = a.g_tile0[a.g_n];
  const int tpw = (n_tiles + 1) / 2;
  const int64_t tbs = ceil_div(a.M, 64);
  // K-parts until the chip is full (twice over for a single adapter, whose parts exchange little): at most 32,
  // at least 512 columns each, one arrival counter per token block, and the parts' sums must fit the exchange area
  int64_t P = 1;
  if (a.tpart && a.counters && tbs <= kDownMaxSlots) {
    P = (tpw == 1 ? 512 : 256) / tbs;
    const int64_t p_max = ceil_div(a.K, 512);
    P = P < p_max ? P : p_max;
    P = P > kDownMaxPartsWide ? kDownMaxPartsWide : (P < 1 ? 1 : P);
    if (g_down64_parts > 0) P = g_down64_parts;
    while (P > 1 && (size_t)(tbs * P) * 4 * tpw * 16 * 64 * sizeof(float) > kDownExchangeBytes) --P;
  }
  const dim3 grid((unsigned)tbs, (unsigned)P);
  if (tpw == 1) return launch_down64_t<1>(a, n_tiles, (int)P, grid, st);
  if (tpw == 2) return launch_down64_t<2>(a, n_tiles, (int)P, grid, st);
  if (tpw == 3) return launch_down64_t<3>(a, n_tiles, (int)P, grid, st);
  if (tpw == 4) return launch_down64_t<4>(a, n_tiles, (int)P, grid, st);
  return QERL_ERR_SHAPE;
}

int launch_lora_down_gemm(const GemmArgs& a, hipStream_t st) {
  if (a.g_n > 0) {   // several adapters reading the same x: one 32-row tile per workgroup
    if (!a.x || a.g_n > kMaxGroup || a.M < 1 || a.K < 8) return QERL_ERR_SHAPE;
    int tiles = 0;
    for (int i = 0; i < a.g_n; ++i) {
      if (!a.g_A[i] || !a.g_ts[i] || !a.g_tensor_scale[i]) return QERL_ERR_NULL;
      if (a.g_r[i] < 1 || a.g_ts_ld[i] < 3 * a.g_r[i] || a.g_tile0[i] != tiles) return QERL_ERR_SHAPE;
      tiles += (int)ceil_div(a.g_r[i], 32);
    }
    if (a.g_tile0[a.g_n] != tiles) return QERL_ERR_SHAPE;
    if (a.M >= g_down64_min_tokens && tiles <= 8 && a.K % 8 == 0) return launch_lora_down64(a, st);
    int64_t P = 1;
    const int64_t base_wgs = ceil_div(a.M, 32) * tiles;
    if (a.tpart && a.counters && base_wgs < 32) {
      P = 64 / base_wgs;
      const int64_t p_max = ceil_div(a.K, 512);
      P = P < p_max ? P : p_max;
      P = P > kDownMaxParts ? kDownMaxParts : (P < 1 ? 1 : P);
    }
    lora_down32_kernel<<<dim3((unsigned)ceil_div(a.M, 32), (unsigned)tiles, (unsigned)P), 512, 0, st>>>(a);
    return launch_status();
  }
  if (!a.x || !a.wbf16 || !a.tensor_scale || !a.ts) return QERL_ERR_NULL;
  if (a.M < 1 || a.N < 1 || a.K < 8 || a.ts_ld < 3 * a.N) return QERL_ERR_SHAPE;
  const int tiles = (int)ceil_div(a.N, 32);
  if (a.M >= g_down64_min_tokens && tiles <= 8 && a.K % 8 == 0) return launch_lora_down64(a, st);
  // While token blocks x rank tiles do not fill the chip, K is split over workgroups (up to eight parts, at
  // least 512 columns each, at most kDownMaxSlots workgroups) when the caller provides the exchange area.
  // (More and shorter parts were tried for 96..255 tokens: 41 -> 32 us for K = 27648, 19 -> 22 us for K = 5120, and
  // 1 % lost on the 7B steps at 32 and 64 tokens; those shapes now carry the down-projection inside the GEMM launch.)
  int64_t P = 1;
  const int64_t base_wgs = ceil_div(a.M, 32) * tiles;
  if (a.tpart && a.counters && base_wgs <= kDownMaxSlots / 2) {
    P = (base_wgs < 32 ? 64 : kDownMaxSlots) / base_wgs;   // a few dozen workgroups for a few tokens, one per CU otherwise
    const int64_t p_max = ceil_div(a.K, 512);
    P = P < p_max ? P : p_max;
    P = P > kDownMaxParts ? kDownMaxParts : (P < 1 ? 1 : P);
  }
  const dim3 grid((unsigned)ceil_div(a.M, 32), (unsigned)tiles, (unsigned)P);
  lora_down32_kernel<<<grid, 512, 0, st>>>(a);
  return launch_status();
}

}  // namespace qerl

// Tuning hook for experiments (not part of the public header): force a GEMM tile configuration, -1 = automatic.
#ifdef QERL_TUNING_HOOKS   // built only for tuning sessions: they change process-wide state
extern "C" QERL_API void qerl_debug_force_gemm(int cfg) { qerl::g_force_cfg = cfg; }
extern "C" QERL_API void qerl_debug_gemm_split(int on) { qerl::g_split = on != 0; }
extern "C" QERL_API void qerl_debug_gemm_ksplit(int s) { qerl::g_force_ksplit = s; }
extern "C" QERL_API void qerl_debug_gemm_fuse_max_tokens(int m) { qerl::g_fuse_max_tokens = m; }
extern "C" QERL_API void qerl_debug_gemm_fuse_wgs(int n) { qerl::g_fuse_wgs = n; }
extern "C" QERL_API void qerl_debug_down64_min_tokens(int m) { qerl::g_down64_min_tokens = m; }
extern "C" QERL_API void qerl_debug_down64_parts(int p) { qerl::g_down64_parts = p; }
#endif  // QERL_TUNING_HOOKS
