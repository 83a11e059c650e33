// Backward pass of the NVFP4 + LoRA linear: only the adapters are trained, the gradient flows through the
// frozen quantised weights (Preliminary, "Low-rank Adaptation"; Eq. 2, Eq. 6).  For an upstream dY [M, N]:
//
//   dX = dY W_hat + s (dY B) A          [M, K]  bf16
//   dA = s (dY B)^T x                   [r, K]  fp32
//   dB = s dY^T (x A^T)                 [N, r]  fp32          (s = lora_scale)
//
// dX contracts over N, i.e. over the ROWS of the packed weight tiles, so the same bytes are needed in a second,
// transposed tile order (nvfp4_prepack_t; the weights are frozen, the order is made once):
//   tile (kt, nt) = 32 inputs k = 32 kt .. + 31  x  128 rows n = 128 nt .. + 127, 2304 bytes like the forward tile:
//   two 1 KiB planes of codes (plane p = rows 64 p .. 64 p + 63; lane l = (c = l % 32, g = l / 32) owns 16 bytes:
//   dword j holds the codes of rows 64 p + 16 j + 8 g .. + 7 at input 32 kt + c, nibble i = row + i), then 256 scale
//   bytes [plane][input block 0..1][64 rows].  Tiles of one kt are consecutive along nt.
// gemm32_kernel<.., TR = true> multiplies dY with it (the eight weights of a lane and step carry eight different
// E4M3 scales; products stay exact in bf16), the LoRA term enters as 3r more contraction columns exactly as in
// the forward pass with the roles of A and B exchanged (both transposed once per call: they change with every
// optimiser step).  dA and dB are skinny products over the token dimension (MFMA, operands transposed through LDS),
// tokens split over a few workgroups whose partial sums are added in order.
// Several linears that read the same x (q / k / v, gate / up: Section 3.3) go through one call: dX is the sum of the
// members' terms, formed by ONE launch of the transposed GEMM whose contraction runs over the members' rows one
// after the other (fp32 throughout, one rounding), and the down-projections of x for all adapters share a launch.
#include "linear.hpp"

namespace qerl {

// ---- transposed tile order -----------------------------------------------------------------------------
__global__ __launch_bounds__(256) void prepack_t_kernel(const uint8_t* __restrict__ codes, const uint8_t* __restrict__ scales,
                                                        int64_t N, int64_t K, int64_t k_tiles32, int64_t n_tiles128,
                                                        uint8_t* __restrict__ out) {
  // one thread per (tile, plane, lane) for the codes; the first 256 threads-worth of each tile also place a scale byte
  const int64_t total = k_tiles32 * n_tiles128 * 128;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int lane = (int)(i & 63), plane = (int)((i >> 6) & 1);
    const int64_t tile = i >> 7, nt = tile % n_tiles128, kt = tile / n_tiles128;
    const int c = lane & 31, g = lane >> 5;
    const int64_t k = kt * 32 + c;
    uint8_t* t = out + tile * kPackTileBytes;
    u32x4 v = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      uint32_t w = 0;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int64_t n = nt * 128 + plane * 64 + 16 * j + 8 * g + e;
        uint32_t nib = 0;
        if (n < N && k < K) nib = (codes[n * (K / 2) + k / 2] >> (4 * (int)(k & 1))) & 0xFu;
        w |= nib << (4 * e);
      }
      v[j] = w;
    }
    *reinterpret_cast<u32x4*>(t + plane * 1024 + lane * 16) = v;
    // scale bytes: [plane][input block kb][64 rows]; this thread places two of the tile's 256
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int idx = plane * 128 + h * 64 + lane;          // = plane * 128 + kb * 64 + row, kb = h, row = lane
      const int64_t n = nt * 128 + plane * 64 + lane, kb = kt * 2 + h;
      uint8_t sc = 0;
      if (n < N && kb * 16 < K) sc = scales[n * (K / 16) + kb];
      t[2048 + idx] = sc;
    }
  }
}

// One launch before the products of a call: AT[c, j] = A[j, c] and BT[j, n] = B[n, j] (the adapters change with every
// optimiser step, so both are transposed per call), and the arrival counters of the K-split down-projections set
// to zero.  Blocks [0, blocks_a) transpose A, the next blocks_b transpose B, the last block clears the counters.
__global__ __launch_bounds__(256) void backward_prepare_kernel(const uint16_t* __restrict__ A, int64_t r, int64_t K, uint16_t* __restrict__ AT,
                                                               const uint16_t* __restrict__ B, int64_t N, uint16_t* __restrict__ BT,
                                                               int blocks_a, int blocks_b, uint32_t* __restrict__ counters, int n_counters) {
  int b = blockIdx.x;
  if (b >= blocks_a + blocks_b) {
    for (int i = threadIdx.x; i < n_counters; i += 256) counters[i] = 0u;
    return;
  }
  const uint16_t* in = A;
  uint16_t* out = AT;
  int64_t R = r, C = K;           // in is [R, C], out [C, R]
  int blocks = blocks_a;
  if (b >= blocks_a) { b -= blocks_a; in = B; out = BT; R = N; C = r; blocks = blocks_b; }
  const int64_t total = R * C;
  for (int64_t i = (int64_t)b * 256 + threadIdx.x; i < total; i += (int64_t)blocks * 256) {
    const int64_t c = i / R, rr = i - c * R;       // consecutive threads write consecutive elements of out
    out[i] = in[rr * C + c];
  }
}

// ---- dA, dB: partial[chunk][c][j] = sum over the chunk's tokens of P[m, j] * Q[m, c] ------------------------
// P [M, r] arrives as the three bf16 terms the LoRA down-projection kernel writes ([M, ts_ld]: hi | mid | lo,
// their sum exact to 2^-24); Q is x or dY (bf16, row-major).  Both operands are contracted over their ROWS, so a
// lane's eight consecutive contraction values lie in eight different rows: tiles of 32 tokens go through LDS
// row by row (coalesced) and are read back column-wise, two bf16 values per dword.  A workgroup owns 128 columns
// of Q (32 per wave), all ranks and one token chunk; three MFMAs per rank tile and 16 tokens (one per term).
constexpr int kGradRanks = 64;       // most ranks
constexpr int kGradChunksMax = 8;    // token chunks (workgroups along M) whose partial sums are added in order
constexpr int kGradTokens = 32;      // tokens per LDS tile
constexpr int kGradQStride = 128 + 8, kGradPStride = 3 * kGradRanks + 8;   // u16 per LDS row: 16 bytes of padding shift the banks from row to row
// RANK_MAJOR: the result is wanted as [r, C] (dA): the MFMA operands change places, so that a lane owns a column
// and the partial sums leave as partial[chunk][j][c], rows of C contiguous like the final result.
template <bool RANK_MAJOR>
__global__ __launch_bounds__(256) void lora_grad_partial_kernel(const uint16_t* __restrict__ ts, int64_t ts_ld, int r,
                                                                const uint16_t* __restrict__ Q, int64_t ldq, int64_t M, int64_t C,
                                                                int64_t tokens_per_chunk, float* __restrict__ partial) {
  __shared__ __attribute__((aligned(16))) uint16_t sQ[kGradTokens * kGradQStride];
  __shared__ __attribute__((aligned(16))) uint16_t sP[kGradTokens * kGradPStride];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n32 = lane & 31, kg = lane >> 5;
  const int64_t c0 = (int64_t)blockIdx.x * 128;
  const int64_t m_lo = (int64_t)blockIdx.y * tokens_per_chunk;
  const int64_t m_hi = m_lo + tokens_per_chunk < M ? m_lo + tokens_per_chunk : M;
  const int p_chunks = 3 * r / 8;      // 16-byte chunks of a row of the three terms
  f32x16 acc[2];
#pragma unroll
  for (int jt = 0; jt < 2; ++jt)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[jt][i] = 0.f;
  // the tile after the current one is requested before the current one is multiplied (registers), so that a
  // workgroup pays the memory latency once, not once per tile
  u32x4 qreg[2], preg[3];
  auto request = [&](int64_t m0) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {      // Q tile: 32 rows x 16 chunks
      const int idx = tid + 256 * i, row = idx >> 4, ch = idx & 15;
      qreg[i] = u32x4{0u, 0u, 0u, 0u};
      if (m0 + row < m_hi && c0 + ch * 8 < C) qreg[i] = *reinterpret_cast<const u32x4*>(Q + (m0 + row) * ldq + c0 + ch * 8);
    }
#pragma unroll
    for (int i = 0; i < 3; ++i) {      // P tile: 32 rows x up to 24 chunks
      const int idx = tid + 256 * i, row = idx / 24, ch = idx - row * 24;
      preg[i] = u32x4{0u, 0u, 0u, 0u};
      if (m0 + row < m_hi && ch < p_chunks) preg[i] = *reinterpret_cast<const u32x4*>(ts + (m0 + row) * ts_ld + ch * 8);
    }
  };
  request(m_lo);
  for (int64_t m0 = m_lo; m0 < m_hi; m0 += kGradTokens) {
    __syncthreads();                   // the previous tile has been read
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int idx = tid + 256 * i, row = idx >> 4, ch = idx & 15;
      *reinterpret_cast<u32x4*>(sQ + row * kGradQStride + ch * 8) = qreg[i];
    }
#pragma unroll
    for (int i = 0; i < 3; ++i) {
      const int idx = tid + 256 * i, row = idx / 24, ch = idx - row * 24;
      *reinterpret_cast<u32x4*>(sP + row * kGradPStride + ch * 8) = preg[i];
    }
    __syncthreads();
    request(m0 + kGradTokens);         // past the chunk's end every guard fails: zeros, no access
#pragma unroll
    for (int ks = 0; ks < kGradTokens / 16; ++ks) {
      const int rb = ks * 16 + 8 * kg;   // this lane's eight tokens of the step
      u32x4 af;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const uint32_t lo = sQ[(rb + 2 * e) * kGradQStride + wave * 32 + n32], hi = sQ[(rb + 2 * e + 1) * kGradQStride + wave * 32 + n32];
        af[e] = lo | (hi << 16);
      }
#pragma unroll
      for (int jt = 0; jt < 2; ++jt) {
        const int j = jt * 32 + n32;
        if (jt * 32 < r) {             // uniform
#pragma unroll
          for (int t = 0; t < 3; ++t) {
            u32x4 bf = {0u, 0u, 0u, 0u};
            if (j < r) {
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                const uint32_t lo = sP[(rb + 2 * e) * kGradPStride + t * r + j], hi = sP[(rb + 2 * e + 1) * kGradPStride + t * r + j];
                bf[e] = lo | (hi << 16);
              }
            }
            if constexpr (RANK_MAJOR)
              acc[jt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, bf), __builtin_bit_cast(bf16x8, af), acc[jt], 0, 0, 0);
            else
              acc[jt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, af), __builtin_bit_cast(bf16x8, bf), acc[jt], 0, 0, 0);
          }
        }
      }
    }
  }
  if constexpr (RANK_MAJOR) {
    // acc[jt][q] = sum for rank 32 jt + 8 (q / 4) + 4 kg + q % 4 and column c0 + 32 wave + n32
    const int64_t c = c0 + wave * 32 + n32;
#pragma unroll
    for (int jt = 0; jt < 2; ++jt)
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int j = jt * 32 + 8 * (q >> 2) + 4 * kg + (q & 3);
        if (c < C && j < r) partial[((int64_t)blockIdx.y * kGradRanks + j) * C + c] = acc[jt][q];
      }
  } else {
    // acc[jt][q] = sum for column c0 + 32 wave + 8 (q / 4) + 4 kg + q % 4 and rank 32 jt + n32
#pragma unroll
    for (int jt = 0; jt < 2; ++jt) {
      const int j = jt * 32 + n32;
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int64_t c = c0 + wave * 32 + 8 * (q >> 2) + 4 * kg + (q & 3);
        if (c < C && j < r) partial[((int64_t)blockIdx.y * C + c) * kGradRanks + j] = acc[jt][q];
      }
    }
  }
}

// out = mult * sum over chunks (in chunk order): [C, r] from partial[chunk][c][j], or (rank_major) [r, C] from
// partial[chunk][j][c]; consecutive threads read and write consecutive elements either way
__global__ __launch_bounds__(256) void lora_grad_reduce_kernel(const float* __restrict__ partial, int n_chunks, int64_t C, int r,
                                                               const float* __restrict__ mult, int rank_major, float* __restrict__ out) {
  const int64_t total = C * r;
  const float s = *mult;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    int64_t first, stride;
    if (rank_major) { first = i; stride = (int64_t)kGradRanks * C; }                       // i = j C + c
    else { const int64_t c = i / r; first = c * kGradRanks + (i - c * r); stride = C * kGradRanks; }
    float sum = 0.f;
    for (int z = 0; z < n_chunks; ++z) sum += partial[first + z * stride];
    out[i] = sum * s;
  }
}

static size_t al256(size_t v) { return (v + 255) & ~(size_t)255; }
// Workspace of a backward call over n members that read the same x: the arrival counters of the K-split
// down-projections, then per member A^T, B^T and the two three-term products, then one area that first holds the
// down-projections' K-part sums and later the gradient products' partial sums.
struct BackwardMemberLayout { size_t at_off, bt_off, tsu_off, tst_off; int64_t ts_ld; int ext_stages; };
struct BackwardLayout { size_t ctr_off, part_off, total; int n_chunks; int64_t tokens_per_chunk; BackwardMemberLayout mem[kMaxGroup]; };
static BackwardLayout backward_layout(int64_t M, int64_t K, const int64_t* Ns, const int64_t* rs, int n) {
  BackwardLayout L{};
  const size_t m = (size_t)(M > 0 ? M : 1), k = (size_t)(K > 0 ? K : 1);
  int64_t chunks = ceil_div((int64_t)m, 64);
  chunks = chunks > kGradChunksMax ? kGradChunksMax : chunks;
  L.n_chunks = (int)chunks;
  L.tokens_per_chunk = ceil_div((int64_t)m, chunks);
  L.ctr_off = 0;                                   // zeroed by every call
  size_t off = al256(kDownMaxSlots * sizeof(uint32_t));
  size_t widest = 0;
  bool any = false;
  for (int i = 0; i < n; ++i) {
    const size_t nn = (size_t)(Ns[i] > 0 ? Ns[i] : 1), rr = (size_t)(rs[i] > 0 ? rs[i] : 0);
    BackwardMemberLayout& b = L.mem[i];
    b.ext_stages = (int)ceil_div(3 * (int64_t)rr, 64);
    b.ts_ld = (int64_t)b.ext_stages * 64;
    b.at_off = off;  off += al256(k * rr * 2);
    b.bt_off = off;  off += al256(nn * rr * 2);
    b.tsu_off = off; off += al256(m * (size_t)b.ts_ld * 2);
    b.tst_off = off; off += al256(m * (size_t)b.ts_ld * 2);
    if (rr) { any = true; widest = widest > nn ? widest : nn; }
  }
  L.part_off = off;
  size_t part = 0;
  if (any) {
    widest = widest > k ? widest : k;
    part = al256((size_t)chunks * widest * kGradRanks * sizeof(float));
    if (part < kDownExchangeBytes) part = kDownExchangeBytes;
  }
  L.total = L.part_off + part;
  return L;
}
static int grid_for(int64_t items) {
  int64_t b = ceil_div(items, 256);
  return (int)(b < 1 ? 1 : (b > 8192 ? 8192 : b));
}

struct BackwardMember {
  const uint16_t* dy; int64_t lddy; int64_t N; const uint8_t* packed_t; const float* tensor_scale;
  const uint16_t* A; const uint16_t* B; int64_t r; float lora_scale; float* dA; float* dB;
};

static int backward_validate(const void* x, int64_t M, int64_t K, int64_t ldx, const BackwardMember* mem, int n, const void* dx, int64_t lddx) {
  if (n < 1 || n > kMaxGroup) return QERL_ERR_SHAPE;
  if (M < 0 || K < 0 || K % kBlock != 0 || ldx < K || lddx < K) return QERL_ERR_SHAPE;
  bool any = false;
  for (int i = 0; i < n; ++i) {
    const BackwardMember& b = mem[i];
    if (b.N < 0 || b.r < 0 || b.N % 8 != 0 || b.lddy < b.N || b.r > kGradRanks || b.r % 8 != 0) return QERL_ERR_SHAPE;
    any = any || b.r > 0;
  }
  if (M == 0) return 1;   // nothing to do
  if (K == 0) return QERL_ERR_SHAPE;
  for (int i = 0; i < n; ++i) if (mem[i].N == 0) return QERL_ERR_SHAPE;
  if (!dx) return QERL_ERR_NULL;
  if (any && !x) return QERL_ERR_NULL;
  for (int i = 0; i < n; ++i) {
    const BackwardMember& b = mem[i];
    if (!b.dy || !b.packed_t || !b.tensor_scale) return QERL_ERR_NULL;
    if (b.r > 0 && (!b.A || !b.B || !b.dA || !b.dB)) return QERL_ERR_NULL;
  }
  if (!aligned(dx, 2)) return QERL_ERR_ALIGN;
  if (any && (!aligned(x, 16) || ldx % 8 != 0)) return QERL_ERR_ALIGN;
  for (int i = 0; i < n; ++i) {
    const BackwardMember& b = mem[i];
    if (!aligned(b.dy, 16) || b.lddy % 8 != 0 || !aligned(b.packed_t, 16)) return QERL_ERR_ALIGN;
    if (b.r > 0 && (!aligned(b.A, 16) || !aligned(b.B, 16) || !aligned(b.dA, 4) || !aligned(b.dB, 4))) return QERL_ERR_ALIGN;
  }
  return QERL_OK;
}

// The members' launches: per member one that transposes its adapter, one down-projection of its own dY, and four
// for its gradient products; shared by the group: the down-projections of x (one launch over all adapters) and dX,
// ONE GEMM whose contraction runs over the members' rows one after the other, so that dX is summed in fp32 and
// rounded once.
static int backward_run(const uint16_t* x, int64_t M, int64_t K, int64_t ldx, const BackwardMember* mem, int n, uint16_t* dx, int64_t lddx,
                        void* workspace, size_t workspace_bytes, hipStream_t st) {
  int64_t Ns[kMaxGroup], rs[kMaxGroup];
  for (int i = 0; i < n; ++i) { Ns[i] = mem[i].N; rs[i] = mem[i].r; }
  const BackwardLayout L = backward_layout(M, K, Ns, rs, n);
  if (!workspace || !aligned(workspace, 256) || workspace_bytes < L.total) return QERL_ERR_WORKSPACE;
  uint8_t* ws = (uint8_t*)workspace;
  uint32_t* counters = (uint32_t*)(ws + L.ctr_off);
  float* part = (float*)(ws + L.part_off);
  int rc = QERL_OK;
  GemmArgs down{};   // t_i = x A_i^T of all adapters, one launch
  down.x = x; down.ldx = ldx; down.M = M; down.K = K; down.k_tiles = ceil_div(K, kPackTileK);
  down.tpart = (uint32_t*)part; down.counters = counters;
  int tiles = 0;
  for (int i = 0; i < n; ++i) {
    const BackwardMember& b = mem[i];
    if (b.r == 0) continue;
    const BackwardMemberLayout& l = L.mem[i];
    uint16_t* AT = (uint16_t*)(ws + l.at_off);
    uint16_t* BT = (uint16_t*)(ws + l.bt_off);
    const int blocks_a = grid_for(b.r * K), blocks_b = grid_for(b.N * b.r);
    backward_prepare_kernel<<<dim3((unsigned)(blocks_a + blocks_b + 1)), dim3(256), 0, st>>>(
        b.A, b.r, K, AT, b.B, b.N, BT, blocks_a, blocks_b, counters, kDownMaxSlots);
    if ((rc = launch_status()) != QERL_OK) return rc;
    // U_i = dY_i B_i as three bf16 terms of (lora_scale / S32) times the product
    GemmArgs d{};
    d.x = b.dy; d.ldx = b.lddy; d.M = M; d.K = b.N; d.k_tiles = ceil_div(b.N, kPackTileK);
    d.N = b.r; d.wbf16 = BT; d.n_tiles = (int)ceil_div(b.r, 32); d.ts = (const uint16_t*)(ws + l.tsu_off); d.ts_ld = l.ts_ld; d.ext_stages = l.ext_stages;
    d.r = (int)b.r; d.lora_scale = b.lora_scale; d.tensor_scale = b.tensor_scale;
    d.tpart = (uint32_t*)part; d.counters = counters;   // K split over workgroups while token blocks alone do not fill the chip
    if ((rc = launch_lora_down_gemm(d, st)) != QERL_OK) return rc;
    const int gi = down.g_n++;
    down.g_tile0[gi] = tiles; down.g_A[gi] = b.A; down.g_ts[gi] = (const uint16_t*)(ws + l.tst_off); down.g_ts_ld[gi] = l.ts_ld;
    down.g_r[gi] = (int)b.r; down.g_lora_scale[gi] = b.lora_scale; down.g_tensor_scale[gi] = b.tensor_scale;
    tiles += (int)ceil_div(b.r, 32);
  }
  if (down.g_n > 0) {
    down.g_tile0[down.g_n] = tiles;
    if ((rc = launch_lora_down_gemm(down, st)) != QERL_OK) return rc;
  }
  {
    GemmArgs g{};
    g.M = M; g.N = K; g.n_tiles = (int)ceil_div(K, 32); g.y = dx; g.ldy = lddx; g.transposed = 1;
    g.seg_n = n;
    int64_t rows = 0;
    for (int i = 0; i < n; ++i) {
      const BackwardMember& b = mem[i];
      const BackwardMemberLayout& l = L.mem[i];
      GemmSeg& sgm = g.seg[i];
      sgm.x = b.dy; sgm.ldx = b.lddy; sgm.K = b.N; sgm.packed = b.packed_t; sgm.k_tiles = ceil_div(b.N, kPackTileK);
      sgm.tensor_scale = b.tensor_scale;
      if (b.r > 0) {
        sgm.ts = (const uint16_t*)(ws + l.tsu_off); sgm.ts_ld = l.ts_ld; sgm.ext_stages = l.ext_stages;
        sgm.B = (const uint16_t*)(ws + l.at_off); sgm.r = (int)b.r;
      }
      rows += b.N;
    }
    // the launcher's own fields describe the first segment (it validates them; the kernel reads the segments)
    g.x = g.seg[0].x; g.ldx = g.seg[0].ldx; g.K = rows; g.k_tiles = g.seg[0].k_tiles; g.packed = g.seg[0].packed; g.tensor_scale = g.seg[0].tensor_scale;
    if ((rc = launch_gemm(g, st)) != QERL_OK) return rc;
  }
  for (int i = 0; i < n; ++i) {
    const BackwardMember& b = mem[i];
    if (b.r == 0) continue;
    const BackwardMemberLayout& l = L.mem[i];
    // the three-term values carry lora_scale / S32; the gradients want lora_scale: one multiplication by S32
    const dim3 blk(256);
    lora_grad_partial_kernel<true><<<dim3((unsigned)ceil_div(K, 128), (unsigned)L.n_chunks), blk, 0, st>>>(
        (const uint16_t*)(ws + l.tsu_off), l.ts_ld, (int)b.r, x, ldx, M, K, L.tokens_per_chunk, part);
    lora_grad_reduce_kernel<<<dim3((unsigned)grid_for(K * b.r)), blk, 0, st>>>(part, L.n_chunks, K, (int)b.r, b.tensor_scale, 1, b.dA);
    lora_grad_partial_kernel<false><<<dim3((unsigned)ceil_div(b.N, 128), (unsigned)L.n_chunks), blk, 0, st>>>(
        (const uint16_t*)(ws + l.tst_off), l.ts_ld, (int)b.r, b.dy, b.lddy, M, b.N, L.tokens_per_chunk, part);
    lora_grad_reduce_kernel<<<dim3((unsigned)grid_for(b.N * b.r)), blk, 0, st>>>(part, L.n_chunks, b.N, (int)b.r, b.tensor_scale, 0, b.dB);
    if ((rc = launch_status()) != QERL_OK) return rc;
  }
  return rc;
}

}  // namespace qerl

using namespace qerl;

extern "C" size_t nvfp4_prepack_t_bytes(int64_t N, int64_t K) {
  if (N <= 0 || K <= 0) return 0;
  return (size_t)ceil_div(K, 32) * (size_t)ceil_div(N, 128) * kPackTileBytes;
}

extern "C" int nvfp4_prepack_t(const uint8_t* codes, const uint8_t* scales, int64_t N, int64_t K, void* packed_t, void* stream) {
  if (N < 0 || K < 0 || K % kBlock != 0) return QERL_ERR_SHAPE;
  if (N == 0 || K == 0) return QERL_OK;
  if (!codes || !scales || !packed_t) return QERL_ERR_NULL;
  if (!aligned(packed_t, 16)) return QERL_ERR_ALIGN;
  const int64_t kt = ceil_div(K, 32), nt = ceil_div(N, 128);
  prepack_t_kernel<<<dim3((unsigned)grid_for(kt * nt * 128)), dim3(256), 0, (hipStream_t)stream>>>(codes, scales, N, K, kt, nt, (uint8_t*)packed_t);
  return launch_status();
}

extern "C" size_t nvfp4_lora_linear_backward_workspace_bytes(int64_t M, int64_t N, int64_t K, int64_t r) {
  const size_t t = backward_layout(M, K, &N, &r, 1).total;
  return t ? t : 256;
}

extern "C" int nvfp4_lora_linear_backward(const void* x, const void* dy, int64_t M, int64_t K, int64_t N, int64_t ldx, int64_t lddy,
                                          const void* packed_t, const float* tensor_scale, const void* A, const void* B,
                                          int64_t r, float lora_scale, void* dx, int64_t lddx, float* dA, float* dB,
                                          void* workspace, size_t workspace_bytes, void* stream) {
  const BackwardMember b{(const uint16_t*)dy, lddy, N, (const uint8_t*)packed_t, tensor_scale, (const uint16_t*)A, (const uint16_t*)B, r, lora_scale, dA, dB};
  const int vr = backward_validate(x, M, K, ldx, &b, 1, dx, lddx);
  if (vr != QERL_OK) return vr > 0 ? QERL_OK : vr;
  return backward_run((const uint16_t*)x, M, K, ldx, &b, 1, (uint16_t*)dx, lddx, workspace, workspace_bytes, (hipStream_t)stream);
}

extern "C" size_t nvfp4_lora_linear_backward_group_workspace_bytes(int64_t M, int64_t K, const qerl_backward_desc* members, int n_members) {
  if (!members || n_members < 1 || n_members > kMaxGroup) return 0;
  int64_t Ns[kMaxGroup], rs[kMaxGroup];
  for (int i = 0; i < n_members; ++i) { Ns[i] = members[i].N; rs[i] = members[i].r; }
  const size_t t = backward_layout(M, K, Ns, rs, n_members).total;
  return t ? t : 256;
}

extern "C" int nvfp4_lora_linear_backward_group(const void* x, int64_t M, int64_t K, int64_t ldx, const qerl_backward_desc* members,
                                                int n_members, void* dx, int64_t lddx, void* workspace, size_t workspace_bytes, void* stream) {
  if (!members) return QERL_ERR_NULL;
  if (n_members < 1 || n_members > kMaxGroup) return QERL_ERR_SHAPE;
  BackwardMember b[kMaxGroup];
  for (int i = 0; i < n_members; ++i) {
    const qerl_backward_desc& d = members[i];
    b[i] = BackwardMember{(const uint16_t*)d.dy_bf16, d.lddy, d.N, (const uint8_t*)d.packed_t, d.tensor_scale, (const uint16_t*)d.A_bf16,
                          (const uint16_t*)d.B_bf16, d.r, d.lora_scale, d.dA_f32, d.dB_f32};
  }
  const int vr = backward_validate(x, M, K, ldx, b, n_members, dx, lddx);
  if (vr != QERL_OK) return vr > 0 ? QERL_OK : vr;
  return backward_run((const uint16_t*)x, M, K, ldx, b, n_members, (uint16_t*)dx, lddx, workspace, workspace_bytes, (hipStream_t)stream);
}
