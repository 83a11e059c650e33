// C-ABI entry points that are not kernels themselves: status strings, the
// sigma schedule, workspace layout and the dispatch of nvfp4_lora_linear.
#include <math.h>
#include "linear.hpp"

namespace qerl {

static thread_local int g_last_hip_error = 0;
void set_last_hip_error(int e) { g_last_hip_error = e; }

// Workspace layout of one linear call (offsets in bytes, all 256-aligned):
//   [0, ctrl_bytes)     arrival counters (uint32): main tiles, then LoRA-down tiles
//   [t_off, ...)        t = x A^T, fp32 [M, r]
//   [partial_off, ...)  split-K partial tiles, fp32
struct WorkspaceLayout { size_t ctrl_bytes, n_main_ctr, n_down_ctr, t_off, partial_off, total; };

constexpr size_t kDecodeTpartWords = 16 * 16 * 256;   // producer partial sums of the fused LoRA down-projection: <= 16 producers x 16 tokens x stacked rank <= 256
constexpr size_t kMaxCounterTiles = 16384;   // rows / 16 the control region can serve

static size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

// The control region has a FIXED size and position (linear.hpp) so that calls of different shapes can share one
// workspace: no call's data region may overlap another call's control words (they must stay zero).
constexpr size_t kCtrlBytes = kCtrlRegionBytes;

// 17..128 tokens: room for the K-splits' partial outputs (up to 8 splits, capped); the K-parts' sums of the
// LoRA down-projection follow it.
static size_t mid_partial_bytes(int64_t M, int64_t N) {
  const size_t b = (size_t)8 * (size_t)(M > 0 ? M : 1) * (size_t)(N > 0 ? N : 1) * sizeof(float);
  return align256(b < kMidPartialCap ? b : kMidPartialCap);
}

static WorkspaceLayout workspace_layout(int64_t M, int64_t N, int64_t K, int64_t r) {
  WorkspaceLayout L;
  L.n_main_ctr = kCtrlMainWords;
  const size_t n_down_ctr = (size_t)ceil_div(r > 0 ? r : 1, 16);
  L.n_down_ctr = kCtrlDownWords;
  L.ctrl_bytes = kCtrlBytes;
  L.t_off = L.ctrl_bytes;
  // t = x A^T: fp32 [M, r] for the decode kernels, or three bf16 terms [M, ceil64(3r)] for the GEMM
  const size_t rows = (size_t)(M > 0 ? M : 1), rr = (size_t)(r > 0 ? r : 1);
  const size_t t_f32 = rows * rr * sizeof(float), t_split = rows * (size_t)(ceil_div(3 * rr, 128) + kMaxGroup - 1) * 128 * 2;   // each member of a group pads its 3r columns to 128
  const size_t t_bytes = align256(t_f32 > t_split ? t_f32 : t_split);
  L.partial_off = L.t_off + t_bytes;
  // worst case over the plans the dispatchers can choose (one K-tile per wave)
  const size_t S_max = (size_t)ceil_div(ceil_div(K > 0 ? K : 1, 256), 8);
  const size_t S_down = (size_t)ceil_div(ceil_div(K > 0 ? K : 1, 256), 2) + 1;
  const size_t n_rows16 = (size_t)ceil_div(N > 0 ? N : 1, 16);
  const size_t skinny_bytes = (S_max * n_rows16 + S_down * n_down_ctr) * 64 * sizeof(f32x4);
  const size_t S_dec = (size_t)ceil_div(ceil_div(K > 0 ? K : 1, kPackTileK), 7);
  const size_t decode_bytes = S_dec * (size_t)ceil_div(N > 0 ? N : 1, kPackTileRows) * 8 * 64 * sizeof(float) +
                              S_down * n_down_ctr * 64 * sizeof(f32x4) + kDecodeTpartWords * sizeof(uint32_t);
  size_t need = skinny_bytes > decode_bytes ? skinny_bytes : decode_bytes;
  if (M > 16 && M <= 128) {
    const size_t mid = mid_partial_bytes(M, N) + kMidDownBytes;
    need = need > mid ? need : mid;
  }
  if (M > 128 && need < kDownExchangeBytes) need = kDownExchangeBytes;   // K-parts of the prefill path's LoRA down-projection
  if (M > 16) {
    // the GEMM path from g_gemm_min_tokens on: a down-projection launched by itself has the whole area for its K-part
    // sums and is through with it when the GEMM starts; one that rides inside the GEMM launch needs the first
    // kFusedDownBytes at most, and the GEMM's own K-parts start behind them
    size_t g = kFusedDownBytes + gemm_split_bytes(M, N);
    g = g > kDownExchangeBytes ? g : kDownExchangeBytes;
    need = need > g ? need : g;
  }
  L.total = L.partial_off + align256(need);
  return L;
}

// act[m, k] = bf16(bf16(SiLU(gate[m, k])) * up[m, k]), eight values per thread
__global__ __launch_bounds__(256) void silu_mul_kernel(const uint16_t* __restrict__ gate, int64_t ldg, const uint16_t* __restrict__ up,
                                                       int64_t ldu, int64_t M, int64_t K, uint16_t* __restrict__ act) {
  const int64_t chunks = K / 8, total = M * chunks;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int64_t m = i / chunks, c = i - m * chunks;
    const u32x4 g = *reinterpret_cast<const u32x4*>(gate + m * ldg + c * 8);
    const u32x4 u = *reinterpret_cast<const u32x4*>(up + m * ldu + c * 8);
    *reinterpret_cast<u32x4*>(act + m * K + c * 8) = silu_mul8(g, u);
  }
}

__global__ void zero_words_kernel(uint32_t* p, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    p[i] = 0u;
}

}  // namespace qerl

using namespace qerl;

extern "C" const char* qerl_status_string(int status) {
  switch (status) {
    case QERL_OK: return "ok";
    case QERL_ERR_NULL: return "a required pointer is NULL";
    case QERL_ERR_SHAPE: return "invalid shape or leading dimension";
    case QERL_ERR_ALIGN: return "pointer or leading dimension not aligned as required";
    case QERL_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case QERL_ERR_LAUNCH: return "HIP runtime error at launch (see qerl_last_hip_error)";
    case QERL_ERR_TIMEOUT: return "a kernel's bounded wait on another workgroup gave up: results unreliable, re-initialise the workspace";
    default: return "unknown status";
  }
}

extern "C" int qerl_last_hip_error(void) { return g_last_hip_error; }

extern "C" double aqn_sigma(int k, int num_stages, double s0, double s1) {
  if (num_stages < 1 || k < 0 || k > num_stages) return NAN;
  if (k == 0) return 0.0;
  if (num_stages == 1) return s0;
  return s0 * pow(s1 / s0, (double)(k - 1) / (double)(num_stages - 1));
}

extern "C" size_t nvfp4_lora_linear_workspace_bytes(int64_t M, int64_t N, int64_t K, int64_t r) {
  return workspace_layout(M, N, K, r).total;
}

extern "C" int qerl_workspace_init(void* workspace, size_t bytes, void* stream) {
  if (!workspace) return QERL_ERR_NULL;
  if (!aligned(workspace, 256)) return QERL_ERR_ALIGN;
  // the control region is a prefix; clearing the whole buffer keeps this independent of shapes
  const size_t words = bytes / 4;
  if (words == 0) return QERL_OK;
  size_t nb = (words + 255) / 256;
  if (nb > 4096) nb = 4096;
  zero_words_kernel<<<(int)nb, 256, 0, (hipStream_t)stream>>>((uint32_t*)workspace, words);
  return launch_status();
}

namespace qerl {

struct LinearCall {
  const uint16_t* x; int64_t M, K, ldx; const float* tensor_scale; int64_t N;
  const uint16_t* A; const uint16_t* B; int64_t r; float lora_scale; uint16_t* y; int64_t ldy;
  void* workspace; size_t workspace_bytes; hipStream_t st;
};

// Checks shared by the canonical and the packed entry point.
static int validate(const LinearCall& c, const void* w0, const void* w1) {
  if (c.M < 0 || c.N < 0 || c.K < 0 || c.r < 0 || c.K % kBlock != 0 || c.ldx < c.K || c.ldy < c.N)
    return QERL_ERR_SHAPE;
  if (c.N / 16 >= (int64_t)kMaxCounterTiles || c.r > 4096) return QERL_ERR_SHAPE;
  if (c.M == 0 || c.N == 0) return 1;   // nothing to do
  if (!c.x || !c.y || !c.tensor_scale) return QERL_ERR_NULL;
  if (c.K > 0 && (!w0 || !w1)) return QERL_ERR_NULL;
  if (c.r > 0 && (!c.A || !c.B)) return QERL_ERR_NULL;
  if (!aligned(c.x, 2) || !aligned(c.y, 2) || (c.r > 0 && (!aligned(c.A, 2) || !aligned(c.B, 2))))
    return QERL_ERR_ALIGN;
  const WorkspaceLayout L = workspace_layout(c.M, c.N, c.K, c.r);
  if (!c.workspace || !aligned(c.workspace, 256) || c.workspace_bytes < L.total) return QERL_ERR_WORKSPACE;
  return QERL_OK;
}

// t[m0 .. m0+mc) = x A^T for one pass of at most 16 tokens.
static int lora_down_pass(const LinearCall& c, const WorkspaceLayout& L, int64_t m0, int mc, f32x4* partial) {
  uint8_t* ws = (uint8_t*)c.workspace;
  float* t = (float*)(ws + L.t_off) + m0 * c.r;
  const bool tiled = (c.K % 64 == 0) && aligned(c.x, 16) && c.ldx % 8 == 0 && aligned(c.A, 16);
  if (!tiled) return launch_generic_lora_down(c.x + m0 * c.ldx, c.ldx, mc, c.K, c.A, c.r, t, c.st);
  const SkinnyPlan pd = plan_skinny(c.r, c.K, kFmtBf16);
  SkinnyArgs d{};
  d.x = c.x + m0 * c.ldx; d.ldx = c.ldx; d.M = mc; d.K = c.K;
  d.N = c.r; d.wbf16 = c.A; d.t_out = t;
  d.partial = partial; d.counters = (uint32_t*)ws + L.n_main_ctr; d.n_tiles = pd.n_tiles;
  return launch_skinny(pd, d, kFmtBf16, c.st);
}

}  // namespace qerl

extern "C" int nvfp4_lora_linear(const void* x, int64_t M, int64_t K, int64_t ldx, const uint8_t* codes,
                                 const uint8_t* scales, const float* tensor_scale, int64_t N,
                                 const void* A, const void* B, int64_t r, float lora_scale, void* y,
                                 int64_t ldy, void* workspace, size_t workspace_bytes, void* stream) {
  LinearCall c{(const uint16_t*)x, M, K, ldx, tensor_scale, N, (const uint16_t*)A, (const uint16_t*)B, r,
               lora_scale, (uint16_t*)y, ldy, workspace, workspace_bytes, (hipStream_t)stream};
  const int vr = validate(c, codes, scales);
  if (vr != QERL_OK) return vr > 0 ? QERL_OK : vr;
  if (K == 0) c.r = r = 0;   // empty sums: y = 0 through the general kernel
  const WorkspaceLayout L = workspace_layout(M, N, K, r);
  uint8_t* ws = (uint8_t*)workspace;
  float* t = (float*)(ws + L.t_off);
  f32x4* partial = (f32x4*)(ws + L.partial_off);

  // The tiled kernels use 16-byte loads; anything else goes to the general kernels.
  const bool tiled = (K % 64 == 0) && K > 0 && aligned(x, 16) && ldx % 8 == 0 && aligned(codes, 16) &&
                     aligned(scales, 4) && (r == 0 || aligned(A, 16));
  if (!tiled) {
    int rc = QERL_OK;
    if (r > 0) rc = launch_generic_lora_down(c.x, ldx, M, K, c.A, r, t, c.st);
    if (rc != QERL_OK) return rc;
    return launch_generic_linear(c.x, ldx, M, K, codes, scales, tensor_scale, N, r > 0 ? t : nullptr, c.B, r,
                                 lora_scale, c.y, ldy, c.st);
  }

  // Tiled path on the canonical layout: passes of up to 16 tokens.
  const SkinnyPlan pm = plan_skinny(N, K, kFmtNvfp4);
  for (int64_t m0 = 0; m0 < M; m0 += 16) {
    const int mc = (int)((M - m0 < 16) ? M - m0 : 16);
    if (r > 0) {
      const int rc = lora_down_pass(c, L, m0, mc, partial + (size_t)pm.S * pm.n_tiles * 64);
      if (rc != QERL_OK) return rc;
    }
    SkinnyArgs a{};
    a.x = c.x + m0 * ldx; a.ldx = ldx; a.M = mc; a.K = K;
    a.N = N; a.codes = codes; a.scales = scales; a.tensor_scale = tensor_scale;
    a.t_in = t + m0 * r; a.B = c.B; a.r = (int)r; a.lora_scale = lora_scale;
    a.y = c.y + m0 * ldy; a.ldy = ldy;
    a.y_vec = aligned(y, 8) && ldy % 4 == 0;
    a.b_vec = r % 8 == 0 && aligned(B, 16);
    a.partial = partial; a.counters = (uint32_t*)ws; a.n_tiles = pm.n_tiles;
    const int rc = launch_skinny(pm, a, kFmtNvfp4, c.st);
    if (rc != QERL_OK) return rc;
  }
  return QERL_OK;
}

namespace qerl {
static bool g_use_stream = true;
static int g_gemm_min_tokens = 96;   // from here on the prefill GEMM (K split over workgroups where the tiles alone would not fill the chip) beats the 17..128-token kernel
static int64_t g_mid_gemm_min_rows = 16384;   // 65..128 tokens: groups with at least this many output rows go to the prefill GEMM
static int64_t g_mid_producer_bytes = 24 << 20;   // 17..128 tokens: LoRA down-projections run inside the main launch when it streams at least this many packed bytes (long enough to hide them)

// One streaming launch for a group of packed linears sharing x (M <= 16; every r in {0} or 8..64 step 8).
static int stream_group(const uint16_t* x, int64_t M, int64_t K, int64_t ldx, const qerl_linear_desc* d, int n,
                        uint8_t* ws, const WorkspaceLayout& L, hipStream_t st, const uint16_t* x2 = nullptr, int64_t ldx2 = 0) {
  StreamArgs a{};
  a.x = x; a.ldx = ldx; a.M = (int)M; a.K = K; a.k_tiles = (int)ceil_div(K, kPackTileK);
  a.x2 = x2; a.ldx2 = ldx2;
  a.n_members = n;
  int tiles = 0, rt = 0, any = 0;
  for (int i = 0; i < n; ++i) {
    StreamMember& m = a.mem[i];
    m.packed = (const uint8_t*)d[i].packed; m.tensor_scale = d[i].tensor_scale;
    m.A = (const uint16_t*)d[i].A_bf16; m.B = (const uint16_t*)d[i].B_bf16; m.y = (uint16_t*)d[i].y_bf16;
    m.ldy = d[i].ldy; m.N = d[i].N; m.n_tiles = (int)ceil_div(d[i].N, kPackTileRows); m.tile_begin = tiles;
    m.r = (int)d[i].r; m.lora_scale = d[i].lora_scale;
    m.y_vec = aligned(d[i].y_bf16, 16) && d[i].ldy % 8 == 0;
    m.t_ext = m.r > 0 ? d[i].t_f32 : nullptr;
    m.bias = (const uint16_t*)d[i].bias_bf16;
    m.t_off = 0x7fffffff;                 // not part of the producers' stack ...
    if (m.r > 0 && !m.t_ext) { m.t_off = rt; rt += m.r; }   // ... unless the launch has to compute its t
    any |= m.r > 0;
    a.any_bias |= m.bias != nullptr;
    tiles += m.n_tiles;
  }
  for (int i = n; i < kMaxGroup; ++i) {   // unused entries: never selected, but valid to read
    a.mem[i] = a.mem[0];
    a.mem[i].tile_begin = 0x7fffffff; a.mem[i].n_tiles = 0; a.mem[i].r = 0; a.mem[i].t_off = 0x7fffffff; a.mem[i].t_ext = nullptr;
  }
  a.tb1 = a.mem[1].tile_begin; a.tb2 = a.mem[2].tile_begin; a.tb3 = a.mem[3].tile_begin;
  a.mp0 = a.mem[0].packed; a.mp1 = a.mem[1].packed; a.mp2 = a.mem[2].packed; a.mp3 = a.mem[3].packed;
  a.total_tiles = tiles; a.r_total = rt; a.any_lora = any;
  if (rt > 0) {
    int64_t np = ceil_div(2 * (int64_t)a.k_tiles, 8);   // one half K-tile per producer wave and tile pair
    a.n_producers = (int)(np < 1 ? 1 : (np > 16 ? 16 : np));
  }
  size_t lds = 0;
  int MR = 4;
  const int prc = plan_stream(a, &lds, &MR);
  if (prc != QERL_OK) return prc;
  uint32_t* partial = (uint32_t*)(ws + L.partial_off);
  const size_t part_words = ((size_t)a.Sk * tiles * MR * 64 + 3) & ~(size_t)3;
  a.partial = partial; a.counters = (uint32_t*)ws;
  a.t = (float*)(ws + L.t_off);
  a.lora_ctl = (uint32_t*)ws + L.n_main_ctr + L.n_down_ctr;
  a.tpart = partial + part_words;
  return launch_stream(a, lds, MR, st);
}

// A few dozen tokens (17..128), one linear or a group reading the same x: the LoRA down-projections of all
// members write lora_scale / S32 * x A^T as three bf16 terms into the workspace (one launch), then the
// weight-streaming kernel computes every member with those 3r columns appended to K (one launch, plus the
// reduction of the K-splits if there are any).
static int mid_group(const uint16_t* x, int64_t M, int64_t K, int64_t ldx, const qerl_linear_desc* d, int n,
                     uint8_t* ws, const WorkspaceLayout& L, hipStream_t st) {
  const bool few = M <= 128;   // K-splits and their workspace areas exist for these only
  MidArgs g{};
  g.x = x; g.ldx = ldx; g.M = M; g.K = K; g.k_tiles = (int)ceil_div(K, kPackTileK); g.n_members = n;
  GemmArgs dn{};
  dn.x = x; dn.ldx = ldx; dn.M = M; dn.K = K; dn.k_tiles = g.k_tiles;
  int64_t n_sum = 0;
  uint16_t* ts = (uint16_t*)(ws + L.t_off);
  int tiles = 0;
  for (int i = 0; i < n; ++i) {
    MidMember& m = g.mem[i];
    m.packed = (const uint8_t*)d[i].packed; m.tensor_scale = d[i].tensor_scale; m.N = d[i].N;
    m.n_tiles = (int)ceil_div(d[i].N, kPackTileRows);
    m.r = (int)d[i].r; m.B = (const uint16_t*)d[i].B_bf16; m.y = (uint16_t*)d[i].y_bf16; m.ldy = d[i].ldy;
    m.bias = (const uint16_t*)d[i].bias_bf16;
    m.ext_stages = (int)ceil_div(3 * d[i].r, 128); m.ts_ld = (int64_t)m.ext_stages * 128; m.ts = ts;
    ts += M * m.ts_ld;
    n_sum += d[i].N;
    if (d[i].r > 0) {
      const int gi = dn.g_n++;
      dn.g_tile0[gi] = tiles; dn.g_A[gi] = (const uint16_t*)d[i].A_bf16; dn.g_ts[gi] = m.ts; dn.g_ts_ld[gi] = m.ts_ld;
      dn.g_r[gi] = (int)d[i].r; dn.g_lora_scale[gi] = d[i].lora_scale; dn.g_tensor_scale[gi] = d[i].tensor_scale;
      tiles += (int)ceil_div(d[i].r, 32);
    }
  }
  uint32_t* partial = (uint32_t*)(ws + L.partial_off);
  g.partial = (float*)partial;
  const int prc = plan_mid(g, few ? mid_partial_bytes(M, n_sum) : 0);
  if (prc != QERL_OK) return prc;
  if (dn.g_n > 0) {
    dn.g_tile0[dn.g_n] = tiles;
    dn.tpart = few ? partial + mid_partial_bytes(M, n_sum) / sizeof(uint32_t) : nullptr;
    dn.counters = (uint32_t*)ws + L.n_main_ctr;
    int64_t packed_bytes = 0;
    for (int i = 0; i < n; ++i) packed_bytes += (int64_t)g.mem[i].n_tiles * g.k_tiles * kPackTileBytes;
    // measured on 7B shapes: above 64 tokens it always pays (7.5 against 8.2 ms per step at 128); below, where the
    // main launch runs long enough to hide producers of two or four waves (gate + up, down: 1-2 % of the step), for
    // a single adapter (o: 24.9 -> 24.6 us at 32 tokens, 29.9 -> 28.8 at 64; 32B 37.3 -> 32.8) and for groups from 33
    // tokens on (q + k + v 34.8 -> 31.7 us at 64 tokens, but 30.1 -> 36.4 at 32)
    if (few && (M > 32 || dn.g_n == 1 || packed_bytes >= g_mid_producer_bytes)) {
      // the down-projections run as the first workgroups of the main launch: token blocks x rank tiles x K-parts
      // (parts as the stand-alone launch would choose them: a few dozen workgroups, at least 512 columns each)
      const int64_t base_wgs = ceil_div(M, 32) * tiles;
      int64_t P = base_wgs < 32 ? 64 / base_wgs : 1;
      const int64_t p_max = ceil_div(K, 512);
      P = P < p_max ? P : p_max;
      P = P > 8 ? 8 : (P < 1 ? 1 : P);
      g.p_tbs = (int)ceil_div(M, 32); g.p_tiles = tiles; g.p_parts = (int)P;
      g.n_prod = (int)(ceil_div(base_wgs * P, 8) * 8);
      g.ready = (uint32_t*)ws + L.n_main_ctr + L.n_down_ctr;      // the hand-over words (zero between calls)
      g.done = g.ready + 2;
      g.n_consumers = g.n_blocks * g.m_chunks * g.S;
      dn.ready = g.ready;
      g.dn = dn;
    } else {
      const int rc = launch_lora_down_gemm(dn, st);
      if (rc != QERL_OK) return rc;
    }
  }
  return launch_mid(g, st);
}
// The GEMM launch and the LoRA down-projections it depends on (dn: the group form, tiles rank tiles; g_n == 0: none).
// launch_gemm either takes the down-projections into its own launch (few tokens) or runs them first; the scratch
// serves the down-projection's K-parts from its front and the GEMM's own K-parts from kFusedDownBytes on (inside
// one launch both are alive at once, and the down-projection stays below that mark).
static int gemm_with_down(GemmArgs& g, GemmArgs& dn, int tiles, int64_t n_sum, uint8_t* ws, const WorkspaceLayout& L, hipStream_t st) {
  if (dn.g_n > 0) {
    dn.g_tile0[dn.g_n] = tiles;
    g.g_n = dn.g_n;
    for (int i = 0; i <= dn.g_n; ++i) g.g_tile0[i] = dn.g_tile0[i];
    for (int i = 0; i < dn.g_n; ++i) {
      g.g_A[i] = dn.g_A[i]; g.g_ts[i] = dn.g_ts[i]; g.g_ts_ld[i] = dn.g_ts_ld[i]; g.g_r[i] = dn.g_r[i];
      g.g_lora_scale[i] = dn.g_lora_scale[i]; g.g_tensor_scale[i] = dn.g_tensor_scale[i];
    }
    g.tpart = (uint32_t*)(ws + L.partial_off); g.counters = (uint32_t*)ws + L.n_main_ctr;   // K-parts while token blocks alone do not fill the chip
    g.ready = (uint32_t*)ws + L.n_main_ctr + L.n_down_ctr;                                   // the hand-over words (zero between calls)
    g.done = g.ready + 2;
    g.n_prod = -1;                                                                           // not run yet: the launcher's to place
  }
  g.kpartial = (float*)(ws + L.partial_off + kFusedDownBytes); g.kpartial_bytes = gemm_split_bytes(g.M, n_sum);
  return launch_gemm(g, st);
}

// More tokens than mid_kernel takes: one launch of the LoRA down-projection for all adapters of the group, then
// one GEMM launch whose column blocks run over all members (k and v alone would fill half the chip).
static int gemm_group(const uint16_t* x, int64_t M, int64_t K, int64_t ldx, const qerl_linear_desc* d, int n,
                      uint8_t* ws, const WorkspaceLayout& L, hipStream_t st) {
  GemmArgs g{};
  g.x = x; g.ldx = ldx; g.M = M; g.K = K; g.k_tiles = ceil_div(K, kPackTileK); g.m_n = n;
  GemmArgs dn{};
  dn.x = x; dn.ldx = ldx; dn.M = M; dn.K = K; dn.k_tiles = g.k_tiles;
  uint16_t* ts = (uint16_t*)(ws + L.t_off);
  int tiles = 0;
  for (int i = 0; i < n; ++i) {
    GemmMember& m = g.m[i];
    m.packed = (const uint8_t*)d[i].packed; m.tensor_scale = d[i].tensor_scale; m.N = d[i].N;
    m.n_tiles = (int)ceil_div(d[i].N, kPackTileRows);
    m.r = (int)d[i].r; m.B = (const uint16_t*)d[i].B_bf16; m.y = (uint16_t*)d[i].y_bf16; m.ldy = d[i].ldy;
    m.bias = (const uint16_t*)d[i].bias_bf16;
    m.ext_stages = (int)ceil_div(3 * d[i].r, 64); m.ts_ld = (int64_t)m.ext_stages * 64; m.ts = ts;
    ts += M * m.ts_ld;
    if (d[i].r > 0) {
      const int gi = dn.g_n++;
      dn.g_tile0[gi] = tiles; dn.g_A[gi] = (const uint16_t*)d[i].A_bf16; dn.g_ts[gi] = m.ts; dn.g_ts_ld[gi] = m.ts_ld;
      dn.g_r[gi] = (int)d[i].r; dn.g_lora_scale[gi] = d[i].lora_scale; dn.g_tensor_scale[gi] = d[i].tensor_scale;
      tiles += (int)ceil_div(d[i].r, 32);
    }
  }
  int64_t n_sum = 0;
  for (int i = 0; i < n; ++i) n_sum += d[i].N;
  return gemm_with_down(g, dn, tiles, n_sum, ws, L, st);
}
}  // namespace qerl

#ifdef QERL_TUNING_HOOKS   // built only for tuning sessions: they change process-wide state
extern "C" QERL_API void qerl_debug_use_stream(int on) { qerl::g_use_stream = on != 0; }
extern "C" QERL_API void qerl_debug_mid_producer_bytes(long long b) { qerl::g_mid_producer_bytes = b; }
extern "C" QERL_API void qerl_debug_mid_gemm_min_rows(long long n) { qerl::g_mid_gemm_min_rows = n; }
extern "C" QERL_API void qerl_debug_gemm_min_tokens(int m) { qerl::g_gemm_min_tokens = m; }
#endif  // QERL_TUNING_HOOKS

static int packed_single(const void* x, int64_t M, int64_t K, int64_t ldx, const void* packed,
                         const float* tensor_scale, int64_t N, const void* A, const void* B,
                         int64_t r, float lora_scale, const void* bias, void* y, int64_t ldy, void* workspace,
                         size_t workspace_bytes, void* stream);

extern "C" int nvfp4_lora_linear_packed_group(const void* x, int64_t M, int64_t K, int64_t ldx,
                                              const qerl_linear_desc* members, int n_members, void* workspace,
                                              size_t workspace_bytes, void* stream) {
  if (!members) return QERL_ERR_NULL;
  if (n_members < 1 || n_members > kMaxGroup) return QERL_ERR_SHAPE;
  int64_t n_sum = 0, r_sum = 0;
  bool stream_ok = M <= 16, mid_ok = true;
  for (int i = 0; i < n_members; ++i) {
    const qerl_linear_desc& d = members[i];
    LinearCall c{(const uint16_t*)x, M, K, ldx, d.tensor_scale, d.N, (const uint16_t*)d.A_bf16, (const uint16_t*)d.B_bf16,
                 d.r, d.lora_scale, (uint16_t*)d.y_bf16, d.ldy, workspace, ~(size_t)0, (hipStream_t)stream};
    const int vr = validate(c, d.packed, d.packed);
    if (vr < 0) return vr;
    if (d.N < 1) return QERL_ERR_SHAPE;
    n_sum += d.N; r_sum += d.r;
    stream_ok = stream_ok && (d.r == 0 || (d.r <= 64 && d.r % 8 == 0 && aligned(d.A_bf16, 16) && aligned(d.B_bf16, 16)));
    mid_ok = mid_ok && (d.r == 0 || (d.r % 8 == 0 && aligned(d.A_bf16, 16) && aligned(d.B_bf16, 16)));
    if (d.r > 0 && d.t_f32 && !aligned(d.t_f32, 32)) return QERL_ERR_ALIGN;
  }
  if (M == 0) return QERL_OK;
  if (K == 0) return QERL_ERR_SHAPE;
  if (!aligned(x, 16) || ldx % 8 != 0) return QERL_ERR_ALIGN;
  const WorkspaceLayout L = workspace_layout(M, n_sum, K, r_sum);
  if (!workspace || !aligned(workspace, 256) || workspace_bytes < L.total) return QERL_ERR_WORKSPACE;
  if (stream_ok && g_use_stream)
    return stream_group((const uint16_t*)x, M, K, ldx, members, n_members, (uint8_t*)workspace, L, (hipStream_t)stream);
  // 65..128 tokens on a group with many output rows (gate + up): the prefill GEMM has enough column blocks to fill
  // the chip with one block of tokens and multiplies faster than the weight-streaming kernel (115 against 181 us
  // for the 32B pair at 128 tokens); the workspace of such a shape holds the GEMM's areas
  const bool wide = M > 64 && n_sum >= g_mid_gemm_min_rows && mid_partial_bytes(M, n_sum) >= kDownExchangeBytes;
  const bool to_gemm = M >= g_gemm_min_tokens || M > g_mid_max_tokens || (wide && n_members > 1);
  if (M > 16 && mid_ok && !to_gemm)
    return mid_group((const uint16_t*)x, M, K, ldx, members, n_members, (uint8_t*)workspace, L, (hipStream_t)stream);
  if (to_gemm && mid_ok && n_members > 1)
    return gemm_group((const uint16_t*)x, M, K, ldx, members, n_members, (uint8_t*)workspace, L, (hipStream_t)stream);
  for (int i = 0; i < n_members; ++i) {   // general case: member by member
    const qerl_linear_desc& d = members[i];
    const int rc = packed_single(x, M, K, ldx, d.packed, d.tensor_scale, d.N, d.A_bf16, d.B_bf16, d.r,
                                 d.lora_scale, d.bias_bf16, d.y_bf16, d.ldy, workspace, workspace_bytes, stream);
    if (rc != QERL_OK) return rc;
  }
  return QERL_OK;
}

extern "C" size_t nvfp4_prepack_bytes(int64_t N, int64_t K) {
  if (N <= 0 || K <= 0) return 0;
  return (size_t)ceil_div(N, kPackTileRows) * (size_t)ceil_div(K, kPackTileK) * kPackTileBytes;
}

extern "C" int nvfp4_prepack(const uint8_t* codes, const uint8_t* scales, int64_t N, int64_t K, void* packed,
                             void* stream) {
  if (N < 0 || K < 0 || K % kBlock != 0) return QERL_ERR_SHAPE;
  if (N == 0 || K == 0) return QERL_OK;
  if (!codes || !scales || !packed) return QERL_ERR_NULL;
  if (!aligned(packed, 16)) return QERL_ERR_ALIGN;
  return launch_prepack(codes, scales, N, K, (uint8_t*)packed, (hipStream_t)stream);
}

extern "C" int nvfp4_lora_linear_packed(const void* x, int64_t M, int64_t K, int64_t ldx, const void* packed,
                                        const float* tensor_scale, int64_t N, const void* A, const void* B,
                                        int64_t r, float lora_scale, void* y, int64_t ldy, void* workspace,
                                        size_t workspace_bytes, void* stream) {
  return packed_single(x, M, K, ldx, packed, tensor_scale, N, A, B, r, lora_scale, nullptr, y, ldy, workspace,
                       workspace_bytes, stream);
}

extern "C" size_t nvfp4_lora_linear_swiglu_workspace_bytes(int64_t M, int64_t N, int64_t K, int64_t r) {
  return workspace_layout(M, N, K, r).total + align256((size_t)(M > 0 ? M : 0) * (size_t)(K > 0 ? K : 0) * sizeof(uint16_t));
}

extern "C" int nvfp4_lora_linear_packed_swiglu(const void* gate, const void* up, int64_t M, int64_t K, int64_t ldg, int64_t ldu,
                                               const void* packed, const float* tensor_scale, int64_t N, const void* A,
                                               const void* B, int64_t r, float lora_scale, void* y, int64_t ldy,
                                               void* workspace, size_t workspace_bytes, void* stream) {
  LinearCall c{(const uint16_t*)gate, M, K, ldg, tensor_scale, N, (const uint16_t*)A, (const uint16_t*)B, r,
               lora_scale, (uint16_t*)y, ldy, workspace, ~(size_t)0, (hipStream_t)stream};
  const int vr = validate(c, packed, packed);
  if (vr != QERL_OK) return vr > 0 ? QERL_OK : vr;
  if (K == 0 || ldu < K) return QERL_ERR_SHAPE;
  if (!up) return QERL_ERR_NULL;
  if (!aligned(packed, 16) || !aligned(gate, 16) || ldg % 8 != 0 || !aligned(up, 16) || ldu % 8 != 0) return QERL_ERR_ALIGN;
  const WorkspaceLayout L = workspace_layout(M, N, K, r);
  const size_t act_bytes = align256((size_t)M * (size_t)K * sizeof(uint16_t));
  if (!workspace || !aligned(workspace, 256) || workspace_bytes < L.total + act_bytes) return QERL_ERR_WORKSPACE;
  uint8_t* ws = (uint8_t*)workspace;
  if (g_use_stream && M <= 16 && (r == 0 || (r <= 64 && r % 8 == 0 && aligned(A, 16) && aligned(B, 16)))) {
    // decode: the product is formed while the kernel stages its input; no intermediate tensor
    qerl_linear_desc d{packed, tensor_scale, N, A, B, r, lora_scale, y, ldy, nullptr, nullptr};
    return stream_group(c.x, M, K, ldg, &d, 1, ws, L, c.st, (const uint16_t*)up, ldu);
  }
  // more tokens: one elementwise pass into the workspace, then the linear on it
  uint16_t* act = (uint16_t*)(ws + L.total);
  const int64_t total = M * (K / 8);
  int64_t blocks = ceil_div(total, 256);
  blocks = blocks > 4096 ? 4096 : blocks;
  silu_mul_kernel<<<dim3((unsigned)blocks), dim3(256), 0, c.st>>>(c.x, ldg, (const uint16_t*)up, ldu, M, K, act);
  const int rc = launch_status();
  if (rc != QERL_OK) return rc;
  return packed_single(act, M, K, K, packed, tensor_scale, N, A, B, r, lora_scale, nullptr, y, ldy, workspace, L.total, stream);
}

static int packed_single(const void* x, int64_t M, int64_t K, int64_t ldx, const void* packed,
                         const float* tensor_scale, int64_t N, const void* A, const void* B,
                         int64_t r, float lora_scale, const void* bias, void* y, int64_t ldy, void* workspace,
                         size_t workspace_bytes, void* stream) {
  LinearCall c{(const uint16_t*)x, M, K, ldx, tensor_scale, N, (const uint16_t*)A, (const uint16_t*)B, r,
               lora_scale, (uint16_t*)y, ldy, workspace, workspace_bytes, (hipStream_t)stream};
  const int vr = validate(c, packed, packed);
  if (vr != QERL_OK) return vr > 0 ? QERL_OK : vr;
  if (K == 0) return QERL_ERR_SHAPE;
  if (!aligned(packed, 16) || !aligned(x, 16) || ldx % 8 != 0) return QERL_ERR_ALIGN;
  const WorkspaceLayout L = workspace_layout(M, N, K, r);
  uint8_t* ws = (uint8_t*)workspace;
  float* t = (float*)(ws + L.t_off);
  uint32_t* partial = (uint32_t*)(ws + L.partial_off);

  const bool lora_gemm_ok = r == 0 || (r % 8 == 0 && aligned(A, 16) && aligned(B, 16));
  if (M > 16 && M <= g_mid_max_tokens && M < g_gemm_min_tokens && lora_gemm_ok) {
    qerl_linear_desc d{packed, tensor_scale, N, A, B, r, lora_scale, y, ldy, nullptr, bias};
    return mid_group(c.x, M, K, ldx, &d, 1, ws, L, c.st);
  }
  if (M > 16 && lora_gemm_ok) {
    // Prefill: one split-K GEMM writes lora_scale * x A^T as three bf16 terms into the workspace,
    // then one GEMM computes the layer with those 3r columns appended to K.
    GemmArgs g{};
    g.x = c.x; g.ldx = ldx; g.M = M; g.K = K; g.k_tiles = ceil_div(K, kPackTileK);
    g.ts = (const uint16_t*)(ws + L.t_off); g.ext_stages = (int)ceil_div(3 * r, 64); g.ts_ld = (int64_t)g.ext_stages * 64;
    g.r = (int)r; g.lora_scale = lora_scale; g.tensor_scale = tensor_scale;
    GemmArgs dn{};
    int tiles = 0;
    if (r > 0) {
      dn.g_n = 1;
      dn.g_tile0[0] = 0; dn.g_A[0] = c.A; dn.g_ts[0] = g.ts; dn.g_ts_ld[0] = g.ts_ld; dn.g_r[0] = (int)r;
      dn.g_lora_scale[0] = lora_scale; dn.g_tensor_scale[0] = tensor_scale;
      tiles = (int)ceil_div(r, 32);
    }
    g.N = N; g.packed = (const uint8_t*)packed; g.n_tiles = (int)ceil_div(N, 32);
    g.B = c.B; g.y = c.y; g.ldy = ldy; g.bias = (const uint16_t*)bias;
    return gemm_with_down(g, dn, tiles, N, ws, L, c.st);
  }

  if (g_use_stream && M <= 16 && (r == 0 || (r <= 64 && r % 8 == 0 && aligned(A, 16) && aligned(B, 16)))) {
    qerl_linear_desc d{packed, tensor_scale, N, A, B, r, lora_scale, y, ldy, nullptr, bias};
    return stream_group(c.x, M, K, ldx, &d, 1, ws, L, c.st);
  }
  if (bias) return QERL_ERR_SHAPE;   // the remaining kernels (adapters of unusual rank or alignment) add no bias

  // Decode: passes of up to 16 tokens.  For the usual adapters (r <= 64, 16-byte aligned) the LoRA
  // down-projection runs on the first workgroups of the same launch; otherwise it gets a launch of its own.
  const bool fused_lora = r > 0 && r <= 64 && r % 8 == 0 && aligned(A, 16) && aligned(B, 16);
  for (int64_t m0 = 0; m0 < M; m0 += 16) {
    const int mc = (int)((M - m0 < 16) ? M - m0 : 16);
    const DecodePlan p = plan_decode(mc, N, K, r);
    const size_t dec_words = ((size_t)p.S * p.n_tiles * p.MR * 64 + 3) & ~(size_t)3;
    if (r > 0 && !fused_lora) {
      const int rc = lora_down_pass(c, L, m0, mc, (f32x4*)(partial + dec_words + kDecodeTpartWords));
      if (rc != QERL_OK) return rc;
    }
    DecodeArgs a{};
    a.x = c.x + m0 * ldx; a.ldx = ldx; a.M = mc; a.K = K; a.N = N;
    a.packed = (const uint8_t*)packed; a.k_tiles = p.k_tiles; a.tensor_scale = tensor_scale;
    a.A = c.A; a.B = c.B; a.r = (int)r; a.lora_scale = lora_scale;
    a.b_vec = r % 8 == 0 && aligned(B, 16);
    a.t = t + m0 * r;
    if (fused_lora) {
      int64_t np = ceil_div(2 * p.k_tiles, p.waves);   // one half K-tile per producer wave
      a.n_producers = (int)(np < 1 ? 1 : (np > 16 ? 16 : np));
      a.lora_ctl = (uint32_t*)ws + L.n_main_ctr + L.n_down_ctr;
      a.tpart = partial + dec_words;
    }
    a.y = c.y + m0 * ldy; a.ldy = ldy;
    a.partial = partial; a.counters = (uint32_t*)ws; a.n_tiles = p.n_tiles; a.S = p.S; a.n_groups = p.groups;
    const int rc = launch_decode(p, a, c.st);
    if (rc != QERL_OK) return rc;
  }
  return QERL_OK;
}

// ---- nvfp4_lora_linear_packed_noalloc: the packed linear for callers that cannot allocate ----------------------
// The scratch that nvfp4_lora_linear_packed takes as its workspace argument lives here in a file-scope device
// array instead.  Each GPU holds its own copy of the array at its own address: the address is looked up once per
// device (with that device current) and only that pointer is ever handed to kernels.
namespace qerl {
constexpr size_t kNoallocScratchBytes = (size_t)36 << 20;   // covers every single linear of the five benchmark configurations (largest: 32.7 MiB)
static __device__ __align__(256) unsigned char scratch[kNoallocScratchBytes];
constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices];   // device address of `scratch` per device, nullptr until first used there

static int noalloc_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return launch_status();
  if (dev < 0 || dev >= kMaxDevices) return QERL_ERR_SHAPE;
  void* p = __atomic_load_n(&g_scratch_ptr[dev], __ATOMIC_ACQUIRE);
  if (!p) {
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) { set_last_hip_error((int)e); (void)hipGetLastError(); return QERL_ERR_LAUNCH; }
    __atomic_store_n(&g_scratch_ptr[dev], p, __ATOMIC_RELEASE);   // racing first calls look up the same address
  }
  *out = p;
  return QERL_OK;
}
}  // namespace qerl

extern "C" size_t nvfp4_lora_linear_packed_noalloc_max_bytes(void) { return kNoallocScratchBytes; }

extern "C" int nvfp4_lora_linear_packed_noalloc(const void* x, int64_t M, int64_t K, int64_t ldx, const void* packed,
                                                const float* tensor_scale, int64_t N, const void* A, const void* B,
                                                int64_t r, float lora_scale, void* y, int64_t ldy, void* stream) {
  // every host-side check of the ordinary entry point first, against the fixed scratch size: nothing is launched
  // and no device is touched for a call that would be rejected
  LinearCall c{(const uint16_t*)x, M, K, ldx, tensor_scale, N, (const uint16_t*)A, (const uint16_t*)B, r,
               lora_scale, (uint16_t*)y, ldy, (void*)(uintptr_t)256, kNoallocScratchBytes, (hipStream_t)stream};
  const int vr = validate(c, packed, packed);
  if (vr != QERL_OK) return vr > 0 ? QERL_OK : vr;
  if (K == 0) return QERL_ERR_SHAPE;
  if (!aligned(packed, 16) || !aligned(x, 16) || ldx % 8 != 0) return QERL_ERR_ALIGN;
  void* ws = nullptr;
  const int rc = noalloc_scratch(&ws);
  if (rc != QERL_OK) return rc;
  // The array keeps whatever the last call on this GPU left in it.  What must start at zero are the control
  // words at its front; they are cleared by a fill kernel (not a memset node, so the call can be captured).
  zero_words_kernel<<<dim3(16), dim3(256), 0, (hipStream_t)stream>>>((uint32_t*)ws, kCtrlBytes / sizeof(uint32_t));
  const int zr = launch_status();
  if (zr != QERL_OK) return zr;
  return packed_single(x, M, K, ldx, packed, tensor_scale, N, A, B, r, lora_scale, nullptr, y, ldy, ws,
                       kNoallocScratchBytes, stream);
}
