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
struct WorkspaceLayout { size_t ctrl_bytes, n_main_ctr, t_off, partial_off, total; };

constexpr size_t kMaxCounterTiles = 1 << 16;   // rows / 16 the control region can serve

static size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

static WorkspaceLayout workspace_layout(int64_t M, int64_t N, int64_t K, int64_t r) {
  WorkspaceLayout L;
  L.n_main_ctr = (size_t)ceil_div(N > 0 ? N : 1, 16);
  const size_t n_down_ctr = (size_t)ceil_div(r > 0 ? r : 1, 16);
  L.ctrl_bytes = align256((L.n_main_ctr + n_down_ctr) * sizeof(uint32_t));
  L.t_off = L.ctrl_bytes;
  const size_t t_bytes = align256((size_t)(M > 0 ? M : 1) * (size_t)(r > 0 ? r : 1) * sizeof(float));
  L.partial_off = L.t_off + t_bytes;
  // worst case over the plans the dispatcher can choose: one K-tile per wave
  const size_t S_max = (size_t)ceil_div(ceil_div(K > 0 ? K : 1, 256), 8);
  const size_t tiles = L.n_main_ctr + n_down_ctr;
  L.total = L.partial_off + align256(S_max * tiles * 64 * sizeof(f32x4));
  return L;
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

extern "C" int nvfp4_lora_linear(const void* x, int64_t M, int64_t K, int64_t ldx, const uint8_t* codes,
                                 const uint8_t* scales, const float* tensor_scale, int64_t N,
                                 const void* A, const void* B, int64_t r, float lora_scale, void* y,
                                 int64_t ldy, void* workspace, size_t workspace_bytes, void* stream) {
  if (M < 0 || N < 0 || K < 0 || r < 0 || K % kBlock != 0 || ldx < K || ldy < N) return QERL_ERR_SHAPE;
  if (N / 16 >= (int64_t)kMaxCounterTiles || r > 4096) return QERL_ERR_SHAPE;
  if (M == 0 || N == 0) return QERL_OK;
  if (!x || !y || !tensor_scale) return QERL_ERR_NULL;
  if (K > 0 && (!codes || !scales)) return QERL_ERR_NULL;
  if (r > 0 && (!A || !B)) return QERL_ERR_NULL;
  if (!aligned(x, 2) || !aligned(y, 2) || (r > 0 && (!aligned(A, 2) || !aligned(B, 2)))) return QERL_ERR_ALIGN;
  const WorkspaceLayout L = workspace_layout(M, N, K, r);
  if (!workspace || !aligned(workspace, 256) || workspace_bytes < L.total) return QERL_ERR_WORKSPACE;

  hipStream_t st = (hipStream_t)stream;
  uint8_t* ws = (uint8_t*)workspace;
  uint32_t* ctr_main = (uint32_t*)ws;
  uint32_t* ctr_down = ctr_main + L.n_main_ctr;
  float* t = (float*)(ws + L.t_off);
  f32x4* partial = (f32x4*)(ws + L.partial_off);
  const uint16_t* xp = (const uint16_t*)x;
  uint16_t* yp = (uint16_t*)y;
  if (K == 0) r = 0;   // empty sums: y = 0 through the general kernel

  // The tiled kernels use 16-byte loads; anything else goes to the general kernels.
  const bool tiled = (K % 64 == 0) && K > 0 && aligned(x, 16) && ldx % 8 == 0 && aligned(codes, 16) &&
                     aligned(scales, 4) && (r == 0 || aligned(A, 16));
  if (!tiled) {
    int rc = QERL_OK;
    if (r > 0) rc = launch_generic_lora_down(xp, ldx, M, K, (const uint16_t*)A, r, t, st);
    if (rc != QERL_OK) return rc;
    return launch_generic_linear(xp, ldx, M, K, codes, scales, tensor_scale, N, r > 0 ? t : nullptr,
                                 (const uint16_t*)B, r, lora_scale, yp, ldy, st);
  }

  // Tiled path: passes of up to 16 tokens through the skinny kernels.
  const SkinnyPlan pm = plan_skinny(N, K, kFmtNvfp4);
  const SkinnyPlan pd = plan_skinny(r > 0 ? r : 1, K, kFmtBf16);
  for (int64_t m0 = 0; m0 < M; m0 += 16) {
    const int mc = (int)((M - m0 < 16) ? M - m0 : 16);
    SkinnyArgs a{};
    a.x = xp + m0 * ldx; a.ldx = ldx; a.M = mc; a.K = K;
    if (r > 0) {
      SkinnyArgs d = a;
      d.N = r; d.wbf16 = (const uint16_t*)A; d.t_out = t + m0 * r;
      d.partial = partial + (size_t)pm.S * pm.n_tiles * 64; d.counters = ctr_down; d.n_tiles = pd.n_tiles;
      const int rc = launch_skinny(pd, d, kFmtBf16, st);
      if (rc != QERL_OK) return rc;
    }
    a.N = N; a.codes = codes; a.scales = scales; a.tensor_scale = tensor_scale;
    a.t_in = t + m0 * r; a.B = (const uint16_t*)B; a.r = (int)r; a.lora_scale = lora_scale;
    a.y = yp + m0 * ldy; a.ldy = ldy;
    a.y_vec = aligned(y, 8) && ldy % 4 == 0;
    a.b_vec = r % 8 == 0 && aligned(B, 16);
    a.partial = partial; a.counters = ctr_main; a.n_tiles = pm.n_tiles;
    const int rc = launch_skinny(pm, a, kFmtNvfp4, st);
    if (rc != QERL_OK) return rc;
  }
  return QERL_OK;
}
