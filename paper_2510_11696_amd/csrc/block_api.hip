// C-ABI entry points of the fused decode launches (block_kernel, linear_block.hip):
//   aqn_rmsnorm_nvfp4_lora_linear_group  RMSNorm with noisy gain (Eq. 10) -> up to four NVFP4 + LoRA linears (Eq. 6, Eq. 2)
//   aqn_rmsnorm_nvfp4_lora_mlp           RMSNorm -> gate_proj, up_proj -> SiLU(gate) (.) up -> down_proj
// one launch each up to 16 tokens; beyond that they run the same operators as separate launches.
#include <stdlib.h>
#include "linear.hpp"

namespace qerl {

static size_t blk_align256(size_t v) { return (v + 255) & ~(size_t)255; }

// Workspace of a block launch: the control region every linear workspace starts with (arrival words of the tiles,
// hand-over words), the producers' partial t of up to three stages, the K-ranges' partial tiles, and room for
// intermediate activations.
struct BlkWorkspace { size_t tpart_off, tfinal_off, partial_off, act_off, total; };
static BlkWorkspace blk_workspace(size_t partial_floats, size_t act_bytes) {
  BlkWorkspace w;
  w.tpart_off = kCtrlRegionBytes;
  w.tfinal_off = w.tpart_off + blk_align256((size_t)kBlkMaxStages * kBlkTpartWords * sizeof(uint32_t));
  w.partial_off = w.tfinal_off + blk_align256((size_t)kBlkMaxStages * kBlkTfinalWords * sizeof(float));
  w.act_off = w.partial_off + blk_align256(partial_floats * sizeof(float));
  w.total = w.act_off + blk_align256(act_bytes);
  return w;
}

// One stage from the caller's descriptors.  Returns a status; checks what the kernel's indexing assumes.
static int blk_fill_stage(BlkStage& S, const void* x, int64_t K, int64_t ldx, const void* gain, const float* noise, float eps,
                          const qerl_linear_desc* const* d, int n, bool pairs) {
  if (n < 1 || n > kMaxGroup) return QERL_ERR_SHAPE;
  if (K < 16 || K % kBlock != 0 || ldx < K) return QERL_ERR_SHAPE;
  if (!x) return QERL_ERR_NULL;
  if (!aligned(x, 16) || ldx % 8 != 0) return QERL_ERR_ALIGN;
  if (gain && (!aligned(gain, 16) || (noise && !aligned(noise, 16)) || K % 8 != 0)) return QERL_ERR_ALIGN;
  S = BlkStage{};
  S.x = (const uint16_t*)x; S.ldx = ldx; S.K = K; S.k_tiles = (int)ceil_div(K, kPackTileK);
  S.gain = (const uint16_t*)gain; S.noise = gain ? noise : nullptr; S.eps = eps;
  S.n_members = n; S.pairs = pairs ? 1 : 0;
  int tiles = 0;
  for (int i = 0; i < n; ++i) {
    const qerl_linear_desc& m = *d[i];
    if (m.N < 1 || m.r < 0 || m.N / 16 >= 16384) return QERL_ERR_SHAPE;
    if (!m.packed || !m.tensor_scale) return QERL_ERR_NULL;
    if (!pairs && (!m.y_bf16 || m.ldy < m.N)) return m.y_bf16 ? QERL_ERR_SHAPE : QERL_ERR_NULL;
    if (m.r > 0 && (!m.A_bf16 || !m.B_bf16)) return QERL_ERR_NULL;
    if (!aligned(m.packed, 16) || (m.y_bf16 && !aligned(m.y_bf16, 2)) || (m.bias_bf16 && !aligned(m.bias_bf16, 2))) return QERL_ERR_ALIGN;
    if (m.r > 0 && (m.r > 64 || m.r % 8 != 0 || !aligned(m.A_bf16, 16) || !aligned(m.B_bf16, 16))) return QERL_ERR_SHAPE;
    BlkMember& b = S.mem[i];
    b.packed = (const uint8_t*)m.packed; b.tensor_scale = m.tensor_scale;
    b.A = (const uint16_t*)m.A_bf16; b.B = (const uint16_t*)m.B_bf16; b.bias = (const uint16_t*)m.bias_bf16;
    b.y = (uint16_t*)m.y_bf16; b.ldy = m.ldy; b.N = m.N; b.n_tiles = (int)ceil_div(m.N, kPackTileRows); b.tile_begin = tiles;
    b.r = (int)m.r; b.lora_scale = m.lora_scale;
    b.stride_k = kPackTileBytes; b.stride_n = (int64_t)S.k_tiles * kPackTileBytes;
#ifdef QERL_TUNING_HOOKS   // timing experiment only (the weights are NOT in that order: results are wrong)
    if (getenv("QERL_BLK_KMAJOR_TIMING")) { b.stride_n = kPackTileBytes; b.stride_k = (int64_t)b.n_tiles * kPackTileBytes; }
    if (getenv("QERL_BLK_SAMETILE_TIMING")) { b.stride_n = 0; b.stride_k = 0; }   // every unit reads one tile: no memory traffic to speak of
#endif
    b.y_vec = (m.y_bf16 && aligned(m.y_bf16, 16) && m.ldy % 8 == 0) ? 1 : 0;
    tiles += b.n_tiles;
  }
  for (int i = n; i < kMaxGroup; ++i) {   // unused entries: never selected, but valid to read
    S.mem[i] = S.mem[0];
    S.mem[i].tile_begin = 0x7fffffff; S.mem[i].n_tiles = 0; S.mem[i].r = 0;
  }
  S.total_tiles = tiles;
  S.total_v = pairs ? S.mem[0].n_tiles : tiles;
  if (pairs && (n != 2 || S.mem[0].N != S.mem[1].N)) return QERL_ERR_SHAPE;
  return QERL_OK;
}

static int blk_plan_and_launch(BlkArgs& a, uint8_t* ws, size_t ws_bytes, size_t act_bytes, bool launch, size_t* need, hipStream_t st) {
  size_t lds = 0, part = 0, ctrs = 0;
  int MR = 4;
  const int prc = plan_block(a, &lds, &MR, &part, &ctrs);
  if (prc != QERL_OK) return prc;
  if (ctrs > kCtrlMainWords) return QERL_ERR_SHAPE;
  const BlkWorkspace w = blk_workspace(part, act_bytes);
  if (need) *need = w.total;
  if (!launch) {
    // sizing call: the plan must also pass the launch's own checks (placeholder workspace pointers, nothing is launched),
    // so that a shape the kernel cannot take reports 0 bytes here rather than an error at the first call
    BlkArgs b = a;
    b.counters = b.ctl = b.tpart = (uint32_t*)(uintptr_t)256; b.tfinal = b.partial = (float*)(uintptr_t)256;
    return check_block(b, lds, MR);
  }
  if (!ws || !aligned(ws, 256) || ws_bytes < w.total) return QERL_ERR_WORKSPACE;
  a.counters = (uint32_t*)ws;
  a.ctl = (uint32_t*)ws + kCtrlMainWords + kCtrlDownWords;
  a.tpart = (uint32_t*)(ws + w.tpart_off);
  a.tfinal = (float*)(ws + w.tfinal_off);
  a.partial = (float*)(ws + w.partial_off);
  return launch_block(a, lds, MR, st);
}

}  // namespace qerl

using namespace qerl;

static int group_impl(const void* x, int64_t M, int64_t K, int64_t ldx, const void* gain, const float* noise, float eps,
                      const qerl_linear_desc* members, int n, void* workspace, size_t bytes, void* stream, bool launch, size_t* need) {
  if (!members) return QERL_ERR_NULL;
  if (n < 1 || n > kMaxGroup || M < 0) return QERL_ERR_SHAPE;
  const qerl_linear_desc* d[kMaxGroup] = {};
  int64_t n_sum = 0, r_sum = 0;
  for (int i = 0; i < n; ++i) { d[i] = members + i; n_sum += members[i].N; r_sum += members[i].r; }
  if (M == 0 && launch) return QERL_OK;
  if (M <= 16) {
    BlkArgs a{};
    a.M = (int)(M > 0 ? M : 1); a.n_stages = 1;
    const int rc = blk_fill_stage(a.st[0], launch ? x : (const void*)(uintptr_t)256, K, ldx, gain, noise, eps, d, n, false);
    if (rc != QERL_OK) return rc;
    return blk_plan_and_launch(a, (uint8_t*)workspace, bytes, 0, launch, need, (hipStream_t)stream);
  }
  // more tokens: the norm's launch (output in the workspace), then the grouped linear
  const size_t lin = nvfp4_lora_linear_workspace_bytes(M, n_sum, K, r_sum);
  const size_t xn_bytes = gain ? blk_align256((size_t)M * (size_t)K * sizeof(uint16_t)) : 0;
  if (need) *need = lin + xn_bytes;
  if (!launch) return QERL_OK;
  if (!workspace || !aligned(workspace, 256) || bytes < lin + xn_bytes) return QERL_ERR_WORKSPACE;
  const void* xin = x;
  int64_t ldin = ldx;
  if (gain) {
    uint16_t* xn = (uint16_t*)((uint8_t*)workspace + lin);
    const int rc = aqn_rmsnorm(x, M, K, ldx, gain, noise, eps, xn, K, stream);
    if (rc != QERL_OK) return rc;
    xin = xn; ldin = K;
  }
  return nvfp4_lora_linear_packed_group(xin, M, K, ldin, members, n, workspace, lin, stream);
}

extern "C" size_t aqn_rmsnorm_nvfp4_lora_linear_group_workspace_bytes(int64_t M, int64_t K, const int64_t* Ns, const int64_t* rs, int n) {
  if (!Ns || !rs || n < 1 || n > kMaxGroup) return 0;
  qerl_linear_desc d[kMaxGroup] = {};
  for (int i = 0; i < n; ++i) {   // placeholders that pass the pointer checks; nothing is dereferenced or launched
    d[i].packed = (const void*)(uintptr_t)256; d[i].tensor_scale = (const float*)(uintptr_t)256; d[i].N = Ns[i];
    d[i].A_bf16 = (const void*)(uintptr_t)256; d[i].B_bf16 = (const void*)(uintptr_t)256; d[i].r = rs[i];
    d[i].y_bf16 = (void*)(uintptr_t)256; d[i].ldy = Ns[i];
  }
  size_t need = 0;
  const int rc = group_impl(nullptr, M, K, K, (const void*)(uintptr_t)256, nullptr, 0.f, d, n, nullptr, 0, nullptr, false, &need);
  return rc == QERL_OK ? need : 0;
}

extern "C" int aqn_rmsnorm_nvfp4_lora_linear_group(const void* x, int64_t M, int64_t K, int64_t ldx, const void* gain,
                                                   const float* noise, float eps, const qerl_linear_desc* members, int n_members,
                                                   void* workspace, size_t workspace_bytes, void* stream) {
  return group_impl(x, M, K, ldx, gain, noise, eps, members, n_members, workspace, workspace_bytes, stream, true, nullptr);
}

static int mlp_impl(const void* x, int64_t M, int64_t H, int64_t ldx, const void* gain, const float* noise, float eps,
                    const qerl_linear_desc* gate, const qerl_linear_desc* up, const qerl_linear_desc* down,
                    void* workspace, size_t bytes, void* stream, bool launch, size_t* need) {
  if (!gate || !up || !down) return QERL_ERR_NULL;
  if (M < 0 || gate->N != up->N || gate->N < 1) return QERL_ERR_SHAPE;
  const int64_t I = gate->N;
  if (I % 8 != 0) return QERL_ERR_SHAPE;             // act rows are staged with 16-byte accesses
  if (M == 0 && launch) return QERL_OK;
  if (launch && (!down->y_bf16 || down->ldy < down->N)) return down->y_bf16 ? QERL_ERR_SHAPE : QERL_ERR_NULL;
  const size_t act_bytes = blk_align256((size_t)(M > 0 ? M : 1) * (size_t)I * sizeof(uint16_t));
  if (M <= 16) {
    BlkArgs a{};
    a.M = (int)(M > 0 ? M : 1); a.n_stages = 2;
    const qerl_linear_desc* gu[2] = {gate, up};
    int rc = blk_fill_stage(a.st[0], launch ? x : (const void*)(uintptr_t)256, H, ldx, gain, noise, eps, gu, 2, true);
    if (rc != QERL_OK) return rc;
    // the activation's place is known once the plan (size of the partial tiles) is: plan with a placeholder first
    const qerl_linear_desc* dn[1] = {down};
    rc = blk_fill_stage(a.st[1], (const void*)(uintptr_t)256, I, I, nullptr, nullptr, 0.f, dn, 1, false);
    if (rc != QERL_OK) return rc;
    a.st[0].act = (uint16_t*)(uintptr_t)256; a.st[0].ld_act = I; a.st[0].act_vec = 1;
    size_t lds = 0, part = 0, ctrs = 0;
    int MR = 4;
    rc = plan_block(a, &lds, &MR, &part, &ctrs);
    if (rc != QERL_OK) return rc;
    if (ctrs > kCtrlMainWords) return QERL_ERR_SHAPE;
    const BlkWorkspace w = blk_workspace(part, act_bytes);
    if (need) *need = w.total;
    if (!launch) return QERL_OK;
    uint8_t* ws = (uint8_t*)workspace;
    if (!ws || !aligned(ws, 256) || bytes < w.total) return QERL_ERR_WORKSPACE;
    uint16_t* act = (uint16_t*)(ws + w.act_off);
    a.st[0].act = act; a.st[1].x = act;
    a.counters = (uint32_t*)ws;
    a.ctl = (uint32_t*)ws + kCtrlMainWords + kCtrlDownWords;
    a.tpart = (uint32_t*)(ws + w.tpart_off);
    a.tfinal = (float*)(ws + w.tfinal_off);
    a.partial = (float*)(ws + w.partial_off);
    return launch_block(a, lds, MR, (hipStream_t)stream);
  }
  // more tokens: norm, grouped gate + up, down on the gated input, as separate launches; the intermediates live in
  // the workspace behind the linear's own area
  const size_t lin_gu = nvfp4_lora_linear_workspace_bytes(M, 2 * I, H, gate->r + up->r);
  const size_t lin_dn = nvfp4_lora_linear_swiglu_workspace_bytes(M, down->N, I, down->r);
  const size_t lin = lin_gu > lin_dn ? lin_gu : lin_dn;
  const size_t xn_bytes = gain ? blk_align256((size_t)M * (size_t)H * sizeof(uint16_t)) : 0;
  if (need) *need = lin + xn_bytes + 2 * act_bytes;
  if (!launch) return QERL_OK;
  uint8_t* ws = (uint8_t*)workspace;
  if (!ws || !aligned(ws, 256) || bytes < lin + xn_bytes + 2 * act_bytes) return QERL_ERR_WORKSPACE;
  const void* xin = x;
  int64_t ldin = ldx;
  if (gain) {
    uint16_t* xn = (uint16_t*)(ws + lin);
    const int rc = aqn_rmsnorm(x, M, H, ldx, gain, noise, eps, xn, H, stream);
    if (rc != QERL_OK) return rc;
    xin = xn; ldin = H;
  }
  qerl_linear_desc gu[2] = {*gate, *up};
  gu[0].y_bf16 = ws + lin + xn_bytes; gu[0].ldy = I; gu[0].t_f32 = nullptr;
  gu[1].y_bf16 = ws + lin + xn_bytes + act_bytes; gu[1].ldy = I; gu[1].t_f32 = nullptr;
  int rc = nvfp4_lora_linear_packed_group(xin, M, H, ldin, gu, 2, ws, lin, stream);
  if (rc != QERL_OK) return rc;
  if (down->bias_bf16) return QERL_ERR_SHAPE;   // (the gated entry point takes no bias)
  return nvfp4_lora_linear_packed_swiglu(gu[0].y_bf16, gu[1].y_bf16, M, I, I, I, down->packed, down->tensor_scale, down->N,
                                         down->A_bf16, down->B_bf16, down->r, down->lora_scale, down->y_bf16, down->ldy, ws, lin, stream);
}

extern "C" size_t aqn_rmsnorm_nvfp4_lora_mlp_workspace_bytes(int64_t M, int64_t H, int64_t I, int64_t N_down, int64_t r_gate,
                                                             int64_t r_up, int64_t r_down) {
  const void* ph = (const void*)(uintptr_t)256;
  qerl_linear_desc g{}, u{}, d{};
  g.packed = ph; g.tensor_scale = (const float*)ph; g.N = I; g.A_bf16 = ph; g.B_bf16 = ph; g.r = r_gate;
  u = g; u.r = r_up;
  d = g; d.N = N_down; d.r = r_down; d.y_bf16 = (void*)(uintptr_t)256; d.ldy = N_down;
  size_t need = 0;
  const int rc = mlp_impl(nullptr, M, H, H, ph, nullptr, 0.f, &g, &u, &d, nullptr, 0, nullptr, false, &need);
  return rc == QERL_OK ? need : 0;
}

extern "C" int aqn_rmsnorm_nvfp4_lora_mlp(const void* x, int64_t M, int64_t H, int64_t ldx, const void* gain, const float* noise,
                                          float eps, const qerl_linear_desc* gate, const qerl_linear_desc* up,
                                          const qerl_linear_desc* down, void* workspace, size_t workspace_bytes, void* stream) {
  return mlp_impl(x, M, H, ldx, gain, noise, eps, gate, up, down, workspace, workspace_bytes, stream, true, nullptr);
}

// Sticky error word of a linear / block workspace: non-zero after a kernel's bounded wait on another workgroup gave
// up (a result of that call is then unreliable, and the workspace must be prepared again with qerl_workspace_init).
// Synchronises with the stream.
extern "C" int qerl_workspace_status(const void* workspace, void* stream) {
  if (!workspace) return QERL_ERR_NULL;
  if (!aligned(workspace, 256)) return QERL_ERR_ALIGN;
  uint32_t word = 0;
  const uint32_t* p = (const uint32_t*)workspace + kCtrlMainWords + kCtrlDownWords + kCtlErr;
  if (hipMemcpyAsync(&word, p, sizeof(word), hipMemcpyDeviceToHost, (hipStream_t)stream) != hipSuccess) return launch_status();
  if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return launch_status();
  return qerl_status_from_error_word(word);
}

extern "C" int qerl_status_from_error_word(uint32_t word) { return word == 0u ? QERL_OK : QERL_ERR_TIMEOUT; }

extern "C" int qerl_selftest_wait_gives_up(void* workspace, size_t workspace_bytes, uint32_t polls, void* stream) {
  if (!workspace) return QERL_ERR_NULL;
  if (!aligned(workspace, 256) || workspace_bytes < kCtrlRegionBytes) return QERL_ERR_WORKSPACE;
  if (polls < 1 || polls > 1024) return QERL_ERR_SHAPE;   // a self-test, not a way to keep a wave spinning
  return launch_block_wait_selftest((uint32_t*)workspace + kCtrlMainWords + kCtrlDownWords, polls, (hipStream_t)stream);
}
