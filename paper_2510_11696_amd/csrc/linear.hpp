// Internal interfaces between the linear-layer translation units.
#pragma once
#include "common.hpp"

namespace qerl {

constexpr int kMaxGroup = 4;   // linears that can share one launch (they read the same x)
// Control region at the front of every linear workspace (fixed size and position, zero between calls):
constexpr size_t kCtrlMainWords = 16384;   // arrival counters of the main kernels: N / 16 <= 16384
constexpr size_t kCtrlDownWords = 256;     // arrival counters of the LoRA down-projection kernel: r / 16 <= 256
constexpr size_t kCtrlRegionBytes = (kCtrlMainWords + kCtrlDownWords + 64) * sizeof(uint32_t);   // + 64 hand-over words, 256-multiple
constexpr int kFmtNvfp4 = 0;   // rows are NVFP4 (codes + scales)
constexpr int kFmtBf16 = 1;    // rows are dense bf16 (the LoRA A matrix); output is fp32 t

struct SkinnyArgs {
  const uint16_t* x; int64_t ldx; int M; int64_t K; int64_t N;
  const uint8_t* codes; const uint8_t* scales; const float* tensor_scale;   // kFmtNvfp4
  const uint16_t* wbf16;                                                    // kFmtBf16: [N, K]
  const float* t_in; const uint16_t* B; int r; float lora_scale;            // LoRA up (kFmtNvfp4)
  uint16_t* y; int64_t ldy; bool y_vec, b_vec;                              // kFmtNvfp4 output; 8/16-byte access allowed
  float* t_out;                                                             // kFmtBf16 output [M, N]
  f32x4* partial; uint32_t* counters; int n_tiles;
};

struct SkinnyPlan { int KT, T, S, waves, n_tiles, groups; };
SkinnyPlan plan_skinny(int64_t N, int64_t K, int fmt);
int launch_skinny(const SkinnyPlan& p, const SkinnyArgs& a, int fmt, hipStream_t st);

// ---- decode path on tile-packed weights (linear_decode.hip) ----
constexpr int kPackTileRows = 32;     // output rows per tile
constexpr int kPackTileK = 128;       // inputs per tile (8 scale blocks)
constexpr int kPackTileBytes = 2304;  // 2048 B codes + 256 B scales = 0.5625 B per weight

struct DecodeArgs {
  const uint16_t* x; int64_t ldx; int M; int64_t K; int64_t N;
  const uint8_t* packed; int64_t k_tiles; const float* tensor_scale;
  const uint16_t* A; const uint16_t* B; int r; float lora_scale; bool b_vec;
  float* t;                        // [M, r] fp32: x A^T (read; written by the producer workgroups when n_producers > 0)
  int n_producers;                 // workgroups at the front of the grid that compute t in this launch (0: t is ready)
  uint32_t* lora_ctl; uint32_t* tpart;   // 3 control words; producer partial sums
  uint16_t* y; int64_t ldy;
  uint32_t* partial; uint32_t* counters; int n_tiles; int S; int n_groups;
};
struct DecodePlan { int KW, T, MR, S, main_waves, waves, n_tiles, groups; int64_t k_tiles; };
DecodePlan plan_decode(int64_t M, int64_t N, int64_t K, int64_t r);
int launch_decode(const DecodePlan& p, const DecodeArgs& a, hipStream_t st);
int launch_prepack(const uint8_t* codes, const uint8_t* scales, int64_t N, int64_t K, uint8_t* out,
                   hipStream_t st);

// ---- streaming decode kernel for one linear or a group sharing x (linear_stream.hip) ----
struct StreamMember {
  const uint8_t* packed; const float* tensor_scale; const uint16_t* A; const uint16_t* B; uint16_t* y;
  int64_t ldy; int64_t N; int n_tiles; int tile_begin;   // row-tiles [tile_begin, tile_begin + n_tiles) of the group
  int r; int t_off;                                      // rank; column offset of this member's t in the stacked t (INT_MAX if t_ext)
  int y_vec;                                             // y rows allow 16-byte stores (aligned base, ldy % 8 == 0)
  const float* t_ext;                                    // x A^T computed before the launch, fp32 [QERL_T_PARTS][M][r] partial sums, or null: producers compute it
  const uint16_t* bias;                                  // [N] bf16 added to every token row, or null
  float lora_scale;
};
struct StreamArgs {
  const uint16_t* x; int64_t ldx; int M; int64_t K; int k_tiles;
  const uint16_t* x2; int64_t ldx2;                       // not null: the input is SiLU(x) (.) x2, formed while x is staged
  int n_members; StreamMember mem[kMaxGroup];
  // flat copy of what the streaming loop needs of the member table (unused entries: INT_MAX / member 0's pointer)
  int tb1, tb2, tb3; const uint8_t* mp0; const uint8_t* mp1; const uint8_t* mp2; const uint8_t* mp3;
  int total_tiles; int r_total; int any_lora; int any_bias;            // row-tiles; stacked rank the producers compute; any member with r > 0
  int Sk; int kr_len; int per_range; int n_producers;    // K-ranges, K-tiles in each, consumer workgroups per range; producers
  int units_base; int units_rem;                         // consumer ci owns units_base (+1 if ci < units_rem) row-tiles
  int prod_steps; int prod_cb; int prod_red_off;          // producers: 16-input steps of K each, steps per LDS column block, offset of their reduction area
  int xs_stride; int red_off; int pend_off; int tsum_off;   // LDS layout (bytes): x row stride, reduction buffers, parked units, t of a member
  int red_bufs; int max_pending; int pend_steps;          // reduction buffers, parking slots, 16-rank steps of B parked per slot
  float* t; uint32_t* lora_ctl; uint32_t* tpart;         // stacked t [M, r_total]; hand-over words; producer partials
  uint32_t* partial; uint32_t* counters;                 // K-range exchange
};
int plan_stream(StreamArgs& a, size_t* lds_bytes, int* MR);
int launch_stream(const StreamArgs& a, size_t lds_bytes, int MR, hipStream_t st);

// ---- persistent multi-stage decode kernel (linear_block.hip) ----
#ifndef QERL_BLK_WAVES
#define QERL_BLK_WAVES 8
#endif
constexpr int kBlkWaves = QERL_BLK_WAVES;   // waves per workgroup, one workgroup per CU
constexpr int kBlkMaxStages = 3;         // dependent stages in one launch
constexpr int kBlkMaxProducers = 32;     // producer workgroups of a stage
constexpr size_t kBlkTpartWords = (size_t)kBlkMaxProducers * 16 * 256;   // per stage: producers along K x tokens x stacked rank
constexpr size_t kBlkTfinalWords = 16 * 256;   // per stage: the finished t, tokens x stacked rank
// control words of the block kernel, relative to the hand-over words of the workspace's control region
constexpr int kBlkArrive = 8;            // + stage: producers of that stage that have stored their partial t
constexpr int kBlkBarrier = 12;          // workgroups past the stage boundaries so far
constexpr int kBlkExit = 13;             // workgroups that have left
constexpr int kBlkReady = 20;            // + stage: the stage's t is complete in memory
constexpr int kCtlErr = 16;              // sticky: a bounded wait gave up (bit 0 stage boundary, bit 1 LoRA hand-over, bit 2 another kernel's hand-over)
struct BlkMember {
  const uint8_t* packed; const float* tensor_scale; const uint16_t* A; const uint16_t* B; const uint16_t* bias;
  uint16_t* y; int64_t ldy; int64_t N; int n_tiles; int tile_begin;   // row tiles [tile_begin, tile_begin + n_tiles) of the stage (unused entries: INT_MAX)
  int r; int t_off; float lora_scale; int y_vec;                       // rank; column of this member's t in the stage's stacked t; y rows allow 16-byte stores
  int64_t stride_k; int64_t stride_n;                                  // bytes from a packed tile to the next K-tile of its row tile / to the same K-tile of the next row tile
};
struct BlkStage {
  const uint16_t* x; int64_t ldx; int64_t K; int k_tiles;              // input [M, K]: memory written before the launch, or by the previous stage
  const uint16_t* gain; const float* noise; float eps;                 // gain != null: the input is the AQN RMSNorm of x (Eq. 10)
  int n_members; BlkMember mem[kMaxGroup];
  int total_tiles; int total_v;                                        // row tiles of all members; units a wave takes whole (pairs: one per gate / up tile pair)
  int pairs; uint16_t* act; int64_t ld_act; int act_vec;               // members 0, 1 are gate_proj, up_proj: act[M, N] = SiLU(gate) (.) up is stored instead of their outputs
  int Sk; int phases; int kr_len; int per_range;                       // K is cut into Sk ranges (of workgroups) x phases (in time) x kr_len K-tiles (a multiple of the ring depth); consumer workgroups per range
  int n_producers; int prod_k; int r_total; int prod_steps; int prod_cb; int prod_red_off;   // LoRA down-projection of the stage (lora_producer.hpp): producer workgroups = pairs of rank tiles x prod_k runs of K
  int ctr_off; int64_t partial_off;                                    // this stage's arrival words / partial tiles (floats) in the workspace areas
};
struct BlkArgs {
  int M; int n_stages; int n_wgs; int n_prod_max;                      // workgroups [0, n_prod_max) are the producers of every stage
  BlkStage st[kBlkMaxStages];
  int g_lds_off; int t_lds_off; int y_lds_off; int p_lds_off; int e_lds_off;   // LDS behind the x slice: gain + noise of the slice; split t of the members; one output tile per wave; parked accumulators; the pairs' hand-over
  int park_units;                                                      // parked accumulator tiles per wave (stages with several phases)
  uint32_t* ctl; uint32_t* counters; float* partial; uint32_t* tpart; float* tfinal;
};
int plan_block(BlkArgs& a, size_t* lds_bytes, int* MR, size_t* partial_floats, size_t* counter_words);
int launch_block_wait_selftest(uint32_t* ctl, uint32_t polls, hipStream_t st);   // error-path self-test: a bounded wait that gives up
int check_block(const BlkArgs& a, size_t lds, int MR);   // the launch's own validation, without the launch
int launch_block(const BlkArgs& a, size_t lds_bytes, int MR, hipStream_t st);

// ---- prefill path: MFMA GEMM on tile-packed weights (linear_gemm.hip) ----
// One linear of a prefill launch: gemm32_kernel's column blocks run over the members of a group that reads the
// same x (q + k + v, gate + up); a single linear is a group of one, filled in from the GemmArgs fields of the
// same names by launch_gemm.
struct GemmMember {
  const uint8_t* packed; const float* tensor_scale; int64_t N; int n_tiles;
  const uint16_t* ts; int64_t ts_ld; int ext_stages;                        // [M, ts_ld] bf16: hi | mid | lo of lora_scale / S32 * t; stages of 64 columns
  const uint16_t* B; int r;
  const uint16_t* bias;                                                     // [N] bf16 or null
  uint16_t* y; int64_t ldy;
  int block_begin;                                                          // first column block of this member (set by the launcher)
  int64_t col0;                                                             // K split over workgroups: this member's first column in the partial outputs (set by the launcher)
};
struct GemmSeg {
  const uint16_t* x; int64_t ldx; int64_t K; const uint8_t* packed; int64_t k_tiles; const float* tensor_scale;
  const uint16_t* ts; int64_t ts_ld; int ext_stages; const uint16_t* B; int r;
};
struct GemmArgs {
  const uint16_t* x; int64_t ldx; int64_t M; int64_t K; int64_t N;
  const uint8_t* packed; int64_t k_tiles; const float* tensor_scale;        // kFmtNvfp4 weights
  const uint16_t* wbf16;                                                    // kFmtBf16: [N, K] dense rows (LoRA A)
  const uint16_t* ts; int64_t ts_ld; int ext_stages;                        // [M, ts_ld] bf16: hi | mid | lo of lora_scale * t
  const uint16_t* B; int r; float lora_scale;
  const uint16_t* bias;                                                     // [N] bf16 or null
  uint16_t* y; int64_t ldy;
  int n_tiles; int n_blocks; int nblk_per_xcd;
  int m_n; GemmMember m[kMaxGroup];                                         // the main launch's members (m_n == 0: one, from the fields above)
  int transposed;                                                           // packed is in nvfp4_prepack_t's order: K counts rows of W, N its columns
  // transposed launches only: the contraction runs over seg_n segments one after the other -- the members of a group
  // of linears that read the same x, each with its own dY (x, ldx), rows (K), transposed tiles, tensor scale and LoRA
  // columns (ts = three terms of lora_scale / S32 * dY B; B = A^T [N, r]).  seg_n == 0: one segment, from the
  // fields above and m[0].
  int seg_n; GemmSeg seg[kMaxGroup];
  // K split over workgroups (forward launches that would leave most of the chip idle): the caller offers kpartial,
  // kpartial_bytes of scratch; the launcher decides on ksplit parts, whose sums (LoRA columns in part 0) go there as
  // fp32 [ksplit][M][kp_ld] and are added in part order, with the bias, by a second small launch.
  float* kpartial; size_t kpartial_bytes; int ksplit; int m_blocks; int64_t kp_ld;
  // LoRA down-projections inside a forward launch of few tokens (n_prod > 0): the g_* fields, tpart, counters and
  // ready describe them as for launch_lora_down_gemm; the first n_prod workgroups (a multiple of 8) compute ts as
  // lora_down_block does -- token block x rank tile x K-part = p_tbs x p_tiles x p_parts of them, the rest idle --
  // and the workgroups that carry the LoRA columns wait (bounded) until `ready` has counted p_tbs * p_tiles of
  // them; every consumer counts itself in `done` when it leaves, the last one zeroes both words for the next call.
  // The launcher may decline (a shape of ten waves, many tokens) and run the down-projection as a launch of its own.
  int n_prod; int p_tbs; int p_tiles; int p_parts; uint32_t* done; int n_consumers;
  uint32_t* ready;                                                          // LoRA down-projection inside another kernel's launch: workgroups that have written ts count themselves here (else null)
  uint32_t* tpart; uint32_t* counters;                                      // LoRA down-projection over several K-parts: partial sums, arrival counts (zero between calls); or null
  // LoRA down-projection of a group of adapters that read the same x (g_n > 0): grid.y runs over the 32-row
  // tiles of all adapters; member i owns tiles [g_tile0[i], g_tile0[i+1]) and has its own A, ts and scales
  int g_n; int g_tile0[kMaxGroup + 1]; const uint16_t* g_A[kMaxGroup]; const uint16_t* g_ts[kMaxGroup]; int64_t g_ts_ld[kMaxGroup];
  int g_r[kMaxGroup]; float g_lora_scale[kMaxGroup]; const float* g_tensor_scale[kMaxGroup];
};
int launch_gemm(const GemmArgs& a, hipStream_t st);
constexpr size_t kGemmSplitCap = (size_t)24 << 20;
constexpr size_t kFusedDownBytes = (size_t)1 << 20;   // K-part sums of down-projections that ride inside a GEMM launch: at most 64 workgroups of one 32 x 32 tile
size_t gemm_split_bytes(int64_t M, int64_t N_total);   // scratch worth offering launch_gemm as kpartial for this shape (0: it would not split K)
constexpr int kDownMaxSlots = 256;                                           // workgroups of a K-split LoRA down-projection
constexpr size_t kDownExchangeBytes = (size_t)16 << 20;   // the K-parts' partial sums (32-token kernel: kDownMaxSlots workgroups of two 32 x 32 tiles; 64-token kernel: up to eight tiles per wave quartet)
int launch_lora_down_gemm(const GemmArgs& a, hipStream_t st);

// ---- 17..128 tokens: weight-streaming MFMA kernel on tile-packed weights (linear_mid.hip) ----
constexpr size_t kMidPartialCap = (size_t)32 << 20;   // most workspace bytes the K-splits' partial outputs may take
constexpr size_t kMidDownBytes = (size_t)64 * 2 * 16 * 64 * sizeof(float);   // K-parts' sums of the LoRA down-projection: at most 64 workgroups, two 32 x 32 tiles each
struct MidMember {
  const uint8_t* packed; const float* tensor_scale; int64_t N; int n_tiles;
  const uint16_t* ts; int64_t ts_ld; int ext_stages;                        // [M, ts_ld] bf16: hi | mid | lo of lora_scale / S32 * t; stages of 128 columns
  const uint16_t* B; int r;
  const uint16_t* bias;                                                     // [N] bf16 or null
  uint16_t* y; int64_t ldy;
  int block_begin;                                                          // first column block (W row-tiles each) of this member
  int64_t partial_off;                                                      // floats: this member's [S][M][N] partial outputs start here
};
struct MidArgs {
  const uint16_t* x; int64_t ldx; int64_t M; int64_t K; int k_tiles;
  int n_members; MidMember mem[kMaxGroup];                                  // unused entries: block_begin = INT_MAX
  float* partial;                                                           // K-splits' partial outputs when S > 1
  int n_blocks; int m_chunks; int S; int kt_per_split; int MT; int W;
  // LoRA down-projections inside the launch (n_prod > 0): the first n_prod workgroups (a multiple of 8) compute ts
  // as lora_down_block does -- token block x rank tile x K-part = p_tbs x p_tiles x p_parts of them, the rest idle --
  // and the workgroups that carry the LoRA columns wait until `ready` has counted p_tbs * p_tiles of them; every
  // consumer workgroup counts itself in `done` when it leaves, the last one zeroes both words for the next call.
  GemmArgs dn; int n_prod; int p_tbs; int p_tiles; int p_parts; uint32_t* ready; uint32_t* done; int n_consumers;
};
extern int g_mid_max_tokens;
int plan_mid(MidArgs& a, size_t partial_cap_bytes);
int launch_mid(const MidArgs& a, hipStream_t st);

// General fallback (any K % 16 == 0, any alignment of rows the ABI allows).
int launch_generic_lora_down(const uint16_t* x, int64_t ldx, int64_t M, int64_t K, const uint16_t* A,
                             int64_t r, float* t, hipStream_t st);
int launch_generic_linear(const uint16_t* x, int64_t ldx, int64_t M, int64_t K, const uint8_t* codes,
                          const uint8_t* scales, const float* tensor_scale, int64_t N, const float* t,
                          const uint16_t* B, int64_t r, float lora_scale, uint16_t* y, int64_t ldy,
                          hipStream_t st);

}  // namespace qerl
