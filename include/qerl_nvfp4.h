/*
 * qerl_nvfp4.h -- C ABI of the MI355X (gfx950) NVFP4 + LoRA linear library.
 *
 * The hot path of QeRL's rollout phase: a weight-only NVFP4 linear layer with
 * a fused LoRA branch, fed by an RMSNorm whose gain carries the Adaptive
 * Quantization Noise.
 *
 * Conventions (all entry points)
 *   - Plain C.  Every pointer is a DEVICE pointer unless its comment says host.
 *   - The caller owns every buffer; the library allocates nothing and keeps
 *     no reference after the call returns.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     All device work is enqueued on it and is asynchronous; the library never
 *     synchronises.  Results are valid once the stream reaches that point.
 *   - bf16 tensors are row-major with a leading dimension in ELEMENTS.
 *   - Return value: QERL_OK, or a negative code for a misuse detected on the
 *     host before anything was launched (nothing has been written then), or
 *     QERL_ERR_LAUNCH if the HIP runtime refused a launch
 *     (qerl_last_hip_error() returns its hipError_t).
 *   - Weight matrix orientation: W[N, K] = out-features x in-features, K
 *     contiguous; scale blocks of 16 run along K.
 *
 * Canonical NVFP4 tensor (Section 3.3 "NVFP4 Quantization", Eq. 6; element
 * format from the Preliminary section):
 *   codes  [N, K/2]  uint8 : two E2M1 codes per byte, low nibble = even k,
 *                            bit 3 of a code is the sign
 *   scales [N, K/16] uint8 : one FP8 E4M3 byte per 16 weights, sign bit clear
 *   tensor_scale   1 float : the FP32 per-tensor scale (device memory)
 *   W_hat[n,k] = tensor_scale * ( E4M3(scales[n,k/16]) * E2M1(code[n,k]) )
 */
#ifndef QERL_NVFP4_H
#define QERL_NVFP4_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define QERL_API __attribute__((visibility("default")))

#define QERL_OK              0
#define QERL_ERR_NULL       -1  /* a required pointer is NULL                          */
#define QERL_ERR_SHAPE      -2  /* M,N < 0, K % 16 != 0, ld < row length, r < 0, ...   */
#define QERL_ERR_ALIGN      -3  /* pointer or leading dimension not aligned as documented */
#define QERL_ERR_WORKSPACE  -4  /* workspace NULL or smaller than *_workspace_bytes()  */
#define QERL_ERR_LAUNCH     -5  /* HIP runtime error; see qerl_last_hip_error()        */
#define QERL_ERR_TIMEOUT    -6  /* reported by qerl_workspace_status(): a kernel's bounded
                                   wait on another workgroup gave up                   */

/* Host.  Static string for a status code. */
QERL_API const char* qerl_status_string(int status);
/* Host.  hipError_t of the most recent QERL_ERR_LAUNCH on this thread (0 if none). */
QERL_API int qerl_last_hip_error(void);

/* ---------------------------------------------------------------------------
 * nvfp4_quantize -- W[N,K] bf16  ->  canonical NVFP4 (codes, scales, tensor_scale).
 *
 * The paper gives only the dequantisation (Eq. 6); the rule implemented is
 * the round-to-nearest chain, every step in IEEE fp32 in this order:
 *     tensor_scale = amax / 2688                (2688 = 6 * 448; 1 if amax = 0)
 *     scale        = E4M3_rne_sat( (block_amax / 6) / tensor_scale )
 *     code         = E2M1_rne_sat( w / (tensor_scale * scale) ), sign = sign(w)
 * A block whose scale byte is 0 stores magnitude 0.  Non-finite weights are
 * not supported (result unspecified).  Output is bit-exact reproducible.
 *
 *   W            [N, ldw] bf16, ldw >= K, ldw % 8 == 0, 16-byte aligned
 *   codes        [N, K/2]  out, 8-byte aligned
 *   scales       [N, K/16] out
 *   tensor_scale 1 float   out
 *   workspace    scratch of >= nvfp4_quantize_workspace_bytes(N,K) bytes,
 *                4-byte aligned; contents on entry are ignored
 * Errors: NULL pointers; N < 0, K < 0, K % 16 != 0, ldw < K; alignment;
 * workspace too small.  N == 0 or K == 0 writes tensor_scale = 1 only.
 */
QERL_API int nvfp4_quantize(const void* W_bf16, int64_t N, int64_t K, int64_t ldw,
                   uint8_t* codes, uint8_t* scales, float* tensor_scale,
                   void* workspace, size_t workspace_bytes, void* stream);
QERL_API size_t nvfp4_quantize_workspace_bytes(int64_t N, int64_t K);   /* host */

/* ---------------------------------------------------------------------------
 * nvfp4_dequantize -- Eq. 6, element by element in fp32 (test/inspection aid).
 *   W_f32 [N, K] out, fp32 row-major.
 */
QERL_API int nvfp4_dequantize(const uint8_t* codes, const uint8_t* scales, const float* tensor_scale,
                     int64_t N, int64_t K, float* W_f32, void* stream);

/* ---------------------------------------------------------------------------
 * nvfp4_lora_linear --
 *   y[M,N] = tensor_scale * ( x . (scales (.) codes)^T ) + lora_scale * (x . A^T) . B^T
 * (Eq. 6 for the main branch, Eq. 2 for the low-rank branch W + B A; lora_scale
 * is alpha / r from Algorithm 1's "LoRA rank, LoRA alpha" inputs).  Products are
 * exact, sums are fp32, x A^T is kept in fp32, the result is rounded once to
 * bf16 (nearest-even).  The summation order is fixed: results are bit-identical
 * from call to call.
 *
 *   x   [M, ldx] bf16            A [r, K] bf16 (dense, or NULL when r == 0)
 *   y   [M, ldy] bf16 out        B [N, r] bf16 (dense, or NULL when r == 0)
 *   workspace: >= nvfp4_lora_linear_workspace_bytes(M,N,K,r) bytes, 256-byte
 *     aligned, prepared ONCE with qerl_workspace_init() and afterwards used
 *     only by this library.  Calls that share a workspace must be ordered on
 *     one stream.  A call that returned an error leaves it valid.  The control
 *     words sit at fixed offsets, so one workspace sized for the largest call
 *     (every argument at its maximum) serves calls of any smaller shape.
 *     Where the adapters' down-projections run as the first workgroups of the
 *     launch (M <= 128), the other workgroups wait for them: a bounded wait under
 *     the co-residency assumption stated with aqn_rmsnorm_nvfp4_lora_mlp below.  A
 *     wait that gives up writes NaN into y, sets the sticky error word of the
 *     workspace and leaves the hand-over words as they are (the call has already
 *     returned QERL_OK by then): qerl_workspace_status() reports it, and the
 *     workspace must be prepared again with qerl_workspace_init() before reuse.
 *   tensor_scale: device pointer to one fp32, finite and non-zero (the
 *     quantizer never writes 0: an all-zero tensor gets 1).
 *
 * Any M >= 0 is accepted (M == 0 is a no-op).  The tiled MFMA kernels need
 * K % 64 == 0, x, codes and A 16-byte aligned, scales 4-byte aligned and
 * ldx % 8 == 0 (true for any real model); everything else takes a slower
 * general kernel with the same results contract.
 * Errors: NULL pointers (A/B only when r > 0); M,N,K,r < 0, K % 16 != 0,
 * ldx < K, ldy < N, N >= 2^20, r > 4096; bf16 pointers not 2-byte aligned;
 * workspace NULL, not 256-byte aligned or too small.
 */
QERL_API int nvfp4_lora_linear(const void* x_bf16, int64_t M, int64_t K, int64_t ldx,
                      const uint8_t* codes, const uint8_t* scales, const float* tensor_scale,
                      int64_t N,
                      const void* A_bf16, const void* B_bf16, int64_t r, float lora_scale,
                      void* y_bf16, int64_t ldy,
                      void* workspace, size_t workspace_bytes, void* stream);
QERL_API size_t nvfp4_lora_linear_workspace_bytes(int64_t M, int64_t N, int64_t K, int64_t r); /* host */

/* ---------------------------------------------------------------------------
 * Tile-packed weights.  The weights of a rollout policy are frozen (Section
 * 3.3: only the low-rank matrices are updated), so the canonical tensor can be
 * re-laid out once for the kernels: nvfp4_prepack copies the same code and
 * scale bytes, unchanged, into 2304-byte tiles of 32 rows x 128 inputs (rows
 * padded to 32 and K to 128 with zero bytes) in the order the MFMA operands
 * consume them, so that every wave-wide load is 1 KiB of consecutive memory.
 * The size stays 0.5625 bytes per (padded) weight.  Layout of a tile: see
 * csrc/linear_decode.hip.
 *   packed: out, nvfp4_prepack_bytes(N,K) bytes, 16-byte aligned.
 * nvfp4_lora_linear_packed computes exactly what nvfp4_lora_linear does, from
 * `packed` instead of (codes, scales); same arguments otherwise, but x must be
 * 16-byte aligned with ldx % 8 == 0 (QERL_ERR_ALIGN) and K > 0.
 */
QERL_API size_t nvfp4_prepack_bytes(int64_t N, int64_t K);   /* host */
QERL_API int nvfp4_prepack(const uint8_t* codes, const uint8_t* scales, int64_t N, int64_t K,
                           void* packed, void* stream);
QERL_API int nvfp4_lora_linear_packed(const void* x_bf16, int64_t M, int64_t K, int64_t ldx,
                                      const void* packed, const float* tensor_scale, int64_t N,
                                      const void* A_bf16, const void* B_bf16, int64_t r, float lora_scale,
                                      void* y_bf16, int64_t ldy,
                                      void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------
 * nvfp4_lora_linear_packed_noalloc -- nvfp4_lora_linear_packed for callers that
 * cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments
 * without the workspace pair, same results bit for bit.  The scratch is an array
 * of nvfp4_lora_linear_packed_noalloc_max_bytes() (36 MiB) inside the library,
 * one copy per GPU, held until the process ends; the call allocates nothing and
 * frees nothing, and enqueues one small fill kernel (which clears the control
 * words at the front of the array) ahead of the linear's own launches.
 *   Limit: nvfp4_lora_linear_workspace_bytes(M, N, K, r) must not exceed
 *   nvfp4_lora_linear_packed_noalloc_max_bytes(), else QERL_ERR_WORKSPACE and
 *   nothing is enqueued (every single linear of Qwen2.5-7B/14B/32B shape up to
 *   4096 tokens and rank 64 fits).
 *   The sticky error word of a wait that gave up is among the control words the
 *   next call clears: with this entry point only the NaN in y shows it.
 *   All calls on one GPU share that GPU's array: calls that overlap in time on
 *   one GPU (different streams, different threads) race; order them on one
 *   stream.  The array belongs to the device that is current at the call.
 * Errors: as nvfp4_lora_linear_packed; QERL_ERR_LAUNCH also if the array's
 * device address cannot be obtained.
 */
QERL_API size_t nvfp4_lora_linear_packed_noalloc_max_bytes(void);   /* host */
QERL_API int nvfp4_lora_linear_packed_noalloc(const void* x_bf16, int64_t M, int64_t K, int64_t ldx,
                                              const void* packed, const float* tensor_scale, int64_t N,
                                              const void* A_bf16, const void* B_bf16, int64_t r, float lora_scale,
                                              void* y_bf16, int64_t ldy, void* stream);

/* ---------------------------------------------------------------------------
 * nvfp4_lora_linear_packed_group -- up to 4 linears that read the same x (the
 * q/k/v or the gate/up projections of a block, which share one noisy RMSNorm
 * output: Section 3.3) in ONE launch.  Each member is the same function of its
 * inputs as in nvfp4_lora_linear_packed; the split of K over workgroups, and
 * with it the fp32 summation order, may differ between the two calls (each is
 * bit-reproducible from call to call).
 *   members: HOST array of n_members descriptors (read during the call only;
 *            the pointers inside are device pointers).
 *   workspace: as for nvfp4_lora_linear, sized with
 *            nvfp4_lora_linear_workspace_bytes(M, sum of N, K, sum of r).
 * Errors: as nvfp4_lora_linear_packed, plus n_members outside 1..4; a bias with an
 * adapter the fast kernels do not take (rank not a multiple of 8, or above 64 at
 * M <= 16, or A/B not 16-byte aligned): QERL_ERR_SHAPE.
 */
#define QERL_T_PARTS 8
typedef struct {
  const void* packed;          /* nvfp4_prepack output for this member's [N, K] weight */
  const float* tensor_scale;
  int64_t N;
  const void* A_bf16;          /* [r, K] or NULL */
  const void* B_bf16;          /* [N, r] or NULL */
  int64_t r;
  float lora_scale;
  void* y_bf16;                /* [M, ldy] out */
  int64_t ldy;
  const float* t_f32;          /* x A^T of this member computed before the call, as aqn_rmsnorm_lora_down
                                  writes it: QERL_T_PARTS partial sums over slices of K, fp32
                                  [QERL_T_PARTS][M][r], 32-byte aligned (the kernel adds them in slice order);
                                  or NULL: the call computes x A^T itself.  Used at M <= 16 only; larger M
                                  recompute it. */
  const void* bias_bf16;       /* [N] bf16 added to every output row before the one rounding to bf16 (the
                                  q/k/v projections of the Qwen2.5 blocks carry one), or NULL */
} qerl_linear_desc;
QERL_API int nvfp4_lora_linear_packed_group(const void* x_bf16, int64_t M, int64_t K, int64_t ldx,
                                            const qerl_linear_desc* members, int n_members,
                                            void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------
 * Fused decode launches.  Up to 16 tokens each of these is ONE persistent launch
 * (one workgroup per compute unit) in which the weight stream never stops: the
 * RMSNorm with the noisy gain (Eq. 10; Section 3.3 "Noise Merging": q, k, v share
 * one such norm, gate and up another) is applied while the input is staged, the
 * adapters' down-projections x A^T (Eq. 2) run on a few workgroups of the same
 * launch, and -- in the feed-forward call -- SiLU(gate) (.) up is formed in the
 * epilogue of the gate / up tiles, a device-wide hand-over follows, and down_proj
 * streams on behind it.  For more tokens the same operators run as separate
 * launches (same results contract).
 *
 * aqn_rmsnorm_nvfp4_lora_linear_group:
 *   xn = aqn_rmsnorm(x, gain, noise, eps) rounded to bf16 (gain == NULL: xn = x),
 *   members[i].y = nvfp4_lora_linear_packed(xn, member i)           i < n_members <= 4
 * aqn_rmsnorm_nvfp4_lora_mlp:
 *   xn as above; g = gate(xn), u = up(xn), both rounded to bf16;
 *   act = bf16( bf16(SiLU(g)) (.) u )   (as nvfp4_lora_linear_packed_swiglu);
 *   down->y = nvfp4_lora_linear_packed(act, down).    gate->y, up->y are not written.
 *   gate->N == up->N == down's K, a multiple of 8.
 * Arguments as in aqn_rmsnorm and nvfp4_lora_linear_packed_group (descriptors are
 * HOST structs read during the call; t_f32 is ignored); x 16-byte aligned, ldx % 8
 * == 0, gain / noise 16-byte aligned; at M <= 16 every adapter needs r % 8 == 0,
 * r <= 64 and 16-byte aligned A and B (QERL_ERR_SHAPE otherwise).
 *   workspace: >= the matching *_workspace_bytes(), 256-byte aligned, prepared once
 *   with qerl_workspace_init(); a linear workspace of that size serves as well (the
 *   control words share one layout).  Calls sharing it must be ordered on one stream.
 * Co-residency: the workgroups of these launches (and of the other decode
 * kernels' in-launch hand-overs) wait for each other, which requires that all of
 * them are resident at once: one process per GPU, no other kernel holding
 * compute units for the duration of the call.  Every such wait is bounded; if one
 * gives up, the sticky error word of the workspace is set, the outputs of that
 * call are unreliable, and qerl_workspace_status() reports QERL_ERR_TIMEOUT until
 * the workspace is prepared again with qerl_workspace_init().
 */
QERL_API size_t aqn_rmsnorm_nvfp4_lora_linear_group_workspace_bytes(int64_t M, int64_t K, const int64_t* Ns,
                                                                    const int64_t* rs, int n_members);   /* host */
QERL_API int aqn_rmsnorm_nvfp4_lora_linear_group(const void* x_bf16, int64_t M, int64_t K, int64_t ldx,
                                                 const void* gain_bf16, const float* noise_f32, float eps,
                                                 const qerl_linear_desc* members, int n_members,
                                                 void* workspace, size_t workspace_bytes, void* stream);
QERL_API size_t aqn_rmsnorm_nvfp4_lora_mlp_workspace_bytes(int64_t M, int64_t H, int64_t I, int64_t N_down,
                                                           int64_t r_gate, int64_t r_up, int64_t r_down);   /* host */
QERL_API int aqn_rmsnorm_nvfp4_lora_mlp(const void* x_bf16, int64_t M, int64_t H, int64_t ldx,
                                        const void* gain_bf16, const float* noise_f32, float eps,
                                        const qerl_linear_desc* gate, const qerl_linear_desc* up,
                                        const qerl_linear_desc* down,
                                        void* workspace, size_t workspace_bytes, void* stream);

/* qerl_workspace_status: reads the sticky error word of a workspace (synchronises
 * with `stream`): QERL_OK, or QERL_ERR_TIMEOUT if a bounded wait of any kernel that
 * used the workspace gave up since the last qerl_workspace_init().
 * qerl_status_from_error_word (host): the decoding of that word. */
QERL_API int qerl_workspace_status(const void* workspace, void* stream);
QERL_API int qerl_status_from_error_word(uint32_t word);
/* qerl_selftest_wait_gives_up: for tests of the error path.  Enqueues one wave that
 * performs the kernels' bounded wait, cut to `polls` (1..1024) polls, on a hand-over
 * word of `workspace` that nobody raises; it gives up, sets the sticky error word
 * as the kernels do and exits.  Afterwards qerl_workspace_status() reports
 * QERL_ERR_TIMEOUT until qerl_workspace_init().  Nothing hangs, nothing faults. */
QERL_API int qerl_selftest_wait_gives_up(void* workspace, size_t workspace_bytes, uint32_t polls, void* stream);

/* ---------------------------------------------------------------------------
 * nvfp4_lora_linear_packed_swiglu -- the feed-forward block's down projection
 * on its gated input (the paper adapts W_gate, W_up, W_down of the cited
 * Qwen2.5 / LLaMA blocks: Preliminary, "Low-rank Adaptation"):
 *   act = bf16( bf16(SiLU(gate)) (.) up ),  SiLU(g) = g / (1 + e^-g)
 *   y   = act . W_hat^T + lora_scale * (act . A^T) . B^T          (Eq. 6, Eq. 2)
 * i.e. nvfp4_lora_linear_packed applied to the tensor a bf16 model evaluated
 * operator by operator would hand it.  At M <= 16 the product is formed while
 * the kernel stages its input (no intermediate tensor, no extra launch); for
 * more tokens one elementwise pass writes act into the workspace first.
 *   gate [M, ldg], up [M, ldu] bf16 (the outputs of the gate / up projections),
 *   16-byte aligned, ldg % 8 == ldu % 8 == 0; everything else as
 *   nvfp4_lora_linear_packed.
 *   workspace: >= nvfp4_lora_linear_swiglu_workspace_bytes(M, N, K, r), prepared
 *   like a linear workspace (qerl_workspace_init once).
 * Errors: as nvfp4_lora_linear_packed.
 */
QERL_API size_t nvfp4_lora_linear_swiglu_workspace_bytes(int64_t M, int64_t N, int64_t K, int64_t r); /* host */
QERL_API int nvfp4_lora_linear_packed_swiglu(const void* gate_bf16, const void* up_bf16, int64_t M, int64_t K,
                                             int64_t ldg, int64_t ldu, const void* packed,
                                             const float* tensor_scale, int64_t N, const void* A_bf16,
                                             const void* B_bf16, int64_t r, float lora_scale, void* y_bf16,
                                             int64_t ldy, void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------
 * nvfp4_lora_linear_backward -- gradients of y = x W_hat^T + s (x A^T) B^T for an
 * upstream dY (the paper trains A and B only and backpropagates through the
 * frozen quantised weights: Preliminary, "Low-rank Adaptation"; Eq. 2, Eq. 6):
 *   dX [M, lddx] bf16 = dY W_hat + s (dY B) A        (one rounding to bf16)
 *   dA [r, K]    fp32 = s (dY B)^T x
 *   dB [N, r]    fp32 = s dY^T (x A^T)               (s = lora_scale)
 * fp32 accumulation; x A^T and dY B are carried as three bf16 terms (exact to
 * 2^-24 relative) as in the forward pass.
 *   nvfp4_prepack_t: the canonical codes / scales re-ordered once into the
 *     transposed tile order dX needs (tiles of 32 inputs x 128 rows, 2304
 *     bytes; nvfp4_prepack_t_bytes(N, K) bytes, 16-byte aligned).  Same size
 *     per weight as the forward order; the weights are frozen, so both orders
 *     are made once.
 *   x [M, ldx], dY [M, lddy] bf16, 16-byte aligned, ld % 8 == 0; N % 8 == 0;
 *   A [r, K], B [N, r] bf16 contiguous, 16-byte aligned; r % 8 == 0, r <= 64.
 *   r == 0: only dX is written (x, A, B, dA, dB may be NULL).
 *   workspace: >= nvfp4_lora_linear_backward_workspace_bytes(M, N, K, r),
 *   256-byte aligned; needs no initialisation.
 * Errors: as the forward functions.
 */
QERL_API size_t nvfp4_prepack_t_bytes(int64_t N, int64_t K);   /* host */
QERL_API int nvfp4_prepack_t(const uint8_t* codes, const uint8_t* scales, int64_t N, int64_t K,
                             void* packed_t, void* stream);
QERL_API size_t nvfp4_lora_linear_backward_workspace_bytes(int64_t M, int64_t N, int64_t K, int64_t r); /* host */
QERL_API int nvfp4_lora_linear_backward(const void* x_bf16, const void* dy_bf16, int64_t M, int64_t K, int64_t N,
                                        int64_t ldx, int64_t lddy, const void* packed_t,
                                        const float* tensor_scale, const void* A_bf16, const void* B_bf16,
                                        int64_t r, float lora_scale, void* dx_bf16, int64_t lddx,
                                        float* dA_f32, float* dB_f32, void* workspace, size_t workspace_bytes,
                                        void* stream);

/* ---------------------------------------------------------------------------
 * nvfp4_lora_linear_backward_group -- the backward pass of up to 4 linears that
 * read the same x (the q / k / v or the gate / up projections of a block:
 * Section 3.3), each with its own upstream gradient dY_i [M, N_i]:
 *   dX [M, lddx] bf16 = sum_i [ dY_i W_hat_i + s_i (dY_i B_i) A_i ]
 *   dA_i, dB_i as in nvfp4_lora_linear_backward, from dY_i alone.
 * dX is formed by one GEMM whose contraction runs over the members' rows one
 * after the other: fp32 throughout (between members the running sums are
 * rescaled from one tensor scale to the next, one fp32 rounding each), ONE
 * rounding to bf16 -- where separate calls would round every member's dX and
 * their sum.  The down-projections x A_i^T of all adapters share one launch.
 * With one member the call is nvfp4_lora_linear_backward, bit for bit.
 *   members: HOST array of n_members descriptors (read during the call only; the
 *            pointers inside are device pointers), each as the arguments of the
 *            same names of nvfp4_lora_linear_backward.  r_i == 0: that member
 *            contributes dY_i W_hat_i only.
 *   workspace: >= nvfp4_lora_linear_backward_group_workspace_bytes(M, K, members,
 *            n_members) (0 for n_members outside 1..4), 256-byte aligned; needs
 *            no initialisation.
 * Errors: as nvfp4_lora_linear_backward; QERL_ERR_SHAPE for n_members outside 1..4.
 */
typedef struct {
  const void* dy_bf16;         /* [M, lddy] upstream gradient of this member's output */
  int64_t lddy;
  int64_t N;                   /* N % 8 == 0 */
  const void* packed_t;        /* nvfp4_prepack_t output for this member's [N, K] weight */
  const float* tensor_scale;
  const void* A_bf16;          /* [r, K] or NULL */
  const void* B_bf16;          /* [N, r] or NULL */
  int64_t r;                   /* r % 8 == 0, r <= 64 */
  float lora_scale;
  float* dA_f32;               /* [r, K] out (NULL when r == 0) */
  float* dB_f32;               /* [N, r] out (NULL when r == 0) */
} qerl_backward_desc;
QERL_API size_t nvfp4_lora_linear_backward_group_workspace_bytes(int64_t M, int64_t K, const qerl_backward_desc* members,
                                                                 int n_members);   /* host */
QERL_API int nvfp4_lora_linear_backward_group(const void* x_bf16, int64_t M, int64_t K, int64_t ldx,
                                              const qerl_backward_desc* members, int n_members,
                                              void* dx_bf16, int64_t lddx,
                                              void* workspace, size_t workspace_bytes, void* stream);

/* Zero the control words of a linear workspace.  Call once after allocating
 * it (and again if a kernel using it was ever aborted). */
QERL_API int qerl_workspace_init(void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------
 * aqn_rmsnorm -- y = (gain + noise) (.) x / sqrt(mean_k(x^2) + eps)   (Eq. 10)
 * gain + noise is formed in fp32 and not re-rounded; eps is inside the root;
 * one final rounding to bf16.  noise == NULL is stage 0 (sigma = 0): the plain
 * RMSNorm.
 *   x [M, ldx] bf16, gain [H] bf16, noise [H] fp32 or NULL, y [M, ldy] bf16 out
 * Errors: NULL x/gain/y; M < 0, H < 1, ld < H.  No alignment requirement
 * (16-byte aligned rows with H % 8 == 0 take the vector kernel).
 */
QERL_API int aqn_rmsnorm(const void* x_bf16, int64_t M, int64_t H, int64_t ldx,
                const void* gain_bf16, const float* noise_f32, float eps,
                void* y_bf16, int64_t ldy, void* stream);

/* ---------------------------------------------------------------------------
 * aqn_rmsnorm_lora_down -- the noisy RMSNorm of Eq. 10 and, in the same launch,
 * the LoRA down-projections t_i = y A_i^T (Eq. 2) of up to 4 adapters that read
 * its output (q/k/v or gate/up: Section 3.3).  At decode sizes the product x A^T
 * is latency, not work; computing it where x is produced takes it off the
 * critical path of the linear that follows (pass t_i as t_f32 of its member).
 *   x [M, ldx] bf16, M <= 16; gain [H] bf16; noise [H] fp32 or NULL; y [M, ldy] bf16 out
 *   A_bf16: HOST array of n_adapters device pointers, A_i [r_i, H] bf16, 16-byte aligned
 *   r:      HOST array of ranks, each a multiple of 8, 8..64
 *   t_f32:  HOST array of device pointers, t_i [QERL_T_PARTS][M][r_i] fp32 out, 32-byte
 *           aligned: part p is the product over the p-th slice of H; their sum in
 *           part order is t_i
 * y is the function aqn_rmsnorm computes (its mean of squares is summed in another
 * order, so a rare element may differ from aqn_rmsnorm's by one bf16 unit); t_i
 * is the fp32 product of the ROUNDED y that this call writes (what the linear
 * kernels would compute themselves from y) in a fixed summation order.
 * Errors: as aqn_rmsnorm, plus M > 16, H % 16 != 0, H > 8192, n_adapters outside
 * 1..4, ranks not multiples of 8 in 8..64
 * (QERL_ERR_SHAPE); unaligned rows or pointers (QERL_ERR_ALIGN).
 */
QERL_API int aqn_rmsnorm_lora_down(const void* x_bf16, int64_t M, int64_t H, int64_t ldx,
                                   const void* gain_bf16, const float* noise_f32, float eps,
                                   void* y_bf16, int64_t ldy,
                                   const void* const* A_bf16, const int64_t* r, float* const* t_f32,
                                   int n_adapters, void* stream);

/* Host.  Eq. 8: sigma(k) = s0 * (s1/s0)^((k-1)/(K-1)), k = 1..K; k = 0 -> 0
 * (Algorithm 1: stage 0 carries quantisation noise only).  NaN on bad stage. */
QERL_API double aqn_sigma(int stage_k, int num_stages, double sigma_start, double sigma_end);

/* Host.  The four sigma decay curves of the scheduler ablation (Section 4, "Noise
 * Scheduler"), k = 1..K, k = 0 -> 0; u = (k-1)/(K-1).  Only the exponential one has
 * a formula in the paper (Eq. 8, = aqn_sigma); the others are this library's reading:
 *   linear       s0 + (s1 - s0) u
 *   cosine       s1 + (s0 - s1) (1 + cos(pi u)) / 2
 *   logarithmic  s0 + (s1 - s0) ln(1 + (k-1)) / ln(K)
 * NaN on a bad kind or stage. */
#define QERL_SCHEDULE_EXPONENTIAL 0
#define QERL_SCHEDULE_LINEAR 1
#define QERL_SCHEDULE_COSINE 2
#define QERL_SCHEDULE_LOGARITHMIC 3
QERL_API double aqn_sigma_schedule(int kind, int stage_k, int num_stages, double sigma_start, double sigma_end);

/* ---------------------------------------------------------------------------
 * aqn_noise_fill -- the noise vector of Section 3.3, "Adaptive Quantization
 * Noise": noise[i] ~ N(0, sigma^2) independently, i < n, generated on the device
 * (the paper resamples it for each forward pass; one call can fill the vectors of
 * all RMSNorms of a model at once).  The paper fixes the distribution only; the
 * construction is counter-based so that a call is a pure function of
 * (seed, subsequence, n, sigma): Philox4x32 with 10 rounds (Salmon et al., SC'11),
 * group b = i / 4 with counter (b lo, b hi, subsequence lo, subsequence hi) and
 * key (seed lo, seed hi); its outputs r0..r3 give two Box-Muller pairs from
 * 24-bit uniforms u1 = ((r0 >> 8) + 1) 2^-24, u2 = (r1 >> 8) 2^-24:
 * z0 = sqrt(-2 ln u1) cos(2 pi u2), z1 = ... sin(...), likewise (r2, r3);
 * noise[4 b + j] = sigma z_j, all in fp32.  Use a new subsequence per forward
 * pass and a new seed per run.
 *   noise: device, fp32 [n] out (4-byte aligned; 16-byte alignment stores faster)
 * Errors: n < 0, sigma negative or not finite (QERL_ERR_SHAPE); NULL noise with n > 0.
 */
QERL_API int aqn_noise_fill(float* noise_f32, int64_t n, float sigma, uint64_t seed, uint64_t subsequence,
                            void* stream);

/* ---------------------------------------------------------------------------
 * MXFP4 variant (Preliminary, "Model Quantization": FP4 E2M1 elements with one
 * shared FP8 E8M0 scale -- a power of two -- per block of 32; the paper evaluates
 * it next to NVFP4).  Blocks run along K.  The paper states no conversion rule;
 * these functions follow the OCP Microscaling (MX) v1.0 one: per block
 * X = floor(log2(max |v|)) - emax_elem (2 for E2M1, 8 for E4M3) clamped to
 * [-127, 127], scale byte = X + 127, element = round-to-nearest-even of v / 2^X,
 * saturating at the largest element (6, 448); an all-zero block gets byte 0.
 *
 * mxfp4_quantize:  W [N, ldw] bf16 -> codes [N, K/2] (low nibble = even k, bit 3
 *                  of a nibble = sign), scales [N, K/32] E8M0.  K % 32 == 0.
 * mxfp4_dequantize: -> W_hat [N, K] fp32 = 2^(scale - 127) * E2M1(code), exact.
 * mxfp8_quantize:  x [M, ldx] bf16 -> codes [M, K] E4M3 bytes (bit 7 = sign),
 *                  scales [M, K/32] E8M0: the activation format of the native path.
 * mxfp4_prepack:   codes/scales -> tiles of 32 rows x 256 inputs (4352 bytes) in the
 *                  operand order of the scaled matrix instruction; packed must be
 *                  16-byte aligned, mxfp4_prepack_bytes(N, K) bytes.
 * mxfp4_linear_native: y [M, N] bf16 = MXFP8(x) . MXFP4(W)^T, both operands
 *   going through CDNA4's block-scaled matrix instruction as stored (no
 *   conversion arithmetic).  NOT the paper's setting: there activations stay
 *   bf16 (weight-only).  x is quantised to MXFP8 (the function mxfp8_quantize
 *   computes) inside the kernel for M <= 32 (a weight-streaming kernel) and by a
 *   launch of its own into the workspace for more tokens (a GEMM, 128 x 256
 *   tiles); the result is the exact product of the two quantised operands summed
 *   in fp32, rounded once to bf16; it differs from the weight-only result by the
 *   activation rounding (up to 2^-4 relative per element).  No LoRA branch and
 *   no bias in this entry point.
 *   x 16-byte aligned with ldx % 8 == 0.
 *   workspace: >= mxfp4_linear_native_workspace_bytes(M, N, K), 256-byte aligned;
 *   needs no initialisation.
 * mxfp4_lora_linear_native: the same base product plus the paper's LoRA branch
 *   (Eq. 2) and an optional bias,
 *     y = MXFP8(x) . MXFP4(W)^T + lora_scale * (x A^T) B^T + bias,
 *   summed in fp32 and rounded once to bf16.  The adapter reads x itself (bf16),
 *   not its MXFP8 rounding: only the frozen base weights' product goes through
 *   the quantised path.  A [r, K], B [N, r] bf16 row-major, 16-byte aligned,
 *   r % 8 == 0 and r <= 128 (r == 0: A and B are ignored); bias [N] bf16 or
 *   NULL.  lora_scale * x A^T is carried between its two launches as three bf16
 *   terms (2^-24 relative); B and bias enter exactly.
 *   workspace: >= mxfp4_lora_linear_native_workspace_bytes(M, N, K, r) (0 for a
 *   rank the function rejects), 256-byte aligned, prepared ONCE with
 *   qerl_workspace_init() and afterwards used only by this library (arrival
 *   counters of the down-projection's K-parts sit at its front and are left at
 *   zero by every call); calls that share it must be ordered on one stream.
 * Errors: as the NVFP4 functions (NULL, shape incl. K % 32, alignment,
 * workspace).
 */
QERL_API int mxfp4_quantize(const void* W_bf16, int64_t N, int64_t K, int64_t ldw,
                            uint8_t* codes, uint8_t* scales_e8m0, void* stream);
QERL_API int mxfp4_dequantize(const uint8_t* codes, const uint8_t* scales_e8m0, int64_t N, int64_t K,
                              float* W_f32, void* stream);
QERL_API int mxfp8_quantize(const void* x_bf16, int64_t M, int64_t K, int64_t ldx,
                            uint8_t* codes_e4m3, uint8_t* scales_e8m0, void* stream);
QERL_API size_t mxfp4_prepack_bytes(int64_t N, int64_t K);   /* host */
QERL_API int mxfp4_prepack(const uint8_t* codes, const uint8_t* scales_e8m0, int64_t N, int64_t K,
                           void* packed, void* stream);
QERL_API size_t mxfp4_linear_native_workspace_bytes(int64_t M, int64_t N, int64_t K);   /* host */
QERL_API int mxfp4_linear_native(const void* x_bf16, int64_t M, int64_t K, int64_t ldx,
                                 const void* packed, int64_t N, void* y_bf16, int64_t ldy,
                                 void* workspace, size_t workspace_bytes, void* stream);
QERL_API size_t mxfp4_lora_linear_native_workspace_bytes(int64_t M, int64_t N, int64_t K, int64_t r);   /* host */
QERL_API int mxfp4_lora_linear_native(const void* x_bf16, int64_t M, int64_t K, int64_t ldx,
                                      const void* packed, int64_t N,
                                      const void* A_bf16, const void* B_bf16, int64_t r, float lora_scale,
                                      const void* bias_bf16, void* y_bf16, int64_t ldy,
                                      void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------
 * Measurement aids: what a kernel on this GPU can reach of the two rooflines the
 * linear is measured against (reported by the benchmark beside the published
 * peaks; no part of the method).
 * qerl_peak_stream_read: `workgroups` persistent workgroups of eight waves read
 *   `bytes` (a multiple of 16 KiB, >= 1 MiB, 16-byte aligned device memory) once
 *   with 16-byte loads, each wave keeping kib_in_flight_per_wave (4, 8 or 16) KiB
 *   requested; bytes / duration is the achievable HBM read rate when the buffer
 *   is far larger than the caches.  sink4: 4 bytes of device memory (practically
 *   never written).
 * qerl_peak_mfma_bf16: `workgroups` workgroups of four waves each issue
 *   8 * iters v_mfma_f32_32x32x16_bf16 on eight independent accumulators;
 *   flops = workgroups * 4 * iters * 8 * 32768.  operands_2kib: 2 KiB of bf16
 *   values (two operand fragments of 16 bytes per lane).
 * Errors: NULL / misaligned pointers, sizes outside the ranges above.
 */
QERL_API int qerl_peak_stream_read(const void* src, size_t bytes, int workgroups, int kib_in_flight_per_wave,
                                   void* sink4, void* stream);
QERL_API int qerl_peak_mfma_bf16(const void* operands_2kib, int workgroups, int iters, void* sink4, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* QERL_NVFP4_H */
