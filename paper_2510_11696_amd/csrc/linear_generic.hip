// General NVFP4 + LoRA linear kernels: any K that is a multiple of 16, any M.
// Plain fp32 VALU arithmetic, one workgroup per output row and group of four
// tokens.  Used for the shapes the tiled kernels do not cover; correctness
// first, no claim on speed.  Same definition as the tiled path (Eq. 6, Eq. 2).
#include "linear.hpp"

namespace qerl {

constexpr int kGenThreads = 256;
constexpr int kGenTokens = 4;

__device__ __forceinline__ void block_sum4(float (&v)[kGenTokens], float (*smem)[kGenTokens]) {
#pragma unroll
  for (int m = 0; m < kGenTokens; ++m) v[m] = wave_sum(v[m]);
  if ((threadIdx.x & 63) == 0)
#pragma unroll
    for (int m = 0; m < kGenTokens; ++m) smem[threadIdx.x >> 6][m] = v[m];
  __syncthreads();
#pragma unroll
  for (int m = 0; m < kGenTokens; ++m) {
    float t = 0.f;
    for (int w = 0; w < kGenThreads / kWave; ++w) t += smem[w][m];
    v[m] = t;
  }
  __syncthreads();
}

// t[m, j] = sum_k x[m,k] * A[j,k]; grid = (r, ceil(M/4))
__global__ __launch_bounds__(kGenThreads) void generic_lora_down_kernel(
    const uint16_t* __restrict__ x, int64_t ldx, int64_t M, int64_t K, const uint16_t* __restrict__ A,
    int64_t r, float* __restrict__ t) {
  __shared__ float smem[kGenThreads / kWave][kGenTokens];
  const int64_t j = blockIdx.x, m0 = (int64_t)blockIdx.y * kGenTokens;
  float acc[kGenTokens] = {0.f, 0.f, 0.f, 0.f};
  for (int64_t k = threadIdx.x; k < K; k += kGenThreads) {
    const float a = bf16_bits_to_f32(A[j * K + k]);
#pragma unroll
    for (int m = 0; m < kGenTokens; ++m)
      if (m0 + m < M) acc[m] += bf16_bits_to_f32(x[(m0 + m) * ldx + k]) * a;
  }
  block_sum4(acc, smem);
  if (threadIdx.x < kGenTokens && m0 + threadIdx.x < M) t[(m0 + threadIdx.x) * r + j] = acc[threadIdx.x];
}

// grid = (N, ceil(M/4)); a thread walks 16-weight blocks of row n.
__global__ __launch_bounds__(kGenThreads) void generic_linear_kernel(
    const uint16_t* __restrict__ x, int64_t ldx, int64_t M, int64_t K, const uint8_t* __restrict__ codes,
    const uint8_t* __restrict__ scales, const float* __restrict__ tensor_scale, int64_t N,
    const float* __restrict__ t, const uint16_t* __restrict__ B, int64_t r, float lora_scale,
    uint16_t* __restrict__ y, int64_t ldy) {
  __shared__ float smem[kGenThreads / kWave][kGenTokens];
  const int64_t n = blockIdx.x, m0 = (int64_t)blockIdx.y * kGenTokens;
  float acc[kGenTokens] = {0.f, 0.f, 0.f, 0.f};
  for (int64_t b = threadIdx.x; b < K / kBlock; b += kGenThreads) {
    const float s = e4m3_to_f32(scales[n * (K / kBlock) + b]);
    const uint8_t* cp = codes + n * (K / 2) + b * 8;
#pragma unroll
    for (int i = 0; i < kBlock; ++i) {
      const uint32_t byte = cp[i >> 1];
      const float w = s * e2m1_to_f32((i & 1) ? (byte >> 4) : (byte & 15u));
#pragma unroll
      for (int m = 0; m < kGenTokens; ++m)
        if (m0 + m < M) acc[m] += bf16_bits_to_f32(x[(m0 + m) * ldx + b * kBlock + i]) * w;
    }
  }
  block_sum4(acc, smem);
  if (threadIdx.x < kGenTokens && m0 + threadIdx.x < M) {
    const int64_t m = m0 + threadIdx.x;
    float o = acc[threadIdx.x] * *tensor_scale;
    if (r > 0) {
      float lo = 0.f;
      for (int64_t j = 0; j < r; ++j) lo += t[m * r + j] * bf16_bits_to_f32(B[n * r + j]);
      o += lora_scale * lo;
    }
    y[m * ldy + n] = (uint16_t)f32_to_bf16_bits(o);
  }
}

int launch_generic_lora_down(const uint16_t* x, int64_t ldx, int64_t M, int64_t K, const uint16_t* A,
                             int64_t r, float* t, hipStream_t st) {
  for (int64_t m0 = 0; m0 < M; m0 += 65535 * kGenTokens) {
    const int64_t mc = (M - m0 < 65535 * kGenTokens) ? M - m0 : 65535 * kGenTokens;
    generic_lora_down_kernel<<<dim3((unsigned)r, (unsigned)ceil_div(mc, kGenTokens)), kGenThreads, 0, st>>>(
        x + m0 * ldx, ldx, mc, K, A, r, t + m0 * r);
  }
  return launch_status();
}

int launch_generic_linear(const uint16_t* x, int64_t ldx, int64_t M, int64_t K, const uint8_t* codes,
                          const uint8_t* scales, const float* tensor_scale, int64_t N, const float* t,
                          const uint16_t* B, int64_t r, float lora_scale, uint16_t* y, int64_t ldy,
                          hipStream_t st) {
  for (int64_t m0 = 0; m0 < M; m0 += 65535 * kGenTokens) {
    const int64_t mc = (M - m0 < 65535 * kGenTokens) ? M - m0 : 65535 * kGenTokens;
    generic_linear_kernel<<<dim3((unsigned)N, (unsigned)ceil_div(mc, kGenTokens)), kGenThreads, 0, st>>>(
        x + m0 * ldx, ldx, mc, K, codes, scales, tensor_scale, N, t ? t + m0 * r : nullptr, B, r,
        lora_scale, y + m0 * ldy, ldy);
  }
  return launch_status();
}

}  // namespace qerl
