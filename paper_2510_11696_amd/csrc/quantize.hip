// nvfp4_quantize / nvfp4_dequantize kernels for gfx950.
//
// Format: Section 3.3 "NVFP4 Quantization" (E2M1 codes, one E4M3 scale per 16
// weights, one FP32 tensor scale) and Eq. 6 for the inverse map.  The forward
// rule is the fp32 round-to-nearest chain stated in the header.  This file is
// compiled with -ffp-contract=off: every fp32 operation below is a single,
// correctly rounded IEEE operation, which is what makes the output bytes
// reproducible.
//
// Both kernels stream: 2 B read + 0.5625 B written per weight (x2 reads, the
// tensor maximum needs its own pass).
#include "common.hpp"

namespace qerl {

constexpr int kAmaxThreads = 256;
constexpr int kAmaxMaxBlocks = 2048;

// Pass 1: maximum |w| as the bf16 bit pattern with the sign cleared (for
// finite values the integer order of those patterns is the order of the
// magnitudes).  One partial per workgroup, no atomics.
__global__ __launch_bounds__(kAmaxThreads) void amax_partial_kernel(
    const uint16_t* __restrict__ W, int64_t N, int64_t K, int64_t ldw, uint32_t* __restrict__ partial) {
  const int64_t chunks_per_row = K / 8;
  const int64_t total = N * chunks_per_row;
  uint32_t m = 0;
  for (int64_t i = (int64_t)blockIdx.x * kAmaxThreads + threadIdx.x; i < total;
       i += (int64_t)gridDim.x * kAmaxThreads) {
    const int64_t row = i / chunks_per_row, c = i - row * chunks_per_row;
    const u32x4 v = *reinterpret_cast<const u32x4*>(W + row * ldw + c * 8);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint32_t lo = v[j] & 0x7fffu, hi = (v[j] >> 16) & 0x7fffu;
      m = lo > m ? lo : m;
      m = hi > m ? hi : m;
    }
  }
  m = wave_max_u32(m);
  __shared__ uint32_t s[kAmaxThreads / kWave];
  if ((threadIdx.x & 63) == 0) s[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < kAmaxThreads / kWave; ++w) m = s[w] > m ? s[w] : m;
    partial[blockIdx.x] = m;
  }
}


// Pass 2: one thread per 16-weight block.
__global__ __launch_bounds__(256) void encode_kernel(
    const uint16_t* __restrict__ W, int64_t N, int64_t K, int64_t ldw,
    const uint32_t* __restrict__ partial, int n_partial,
    uint8_t* __restrict__ codes, uint8_t* __restrict__ scales, float* __restrict__ tensor_scale) {
  __shared__ uint32_t s_amax;
  {
    uint32_t m = 0;
    for (int i = threadIdx.x; i < n_partial; i += 256) { uint32_t p = partial[i]; m = p > m ? p : m; }
    m = wave_max_u32(m);
    __shared__ uint32_t s[4];
    if ((threadIdx.x & 63) == 0) s[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
      for (int w = 1; w < 4; ++w) m = s[w] > m ? s[w] : m;
      s_amax = m;
    }
    __syncthreads();
  }
  const float amax = bf16_bits_to_f32(s_amax);
  const float S32 = (amax == 0.0f) ? 1.0f : amax / 2688.0f;
  if (blockIdx.x == 0 && threadIdx.x == 0) *tensor_scale = S32;

  const int64_t blocks_per_row = K / kBlock;
  const int64_t total = N * blocks_per_row;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int64_t row = i / blocks_per_row, j = i - row * blocks_per_row;
    const u32x4* src = reinterpret_cast<const u32x4*>(W + row * ldw + j * kBlock);
    const u32x4 v0 = src[0], v1 = src[1];
    uint32_t w[8] = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
    uint32_t bm = 0;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const uint32_t lo = w[t] & 0x7fffu, hi = (w[t] >> 16) & 0x7fffu;
      bm = lo > bm ? lo : bm;
      bm = hi > bm ? hi : bm;
    }
    const float bamax = bf16_bits_to_f32(bm);
    const float v = (bamax / 6.0f) / S32;
    const uint32_t s8 = e4m3_encode_rne_sat(v);
    const float d = S32 * e4m3_to_f32(s8);
    uint32_t packed[2] = {0u, 0u};
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      uint32_t byte = 0;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const uint32_t bits = (w[t] >> (16 * h)) & 0xffffu;
        const float a = bf16_bits_to_f32(bits & 0x7fffu);
        const uint32_t mag = (d == 0.0f) ? 0u : e2m1_encode_rne_sat(a / d);
        byte |= (mag | ((bits >> 15) << 3)) << (4 * h);
      }
      packed[t >> 2] |= byte << (8 * (t & 3));
    }
    *reinterpret_cast<u32x2*>(codes + row * (K / 2) + j * 8) = u32x2{packed[0], packed[1]};
    scales[row * blocks_per_row + j] = (uint8_t)s8;
  }
}

__global__ void write_one_kernel(float* p) { *p = 1.0f; }

// Eq. 6, one thread per byte pair-of-codes group of 8 weights.
__global__ __launch_bounds__(256) void dequantize_kernel(
    const uint8_t* __restrict__ codes, const uint8_t* __restrict__ scales,
    const float* __restrict__ tensor_scale, int64_t N, int64_t K, float* __restrict__ out) {
  const float S32 = *tensor_scale;
  const int64_t total = N * K / 8;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const uint32_t c = *reinterpret_cast<const uint32_t*>(codes + i * 4);
    const float s = e4m3_to_f32(scales[i / 2]);
    float o[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) o[t] = S32 * (s * e2m1_to_f32((c >> (4 * t)) & 15u));
    f32x4* dst = reinterpret_cast<f32x4*>(out + i * 8);
    dst[0] = f32x4{o[0], o[1], o[2], o[3]};
    dst[1] = f32x4{o[4], o[5], o[6], o[7]};
  }
}

}  // namespace qerl

using namespace qerl;

extern "C" size_t nvfp4_quantize_workspace_bytes(int64_t, int64_t) {
  return (size_t)kAmaxMaxBlocks * sizeof(uint32_t);
}

extern "C" int nvfp4_quantize(const void* W, int64_t N, int64_t K, int64_t ldw, uint8_t* codes,
                              uint8_t* scales, float* tensor_scale, void* workspace,
                              size_t workspace_bytes, void* stream) {
  if (!tensor_scale) return QERL_ERR_NULL;
  if (N < 0 || K < 0 || K % kBlock != 0 || ldw < K) return QERL_ERR_SHAPE;
  hipStream_t st = (hipStream_t)stream;
  if (N == 0 || K == 0) {
    write_one_kernel<<<1, 1, 0, st>>>(tensor_scale);
    return launch_status();
  }
  if (!W || !codes || !scales) return QERL_ERR_NULL;
  if (!aligned(W, 16) || ldw % 8 != 0 || !aligned(codes, 8) || !aligned(tensor_scale, 4))
    return QERL_ERR_ALIGN;
  if (!workspace || !aligned(workspace, 4) || workspace_bytes < nvfp4_quantize_workspace_bytes(N, K))
    return QERL_ERR_WORKSPACE;
  const int64_t chunks = N * (K / 8);
  int nb = (int)(ceil_div(chunks, kAmaxThreads * 4) < kAmaxMaxBlocks ? ceil_div(chunks, kAmaxThreads * 4)
                                                                    : kAmaxMaxBlocks);
  if (nb < 1) nb = 1;
  uint32_t* partial = (uint32_t*)workspace;
  amax_partial_kernel<<<nb, kAmaxThreads, 0, st>>>((const uint16_t*)W, N, K, ldw, partial);
  int rc = launch_status();
  if (rc != QERL_OK) return rc;
  const int64_t blocks = N * (K / kBlock);
  int64_t eb = ceil_div(blocks, 256);
  if (eb > 65536) eb = 65536;
  encode_kernel<<<(int)eb, 256, 0, st>>>((const uint16_t*)W, N, K, ldw, partial, nb, codes, scales,
                                         tensor_scale);
  return launch_status();
}

extern "C" int nvfp4_dequantize(const uint8_t* codes, const uint8_t* scales, const float* tensor_scale,
                                int64_t N, int64_t K, float* W_f32, void* stream) {
  if (N < 0 || K < 0 || K % kBlock != 0) return QERL_ERR_SHAPE;
  if (N == 0 || K == 0) return QERL_OK;
  if (!codes || !scales || !tensor_scale || !W_f32) return QERL_ERR_NULL;
  if (!aligned(codes, 4) || !aligned(W_f32, 16)) return QERL_ERR_ALIGN;
  int64_t nb = ceil_div(N * K / 8, 256);
  if (nb > 65536) nb = 65536;
  dequantize_kernel<<<(int)nb, 256, 0, (hipStream_t)stream>>>(codes, scales, tensor_scale, N, K, W_f32);
  return launch_status();
}
