// Achievable-ceiling microbenchmarks for the two rooflines the linear kernels are measured against:
//   qerl_peak_stream_read  -- nothing but coalesced 16-byte loads over a large buffer (the HBM roof as a kernel
//                             can reach it), shaped like the decode kernel's weight stream: persistent
//                             workgroups, every wave keeping a fixed number of 1 KiB requests in flight;
//   qerl_peak_mfma_bf16    -- nothing but v_mfma_f32_32x32x16_bf16 on eight independent accumulators per wave
//                             (the matrix pipe as the prefill kernel's inner loop could drive it), operands
//                             taken from memory once so that they hold real bit patterns.
// Both write a value that depends on everything they computed, so nothing is optimised away.
#include "common.hpp"

namespace qerl {

template <int U>
__global__ __launch_bounds__(512) void peak_read_kernel(const u32x4* __restrict__ src, size_t n16, uint32_t* __restrict__ sink) {
  // the buffer is cut into chunks of U KiB per wave-iteration; wave (global index w of W) takes chunks w, w + W, ...
  const int lane = threadIdx.x & 63;
  const size_t wave = (size_t)blockIdx.x * 8 + (threadIdx.x >> 6), waves = (size_t)gridDim.x * 8;
  const size_t chunk = (size_t)U * 64;                      // 16-byte words per chunk
  const size_t n_chunks = n16 / chunk;
  u32x4 acc = {0u, 0u, 0u, 0u};
  for (size_t c = wave; c < n_chunks; c += waves) {
    const u32x4* p = src + c * chunk + lane;
    u32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load(p + u * 64);
#pragma unroll
    for (int u = 0; u < U; ++u) acc ^= v[u];
  }
  const uint32_t r = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
  if (r == 0x9e3779b9u) sink[0] = r;                        // practically never true; keeps the loads alive
}

#ifdef QERL_TUNING_HOOKS
// Experiment: the weight stream's access pattern on its own.  Every wave reads private contiguous regions of
// `region_tiles` packed tiles (2304 bytes: two 1 KiB loads and one 256-byte load), `D` tiles in flight, regions
// dealt round-robin over all waves; `wave_stride_tiles` > 0 instead interleaves the waves of a workgroup tile by tile.
__device__ unsigned long long g_tiles_t0[1024], g_tiles_t1[1024];
template <int D>
__global__ __launch_bounds__(512) void peak_tiles_kernel(const uint8_t* __restrict__ src, int n_regions, int region_tiles, int interleave,
                                                         uint32_t* __restrict__ sink) {
  extern __shared__ __attribute__((aligned(256))) unsigned char ballast[];
  if (threadIdx.x == 0) { g_tiles_t0[blockIdx.x] = wall_clock64(); if (n_regions < 0) ballast[0] = 1; }
  const int lane = threadIdx.x & 63, n32 = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int gw = (int)blockIdx.x * 8 + wave, waves = (int)gridDim.x * 8;
  u32x4 acc = {0u, 0u, 0u, 0u};
  for (int r = gw; r < n_regions; r += waves) {
    // interleave: the 8 waves of a workgroup share 8 consecutive regions and walk them tile-interleaved
    const uint8_t* base; int64_t step;
    if (interleave) { base = src + ((int64_t)(r - wave) * region_tiles + wave) * 2304; step = 8 * 2304; }
    else { base = src + (int64_t)r * region_tiles * 2304; step = 2304; }
    u32x4 c0[D], c1[D]; u32x2 sc[D];
#pragma unroll
    for (int d = 0; d < D; ++d) {
      const uint8_t* p = base + (int64_t)d * step;
      c0[d] = *reinterpret_cast<const u32x4*>(p + lane * 16); c1[d] = *reinterpret_cast<const u32x4*>(p + 1024 + lane * 16);
      sc[d] = *reinterpret_cast<const u32x2*>(p + 2048 + n32 * 8);
    }
    for (int i0 = 0; i0 < region_tiles; i0 += D) {
#pragma unroll
      for (int d = 0; d < D; ++d) {
        acc ^= c0[d]; acc ^= c1[d]; acc[0] ^= sc[d][0] ^ sc[d][1];
        asm volatile("" : "+v"(acc));
        __builtin_amdgcn_sched_barrier(0);
        const int nx = i0 + D + d < region_tiles ? i0 + D + d : region_tiles - 1;
        const uint8_t* p = base + (int64_t)nx * step;
        c0[d] = *reinterpret_cast<const u32x4*>(p + lane * 16); c1[d] = *reinterpret_cast<const u32x4*>(p + 1024 + lane * 16);
        sc[d] = *reinterpret_cast<const u32x2*>(p + 2048 + n32 * 8);
      }
    }
  }
  const uint32_t r = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
  if (r == 0x9e3779b9u) sink[0] = r;
  __syncthreads();
  if (threadIdx.x == 0) g_tiles_t1[blockIdx.x] = wall_clock64();
}
#endif

__global__ __launch_bounds__(256) void peak_mfma_kernel(const u32x4* __restrict__ operands, int iters, float* __restrict__ sink) {
  const int lane = threadIdx.x & 63;
  const bf16x8 a = __builtin_bit_cast(bf16x8, operands[lane]);
  const bf16x8 b = __builtin_bit_cast(bf16x8, operands[64 + lane]);
  f32x16 acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) s += acc[i][j];
  if (s == 12345.678f) sink[0] = s;
}

}  // namespace qerl

using namespace qerl;

extern "C" int qerl_peak_stream_read(const void* src, size_t bytes, int workgroups, int kib_in_flight_per_wave, void* sink4,
                                     void* stream) {
  if (!src || !sink4) return QERL_ERR_NULL;
  if (!aligned(src, 16) || !aligned(sink4, 4)) return QERL_ERR_ALIGN;
  if (workgroups < 1 || workgroups > 65535 || bytes < ((size_t)1 << 20) || bytes % ((size_t)16 << 10) != 0) return QERL_ERR_SHAPE;
  const size_t n16 = bytes / 16;
  const dim3 g((unsigned)workgroups), b(512);
  switch (kib_in_flight_per_wave) {
    case 4: peak_read_kernel<4><<<g, b, 0, (hipStream_t)stream>>>((const u32x4*)src, n16, (uint32_t*)sink4); break;
    case 8: peak_read_kernel<8><<<g, b, 0, (hipStream_t)stream>>>((const u32x4*)src, n16, (uint32_t*)sink4); break;
    case 16: peak_read_kernel<16><<<g, b, 0, (hipStream_t)stream>>>((const u32x4*)src, n16, (uint32_t*)sink4); break;
    default: return QERL_ERR_SHAPE;
  }
  return launch_status();
}

extern "C" int qerl_peak_mfma_bf16(const void* operands_2kib, int workgroups, int iters, void* sink4, void* stream) {
  if (!operands_2kib || !sink4) return QERL_ERR_NULL;
  if (!aligned(operands_2kib, 16) || !aligned(sink4, 4)) return QERL_ERR_ALIGN;
  if (workgroups < 1 || workgroups > 65535 || iters < 1) return QERL_ERR_SHAPE;
  peak_mfma_kernel<<<dim3((unsigned)workgroups), dim3(256), 0, (hipStream_t)stream>>>((const u32x4*)operands_2kib, iters,
                                                                                       (float*)sink4);
  return launch_status();
}

#ifdef QERL_TUNING_HOOKS
extern "C" QERL_API double qerl_debug_peak_tiles_us(int workgroups) {   // span of the last launch, first start to last end
  static unsigned long long t0[1024], t1[1024];
  if (hipMemcpyFromSymbol(t0, HIP_SYMBOL(qerl::g_tiles_t0), sizeof(t0)) != hipSuccess || hipMemcpyFromSymbol(t1, HIP_SYMBOL(qerl::g_tiles_t1), sizeof(t1)) != hipSuccess) return -1;
  unsigned long long a = ~0ull, b = 0;
  for (int i = 0; i < workgroups && i < 1024; ++i) { a = t0[i] < a ? t0[i] : a; b = t1[i] > b ? t1[i] : b; }
  return (double)(b - a) / 100.0;
}
static int g_tiles_lds = 0;
extern "C" QERL_API void qerl_debug_peak_tiles_lds(int bytes) { g_tiles_lds = bytes; }
extern "C" QERL_API int qerl_debug_peak_tiles(const void* src, int n_regions, int region_tiles, int workgroups, int depth, int interleave,
                                              void* sink4, void* stream) {
  const dim3 g((unsigned)workgroups), b(512);
  if (g_tiles_lds > 0) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&peak_tiles_kernel<4>), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 256);
    peak_tiles_kernel<4><<<g, b, g_tiles_lds, (hipStream_t)stream>>>((const uint8_t*)src, n_regions, region_tiles, interleave, (uint32_t*)sink4);
    return launch_status();
  }
  if (depth == 2) peak_tiles_kernel<2><<<g, b, 0, (hipStream_t)stream>>>((const uint8_t*)src, n_regions, region_tiles, interleave, (uint32_t*)sink4);
  else if (depth == 4) peak_tiles_kernel<4><<<g, b, 0, (hipStream_t)stream>>>((const uint8_t*)src, n_regions, region_tiles, interleave, (uint32_t*)sink4);
  else peak_tiles_kernel<8><<<g, b, 0, (hipStream_t)stream>>>((const uint8_t*)src, n_regions, region_tiles, interleave, (uint32_t*)sink4);
  return launch_status();
}
#endif
