// Adaptive Quantization Noise on the device: the noise vector of Section 3.3
//   Z ~ N(0, sigma^2 I), drawn anew per forward pass (Section 3.3, "Adaptive Quantization Noise"),
// and the sigma decay curves of the scheduler ablation (Eq. 8 for the exponential one).
//
// aqn_noise_fill writes Z for any number of RMSNorm gains in one launch (a model keeps the vectors
// of all its layers in one buffer), so a forward pass costs one small kernel and no host upload.
// The generator is counter-based (Philox4x32 with 10 rounds; Salmon et al., SC'11): element group
// b of a call depends only on (seed, subsequence, b), not on the launch shape, so results are
// reproducible and any part of a vector can be regenerated on its own.
//   counter = (b mod 2^32, b >> 32, subsequence mod 2^32, subsequence >> 32), key = (seed mod 2^32, seed >> 32)
//   outputs r0..r3 -> two Box-Muller pairs from 24-bit uniforms (exact in fp32):
//     u1 = ((r0 >> 8) + 1) 2^-24 in (0, 1],  u2 = (r1 >> 8) 2^-24 in [0, 1)
//     z0 = sqrt(-2 ln u1) cos(2 pi u2),  z1 = sqrt(-2 ln u1) sin(2 pi u2);  (r2, r3) -> (z2, z3)
//   Z[4 b + j] = sigma z_j
// fp32 throughout; sin and cos take the argument in half-turns (exact range reduction).
#include <math.h>
#include "common.hpp"

namespace qerl {

struct Philox4 { uint32_t v[4]; };

__device__ __forceinline__ Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1) {
  constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
  for (int rnd = 0; rnd < 10; ++rnd) {
    if (rnd) { k0 += W0; k1 += W1; }
    const uint32_t hi0 = __umulhi(M0, c0), lo0 = M0 * c0;
    const uint32_t hi1 = __umulhi(M1, c2), lo1 = M1 * c2;
    const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
    c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
  }
  return Philox4{{c0, c1, c2, c3}};
}

__device__ __forceinline__ void box_muller(uint32_t ra, uint32_t rb, float& z0, float& z1) {
  const float u1 = (float)((ra >> 8) + 1u) * 0x1p-24f;
  const float u2 = (float)(rb >> 8) * 0x1p-24f;
  const float radius = sqrtf(-2.0f * logf(u1));
  float s, c;
  sincospif(2.0f * u2, &s, &c);
  z0 = radius * c;
  z1 = radius * s;
}

__global__ __launch_bounds__(256) void aqn_noise_kernel(float* z, int64_t n, float sigma, uint32_t k0, uint32_t k1,
                                                        uint32_t s0, uint32_t s1) {
  const int64_t groups = (n + 3) / 4;
  for (int64_t b = (int64_t)blockIdx.x * 256 + threadIdx.x; b < groups; b += (int64_t)gridDim.x * 256) {
    const Philox4 r = philox4x32_10((uint32_t)b, (uint32_t)((uint64_t)b >> 32), s0, s1, k0, k1);
    float v[4];
    box_muller(r.v[0], r.v[1], v[0], v[1]);
    box_muller(r.v[2], r.v[3], v[2], v[3]);
    const int64_t i0 = 4 * b;
    if (i0 + 4 <= n && (reinterpret_cast<uintptr_t>(z) & 15) == 0) {
      *reinterpret_cast<f32x4*>(z + i0) = f32x4{sigma * v[0], sigma * v[1], sigma * v[2], sigma * v[3]};
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (i0 + j < n) z[i0 + j] = sigma * v[j];
    }
  }
}

}  // namespace qerl

using namespace qerl;

extern "C" int aqn_noise_fill(float* noise, int64_t n, float sigma, uint64_t seed, uint64_t subsequence, void* stream) {
  if (n < 0) return QERL_ERR_SHAPE;
  if (n == 0) return QERL_OK;
  if (!noise) return QERL_ERR_NULL;
  if (!aligned(noise, 4)) return QERL_ERR_ALIGN;
  if (!(sigma >= 0.0f) || !isfinite(sigma)) return QERL_ERR_SHAPE;
  const int64_t groups = (n + 3) / 4;
  int64_t blocks = (groups + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  aqn_noise_kernel<<<dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream>>>(
      noise, n, sigma, (uint32_t)seed, (uint32_t)(seed >> 32), (uint32_t)subsequence, (uint32_t)(subsequence >> 32));
  return launch_status();
}

extern "C" double aqn_sigma_schedule(int kind, int k, int num_stages, double s0, double s1) {
  if (kind < QERL_SCHEDULE_EXPONENTIAL || kind > QERL_SCHEDULE_LOGARITHMIC) return NAN;
  if (num_stages < 1 || k < 0 || k > num_stages) return NAN;
  if (k == 0) return 0.0;
  if (num_stages == 1) return s0;
  const double u = (double)(k - 1) / (double)(num_stages - 1);
  switch (kind) {
    case QERL_SCHEDULE_EXPONENTIAL: return s0 * pow(s1 / s0, u);
    case QERL_SCHEDULE_LINEAR: return s0 + (s1 - s0) * u;
    case QERL_SCHEDULE_COSINE: return s1 + (s0 - s1) * (1.0 + cos(M_PI * u)) / 2.0;
    default: return s0 + (s1 - s0) * log(1.0 + (double)(k - 1)) / log((double)num_stages);
  }
}
