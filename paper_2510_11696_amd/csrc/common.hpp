// Shared host/device helpers of the gfx950 NVFP4 library (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <type_traits>
#include "../../include/qerl_nvfp4.h"

namespace qerl {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kBlock = 16;          // weights per E4M3 scale (Section 3.3)
constexpr int kWave = 64;

// ---- host side ------------------------------------------------------------
void set_last_hip_error(int e);
inline int launch_status() {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_last_hip_error((int)e); return QERL_ERR_LAUNCH; }
  return QERL_OK;
}
inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// ---- device side ----------------------------------------------------------
__device__ __forceinline__ int64_t ceil_div_dev(int64_t a, int64_t b) { return (a + b - 1) / b; }
// bf16 <-> fp32 by bit manipulation (bf16 is the top half of an fp32).
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

// fp32 -> bf16 bits, round-to-nearest-even (finite inputs).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  return (uint32_t)__builtin_bit_cast(unsigned short, (__bf16)f);
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  bf16x2 v; v.x = (__bf16)lo; v.y = (__bf16)hi;      // v_cvt_pk_bf16_f32
  return __builtin_bit_cast(uint32_t, v);
}

// Eight gated activations: bf16(bf16(SiLU(g)) * u), SiLU(g) = g / (1 + e^-g) -- the roundings of a bf16 model
// evaluated operator by operator.  The function itself is evaluated in fp32 with the hardware's exp2 and
// reciprocal (about 1 ulp each: every consumer workgroup of the decode kernel recomputes its slice, so the
// dozens of instructions of the exactly rounded library routines would cost microseconds per launch); the
// result before the rounding to bf16 is within a few fp32 ulp of the exact one.  g -> -inf gives -0, g -> +inf gives g.
__device__ __forceinline__ float silu_f32(float g) {
  const float e = __builtin_amdgcn_exp2f(g * -1.44269504088896341f);   // e^-g; +inf for g << 0
  return g * __builtin_amdgcn_rcpf(1.0f + e);
}
__device__ __forceinline__ uint32_t silu_mul2(uint32_t g, uint32_t u) {
  const float g0 = bf16_bits_to_f32(g & 0xffffu), g1 = __uint_as_float(g & 0xffff0000u);
  const float u0 = bf16_bits_to_f32(u & 0xffffu), u1 = __uint_as_float(u & 0xffff0000u);
  const uint32_t s = pack_bf16x2(silu_f32(g0), silu_f32(g1));
  return pack_bf16x2(bf16_bits_to_f32(s & 0xffffu) * u0, __uint_as_float(s & 0xffff0000u) * u1);
}
__device__ __forceinline__ u32x4 silu_mul8(u32x4 g, u32x4 u) {
  return u32x4{silu_mul2(g[0], u[0]), silu_mul2(g[1], u[1]), silu_mul2(g[2], u[2]), silu_mul2(g[3], u[3])};
}

// Eight normalised activations of one token row (Eq. 10): bf16((gain[k] + noise[k]) * (x[k] * rstd)) for
// k = k0 .. k0 + 7 (k0 a multiple of 8; gain 16-byte aligned, noise 16-byte aligned or null); gain + noise is
// formed in fp32 and not re-rounded, one rounding at the end -- the arithmetic of aqn_rmsnorm.
__device__ __forceinline__ u32x4 norm_scale8(u32x4 v, float rstd, const uint16_t* __restrict__ gain,
                                             const float* __restrict__ noise, int64_t k0) {
  const u32x4 g = *reinterpret_cast<const u32x4*>(gain + k0);
  f32x4 z0 = {0.f, 0.f, 0.f, 0.f}, z1 = {0.f, 0.f, 0.f, 0.f};
  if (noise) {
    z0 = *reinterpret_cast<const f32x4*>(noise + k0);
    z1 = *reinterpret_cast<const f32x4*>(noise + k0 + 4);
  }
  const float z[8] = {z0[0], z0[1], z0[2], z0[3], z1[0], z1[1], z1[2], z1[3]};
  u32x4 o;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float ga = bf16_bits_to_f32(g[j] & 0xffffu) + z[2 * j];
    const float gb = bf16_bits_to_f32(g[j] >> 16) + z[2 * j + 1];
    const float a = bf16_bits_to_f32(v[j] & 0xffffu), b = bf16_bits_to_f32(v[j] >> 16);
    o[j] = pack_bf16x2(ga * (a * rstd), gb * (b * rstd));
  }
  return o;
}

// E4M3 byte (sign clear, not NaN) -> fp32, exact.  (b << 20) places the 4+3
// bits at an fp32's low exponent / top mantissa bits; multiplying by 2^120
// re-biases 127 -> 7 and, with fp32 denormals enabled, also covers the
// subnormal bytes (exponent field 0).
__device__ __forceinline__ float e4m3_to_f32(uint32_t b) {
  return __uint_as_float(b << 20) * 0x1p120f;
}

// E2M1 code (4 bits, bit 3 = sign) -> fp32, exact: {0, .5, 1, 1.5, 2, 3, 4, 6}.
__device__ __forceinline__ float e2m1_to_f32(uint32_t c) {
  // place exponent(2)+mantissa(1) like above, re-bias 127 -> 1
  float mag = __uint_as_float((c & 7u) << 22) * 0x1p126f;
  return __uint_as_float(__float_as_uint(mag) | ((c & 8u) << 28));
}

// Two fp32 values that are exactly representable in bf16 (low halves zero, e.g. an E2M1 value times an E4M3
// scale: at most 6 significant bits) -> packed bf16 pair.  One byte permute; the rounding conversion costs twice
// the issue time and does not run beside matrix instructions.
__device__ __forceinline__ uint32_t pack_bf16x2_exact(float lo, float hi) {
  return __builtin_amdgcn_perm(__float_as_uint(hi), __float_as_uint(lo), 0x07060302u);
}

// 8 weights of one lane (one dword of codes) times their block scale -> bf16 x8
__device__ __forceinline__ bf16x8 dequant8_bf16(uint32_t codes, float s) {
  const f32x2 p0 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(codes, 1.0f, 0);
  const f32x2 p1 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(codes, 1.0f, 1);
  const f32x2 p2 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(codes, 1.0f, 2);
  const f32x2 p3 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(codes, 1.0f, 3);
  u32x4 o;
  o[0] = pack_bf16x2_exact(p0.x * s, p0.y * s);
  o[1] = pack_bf16x2_exact(p1.x * s, p1.y * s);
  o[2] = pack_bf16x2_exact(p2.x * s, p2.y * s);
  o[3] = pack_bf16x2_exact(p3.x * s, p3.y * s);
  return __builtin_bit_cast(bf16x8, o);
}

// 8 weights of one lane that lie along the rows of W (one dword of codes of the transposed tile order), each
// times its own block scale (the 8 scale bytes in sc) -> bf16 x8; every product is exact
__device__ __forceinline__ bf16x8 dequant8_t_bf16(uint32_t codes, u32x2 sc) {
  const f32x2 p0 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(codes, 1.0f, 0);
  const f32x2 p1 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(codes, 1.0f, 1);
  const f32x2 p2 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(codes, 1.0f, 2);
  const f32x2 p3 = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(codes, 1.0f, 3);
  u32x4 o;
  o[0] = pack_bf16x2_exact(p0.x * __builtin_amdgcn_cvt_f32_fp8(sc[0], 0), p0.y * __builtin_amdgcn_cvt_f32_fp8(sc[0], 1));
  o[1] = pack_bf16x2_exact(p1.x * __builtin_amdgcn_cvt_f32_fp8(sc[0], 2), p1.y * __builtin_amdgcn_cvt_f32_fp8(sc[0], 3));
  o[2] = pack_bf16x2_exact(p2.x * __builtin_amdgcn_cvt_f32_fp8(sc[1], 0), p2.y * __builtin_amdgcn_cvt_f32_fp8(sc[1], 1));
  o[3] = pack_bf16x2_exact(p3.x * __builtin_amdgcn_cvt_f32_fp8(sc[1], 2), p3.y * __builtin_amdgcn_cvt_f32_fp8(sc[1], 3));
  return __builtin_bit_cast(bf16x8, o);
}

__device__ __forceinline__ float e4m3_byte_f32(uint32_t v, int b) {
  switch (b) {
    case 0: return __builtin_amdgcn_cvt_f32_fp8(v, 0);
    case 1: return __builtin_amdgcn_cvt_f32_fp8(v, 1);
    case 2: return __builtin_amdgcn_cvt_f32_fp8(v, 2);
    default: return __builtin_amdgcn_cvt_f32_fp8(v, 3);
  }
}

// Eight fp32 values -> three bf16 terms hi + mid + lo (packed pairs) whose sum equals the value to 2^-24
// relative: lets an fp32 operand (t = x A^T) ride through bf16 matrix instructions without losing precision.
__device__ __forceinline__ void split3_bf16(const float (&v)[8], u32x4& hi, u32x4& mid, u32x4& lo) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t h = pack_bf16x2(v[2 * i], v[2 * i + 1]);
    const float r0 = v[2 * i] - bf16_bits_to_f32(h & 0xffffu), r1 = v[2 * i + 1] - __uint_as_float(h & 0xffff0000u);
    const uint32_t m = pack_bf16x2(r0, r1);
    const float q0 = r0 - bf16_bits_to_f32(m & 0xffffu), q1 = r1 - __uint_as_float(m & 0xffff0000u);
    hi[i] = h; mid[i] = m; lo[i] = pack_bf16x2(q0, q1);
  }
}

// fp32 v >= 0 -> E4M3 byte, nearest-even, subnormals kept, saturating at 448.
__device__ __forceinline__ uint32_t e4m3_encode_rne_sat(float v) {
  if (v >= 448.0f) return 0x7Eu;
  if (v < 0x1p-6f) return (uint32_t)__builtin_rintf(v * 512.0f);   // units of 2^-9; 8 carries into 0x08
  uint32_t b = __float_as_uint(v);
  b += 0x7FFFFu + ((b >> 20) & 1u);                                // round the 20 dropped bits to even
  return (b >> 20) - (120u << 3);                                  // re-bias 127 -> 7
}

// fp32 q >= 0 -> E2M1 magnitude index.  The boundaries are the midpoints of
// {0,.5,1,1.5,2,3,4,6}; a midpoint goes to the neighbour with mantissa bit 0.
__device__ __forceinline__ uint32_t e2m1_encode_rne_sat(float q) {
  return (uint32_t)(q > 0.25f) + (uint32_t)(q >= 0.75f) + (uint32_t)(q > 1.25f) +
         (uint32_t)(q >= 1.75f) + (uint32_t)(q > 2.5f) + (uint32_t)(q >= 3.5f) + (uint32_t)(q > 5.0f);
}

// Sum of S fp32 values `stride` words apart, read with agent-scope atomic loads
// (they bypass the per-XCD L2).  Loads are issued eight at a time before any
// is consumed, and added in index order, so the result does not depend on timing.
__device__ __forceinline__ float ordered_sum_sc1(const uint32_t* p, int64_t stride, int S) {
  float sum = 0.f;
  for (int z0 = 0; z0 < S; z0 += 8) {
    uint32_t v[8];
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      v[b] = 0u;   // +0.0f
      if (z0 + b < S) v[b] = __hip_atomic_load(p + (int64_t)(z0 + b) * stride, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
#pragma unroll
    for (int b = 0; b < 8; ++b) sum += __uint_as_float(v[b]);
  }
  return sum;
}

// Sum over the 64 lanes, the same value (and the same association order) in every lane.  Within
// each row of 16 lanes a butterfly on the data-parallel-primitive path (no LDS round trips):
// neighbours, pairs, the mirrored quad of the other half-row, the mirrored half-row; then the four
// row sums are read out and added as (r0 + r1) + (r2 + r3).
__device__ __forceinline__ float wave_sum(float v) {
  auto dpp_add = [](float x, auto ctrl) {
    const int y = __builtin_amdgcn_update_dpp(0, __float_as_int(x), decltype(ctrl)::value, 0xf, 0xf, false);
    return x + __int_as_float(y);
  };
  v = dpp_add(v, std::integral_constant<int, 0xB1>{});    // quad_perm [1,0,3,2]
  v = dpp_add(v, std::integral_constant<int, 0x4E>{});    // quad_perm [2,3,0,1]
  v = dpp_add(v, std::integral_constant<int, 0x141>{});   // row_half_mirror
  v = dpp_add(v, std::integral_constant<int, 0x140>{});   // row_mirror
  const float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
  const float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
  const float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
  const float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
  return (r0 + r1) + (r2 + r3);
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) { uint32_t t = __shfl_xor(v, o, 64); v = t > v ? t : v; }
  return v;
}

}  // namespace qerl
