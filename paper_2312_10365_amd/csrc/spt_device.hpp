// Device-side helpers shared by the routed-FFN kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace spt {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// Round-to-nearest-even float -> bf16 bit pattern (finite inputs).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  const uint32_t u = __float_as_uint(f);
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
// Two floats -> packed bf16 pair, round-to-nearest-even: one v_cvt_pk_bf16_f32 on gfx950.
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
__device__ __forceinline__ float lo_bf16(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float hi_bf16(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// Standard normal CDF Phi(z) and exp(-z^2/2), branch-free.  erf comes from the rational
// approximation 7.1.26 of Abramowitz & Stegun (absolute error 1.5e-7 as published, 2.6e-7
// as evaluated here in fp32; far under the bf16 rounding of everything it feeds): erfc(x) = t (a1 + t (a2 + ... t a5)) exp(-x^2),
// t = 1 / (1 + p x), x >= 0.  For z < 0, Phi(z) = erfc(|z|/sqrt 2) / 2 is used directly, so
// the negative tail keeps its relative accuracy.
__device__ __forceinline__ float normal_cdf(float z, float& gauss) {
  const float x = fabsf(z) * 0.70710678118654752f;
  const float t = __frcp_rn(fmaf(0.3275911f, x, 1.0f));
  gauss = __expf(-x * x);
  float poly = fmaf(t, 1.061405429f, -1.453152027f);
  poly = fmaf(t, poly, 1.421413741f);
  poly = fmaf(t, poly, -0.284496736f);
  poly = fmaf(t, poly, 0.254829592f);
  const float half_erfc = 0.5f * t * poly * gauss;
  return z >= 0.f ? 1.0f - half_erfc : half_erfc;
}

// Activation of Eq. 4 (ReLU) or the erf-form GELU z*Phi(z), and its derivative
// Phi(z) + z phi(z).
template <int ACT>
__device__ __forceinline__ float act_fn(float z) {
  if (ACT == 1) return z > 0.f ? z : 0.f;
  float g;
  return z * normal_cdf(z, g);
}
template <int ACT>
__device__ __forceinline__ float act_grad(float z) {
  if (ACT == 1) return z > 0.f ? 1.f : 0.f;
  float g;
  const float cdf = normal_cdf(z, g);
  return fmaf(z * 0.39894228040143268f, g, cdf);
}

}  // namespace spt
