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

// Activation of Eq. 4 (ReLU) or the erf-form GELU z*Phi(z), and its derivative.
template <int ACT>
__device__ __forceinline__ float act_fn(float z) {
  if (ACT == 1) return z > 0.f ? z : 0.f;
  return 0.5f * z * (1.f + erff(z * 0.70710678118654752f));
}
template <int ACT>
__device__ __forceinline__ float act_grad(float z) {
  if (ACT == 1) return z > 0.f ? 1.f : 0.f;
  const float cdf = 0.5f * (1.f + erff(z * 0.70710678118654752f));
  return cdf + z * 0.39894228040143268f * __expf(-0.5f * z * z);
}

}  // namespace spt
