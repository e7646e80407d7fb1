// Small device helpers shared by the kernels: bf16 <-> fp32 (round to nearest even) and the
// activation functions with their derivatives.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tp {

__device__ __forceinline__ float bf16_to_float(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

__device__ __forceinline__ uint16_t float_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);  // quiet NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// two fp32 -> packed bf16 pair, round to nearest even (v_cvt_pk_bf16_f32 on gfx950)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef float floatx2_t __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  const floatx2_t f = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_t));
}

__device__ __forceinline__ float to_float(float v) { return v; }
__device__ __forceinline__ float to_float(uint16_t v) { return bf16_to_float(v); }

template <typename T>
__device__ __forceinline__ T from_float(float v);
template <>
__device__ __forceinline__ float from_float<float>(float v) { return v; }
template <>
__device__ __forceinline__ uint16_t from_float<uint16_t>(float v) { return float_to_bf16(v); }

// act: 0 none, 1 ReLU, 2 GELU (exact erf form)
__device__ __forceinline__ float act_forward(float z, int act) {
  if (act == 1) return fmaxf(z, 0.f);
  if (act == 2) return 0.5f * z * (1.f + erff(z * 0.70710678118654752f));
  return z;
}

__device__ __forceinline__ float act_derivative(float z, int act) {
  if (act == 1) return z > 0.f ? 1.f : 0.f;
  if (act == 2)
    return 0.5f * (1.f + erff(z * 0.70710678118654752f)) + z * 0.39894228040143268f * __expf(-0.5f * z * z);
  return 1.f;
}

// GELU (erf form) and its derivative with one exponential and one reciprocal:
//   erf(x) = 1 - (a1 t + a2 t^2 + a3 t^3 + a4 t^4 + a5 t^5) exp(-x^2),  t = 1/(1 + p x),  x >= 0
// (Abramowitz & Stegun 7.1.26, |error| <= 1.5e-7), evaluated at x = |z|/sqrt(2), where
// exp(-x^2) = exp(-z^2/2) is also the Gaussian factor of the derivative.
struct GeluParts {
  float cdf;  // Phi(z) = 0.5 (1 + erf(z/sqrt 2))
  float pdf;  // phi(z) = exp(-z^2/2)/sqrt(2 pi)
};
__device__ __forceinline__ GeluParts gelu_parts(float z) {
  const float x = fabsf(z) * 0.70710678118654752f;
  const float t = __frcp_rn(fmaf(0.3275911f, x, 1.0f));
  const float e = __expf(-0.5f * z * z);
  float poly = fmaf(1.061405429f, t, -1.453152027f);
  poly = fmaf(poly, t, 1.421413741f);
  poly = fmaf(poly, t, -0.284496736f);
  poly = fmaf(poly, t, 0.254829592f);
  const float half_erfc = 0.5f * poly * t * e;        // 0.5 * (1 - erf(x))
  GeluParts g;
  g.cdf = z >= 0.f ? 1.0f - half_erfc : half_erfc;
  g.pdf = 0.39894228040143268f * e;
  return g;
}
// act(z) and act'(z) together (they share the exponential and the reciprocal)
struct ActPair {
  float a, d;
};
__device__ __forceinline__ ActPair act_pair_fast(float z, int act) {
  ActPair p;
  if (act == 2) {
    const GeluParts g = gelu_parts(z);
    p.a = z * g.cdf;
    p.d = fmaf(z, g.pdf, g.cdf);
  } else if (act == 1) {
    p.a = fmaxf(z, 0.f);
    p.d = z > 0.f ? 1.f : 0.f;
  } else {
    p.a = z;
    p.d = 1.f;
  }
  return p;
}
__device__ __forceinline__ float act_forward_fast(float z, int act) {
  if (act == 1) return fmaxf(z, 0.f);
  if (act == 2) return z * gelu_parts(z).cdf;
  return z;
}
__device__ __forceinline__ float act_derivative_fast(float z, int act) {
  if (act == 1) return z > 0.f ? 1.f : 0.f;
  if (act == 2) {
    const GeluParts g = gelu_parts(z);
    return fmaf(z, g.pdf, g.cdf);
  }
  return 1.f;
}

}  // namespace tp
