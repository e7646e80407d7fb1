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

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return (uint32_t)float_to_bf16(lo) | ((uint32_t)float_to_bf16(hi) << 16);
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

}  // namespace tp
