// Small device-side helpers shared by the gfx950 kernels: vector types, bf16 conversion, GELU.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace wf {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// float -> bf16 with round-to-nearest-even (gfx950 has the conversion in hardware).
__device__ __forceinline__ bf16x4 to_bf16x4(f32x4 v) { return __builtin_convertvector(v, bf16x4); }
__device__ __forceinline__ float bf16_to_float(__bf16 v) { return (float)v; }

// Exact-form GELU, z/2 (1 + erf(z / sqrt 2)), for the fp32 debug path.
__device__ __forceinline__ float gelu_erf(float z) { return 0.5f * z * (1.0f + erff(z * 0.70710678118654752f)); }

// GELU for the bf16 path.  erf by the rational-times-Gaussian formula 7.1.26 of Abramowitz & Stegun
// (|error| <= 1.5e-7, far below bf16 resolution): erf(x) = 1 - (a1 t + ... + a5 t^5) exp(-x^2),
// t = 1/(1 + p x), x >= 0; odd extension for x < 0.
__device__ __forceinline__ float gelu_fast(float z) {
  const float x = fabsf(z) * 0.70710678118654752f;
  const float t = __frcp_rn(1.0f + 0.3275911f * x);
  float poly = 1.061405429f;
  poly = poly * t - 1.453152027f;
  poly = poly * t + 1.421413741f;
  poly = poly * t - 0.284496736f;
  poly = poly * t + 0.254829592f;
  poly *= t;
  const float e = __expf(-x * x);
  const float erf_abs = 1.0f - poly * e;         // erf(|z|/sqrt2)
  const float erf_z = copysignf(erf_abs, z);
  return 0.5f * z * (1.0f + erf_z);
}

// First stream index i with cu[i+1] > r, for a row r in [0, cu[B]).
__device__ __forceinline__ int find_stream(const int32_t *cu, int B, int r) {
  int lo = 0, hi = B - 1;
  while (lo < hi) {
    int mid = (lo + hi) >> 1;
    if (cu[mid + 1] > r) hi = mid; else lo = mid + 1;
  }
  return lo;
}

}  // namespace wf
