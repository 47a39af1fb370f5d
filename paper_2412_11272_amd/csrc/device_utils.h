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

// GELU for the bf16 path, z/2 (1 + erf(z / sqrt 2)), without transcendental instructions: its cost sits
// in the GEMM epilogue while the matrix pipe idles.  erf(x) ~ x P(x^2) on [0, 2.8] with P a degree-7
// near-minimax polynomial (|erf error| <= 7.5e-5), x clamped to 2.8 beyond (erf(2.8) = 0.99992).
// Relative error of the result <= 4.7e-4 wherever |GELU| > 0.05, i.e. 8 times below the half-ulp of the
// bf16 value it is rounded to; absolute error <= 1.5e-4 for |z| <= 4.
__device__ __forceinline__ float gelu_fast(float z) {
  const float az = fabsf(z);
  const float x = fminf(az * 0.70710678118654752f, 2.8f);
  const float t = x * x;
  float p = -6.054487471e-07f;
  p = p * t + 2.293834950e-05f;
  p = p * t - 3.810082562e-04f;
  p = p * t + 3.704522969e-03f;
  p = p * t - 2.387478016e-02f;
  p = p * t + 1.095759571e-01f;
  p = p * t - 3.744913936e-01f;
  p = p * t + 1.128137589e+00f;
  const float e = x * p;                  // erf(|z| / sqrt 2)
  return 0.5f * (z + az * e);             // z/2 + |z| erf(|z|/sqrt2)/2 = z/2 (1 + erf(z/sqrt2))
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
