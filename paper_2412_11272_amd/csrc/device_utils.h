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

// GELU for the bf16 path, z Phi(z) = z (1/2 + erf(z / sqrt 2) / 2), without transcendental instructions: its cost
// sits in the GEMM epilogue while the matrix pipe idles.  erf(z / sqrt 2) / 2 ~ c Q(c^2) with c = z clamped to
// +-2.8 sqrt 2 and Q a degree-7 near-minimax polynomial (|erf error| <= 7.5e-5; erf(2.8) = 0.99992 beyond the clamp):
// 11 instructions per value (clamp, square, 7 fused multiply-adds, one more, one multiply).
// Relative error of the result <= 4.7e-4 wherever |GELU| > 0.05, i.e. 8 times below the half-ulp of the
// bf16 value it is rounded to; absolute error <= 1.5e-4 for |z| <= 4 and <= 6e-5 |z| beyond (past the clamp
// Phi saturates at 0.99994 / 0.00006 instead of 1 / 0).
__host__ __device__ __forceinline__ float gelu_fast(float z) {
  const float c = fminf(fmaxf(z, -3.959797975f), 3.959797975f);
  const float t = c * c;
  float q = -1.672331698e-09f;
  q = q * t + 1.267176756e-07f;
  q = q * t - 4.209586276e-06f;
  q = q * t + 8.185916601e-05f;
  q = q * t - 1.055126184e-03f;
  q = q * t + 9.685237790e-03f;
  q = q * t - 6.620135098e-02f;
  q = q * t + 3.988568696e-01f;
  return z * (c * q + 0.5f);              // z (1/2 + erf(z / sqrt 2) / 2)
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
