// fp32 debug path: the same operators as the bf16 MFMA path, with fp32 storage and plain FMA
// arithmetic.  Meant for checking the call graph and the index maps to 1e-4 against the definition,
// not for speed.
#include "device_utils.h"
#include "kernels.h"

namespace wf {

namespace {

// 64x64 tile, 16-deep K steps, 256 threads, 4x4 outputs per thread.
template <int AMODE, int EPI>
__global__ void __launch_bounds__(256) gemm_f32_kernel(GemmArgs p) {
  __shared__ float sA[16][64 + 1];
  __shared__ float sW[16][64 + 1];
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;        // outputs rows ty*4.., cols tx*4..
  const float *A = (const float *)p.A;
  const float *W = (const float *)p.W;
  float acc[4][4] = {};
  // load mapping: 64 rows x 16 k = 1024 elements, 4 per thread: row = e >> 4, k = e & 15
  for (int k0 = 0; k0 < p.K; k0 += 16) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = i * 256 + tid;
      const int r = e >> 4, k = e & 15;
      const int kk = k0 + k;
      float a = 0.0f;
      const int row = m0 + r;
      if (row < p.M && kk < p.K) {
        if (AMODE == A_PLAIN) {
          a = A[(size_t)row * p.lda + kk];
        } else {
          const int tap = kk / p.C;
          const int fl = p.row_flags[row];
          const bool ok = (kk < 3 * p.C) && !((tap == 0) && (fl & 1)) && !((tap == 2) && (fl & 2));
          if (ok) a = A[(long)p.row_src[row] * p.C + kk];
        }
      }
      sA[k][r] = a;
      sW[k][r] = (kk < p.K) ? W[(size_t)(n0 + r) * p.K + kk] : 0.0f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      float a[4], w[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = sA[k][ty * 4 + i]; w[i] = sW[k][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], w[j], acc[i][j]);
    }
    __syncthreads();
  }
  float *out = (float *)p.out;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= p.M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      float v = acc[i][j] + p.bias[n];
      float *o = out + (size_t)m * p.ldo + n;
      if (EPI == EPI_BIAS) *o = v;
      else if (EPI == EPI_BIAS_GELU) *o = gelu_erf(v);
      else if (EPI == EPI_BIAS_RESID) *o += v;
      else if (EPI == EPI_BIAS_F32) *o = v;
      else *o = gelu_erf(v) + p.pos[(size_t)p.row_pos[m] * p.N + n];
    }
  }
}

// One wave per (query token, head).  Keys are visited 64 at a time: lane = key for the logits,
// lane = feature for the weighted sum of values; running max / running sum softmax.
__global__ void __launch_bounds__(256) attention_f32_kernel(AttnArgs p) {
  __shared__ float sQ[4][64];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int m = blockIdx.x * 4 + wave;
  const int head = blockIdx.y;
  const bool active = m < p.M;
  const int mm = active ? m : p.M - 1;
  const int i = find_stream(p.cu_q, p.B, mm);
  const int tok0 = p.cu_kv[i];
  const int ld = p.ldkv;
  // causal: query at position r of its stream sees keys 0..r
  const int L = p.causal ? mm - p.cu_q[i] + 1 : p.cu_kv[i + 1] - tok0;
  sQ[wave][lane] = ((const float *)p.q)[(size_t)mm * p.ldq + head * 64 + lane];
  __syncthreads();
  if (!active) return;
  const float *Kb = (const float *)p.k + (size_t)tok0 * ld + head * 64;
  const float *Vb = (const float *)p.v + (size_t)tok0 * ld + head * 64;
  float m_run = -INFINITY, l_run = 0.0f, o = 0.0f;
  for (int k0 = 0; k0 < L; k0 += 64) {
    const int key = k0 + lane;
    float s = -INFINITY;
    if (key < L) {
      const float *kr = Kb + (size_t)key * ld;
      float dot = 0.0f;
#pragma unroll 8
      for (int f = 0; f < 64; ++f) dot = fmaf(sQ[wave][f], kr[f], dot);
      s = dot * p.scale;
    }
    float tmax = s;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) tmax = fmaxf(tmax, __shfl_xor(tmax, off));
    const float m_new = fmaxf(m_run, tmax);
    const float alpha = expf(m_run - m_new);
    const float pr = (key < L) ? expf(s - m_new) : 0.0f;
    float psum = pr;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) psum += __shfl_xor(psum, off);
    l_run = l_run * alpha + psum;
    o *= alpha;
    const int nkeys = min(64, L - k0);
    for (int kk = 0; kk < nkeys; ++kk) {
      const float pk = __shfl(pr, kk);
      o = fmaf(pk, Vb[(size_t)(k0 + kk) * ld + lane], o);
    }
    m_run = m_new;
  }
  ((float *)p.out)[(size_t)m * p.d_model + head * 64 + lane] = o / l_run;
}

template <int AMODE, int EPI>
hipError_t launch_f32(const GemmArgs &a, hipStream_t s) {
  hipLaunchKernelGGL((gemm_f32_kernel<AMODE, EPI>), dim3(a.N / 64, (a.M + 63) / 64), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm_f32(const GemmArgs &a, AMode amode, Epilogue epi, hipStream_t s) {
  if (a.M <= 0) return hipSuccess;
  if (a.N % 64 != 0 || a.K <= 0) return hipErrorInvalidValue;
  if (amode == A_PLAIN) {
    switch (epi) {
      case EPI_BIAS: return launch_f32<A_PLAIN, EPI_BIAS>(a, s);
      case EPI_BIAS_GELU: return launch_f32<A_PLAIN, EPI_BIAS_GELU>(a, s);
      case EPI_BIAS_RESID: return launch_f32<A_PLAIN, EPI_BIAS_RESID>(a, s);
      case EPI_BIAS_F32: return launch_f32<A_PLAIN, EPI_BIAS_F32>(a, s);
      default: return hipErrorInvalidValue;
    }
  }
  switch (epi) {
    case EPI_BIAS_GELU: return launch_f32<A_CONV3, EPI_BIAS_GELU>(a, s);
    case EPI_BIAS_GELU_POS: return launch_f32<A_CONV3, EPI_BIAS_GELU_POS>(a, s);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_attention_f32(const AttnArgs &a, hipStream_t s) {
  if (a.M <= 0) return hipSuccess;
  if (!a.q || !a.k || !a.v || !a.cu_q || !a.cu_kv || (a.causal && a.cu_q != a.cu_kv)) return hipErrorInvalidValue;
  hipLaunchKernelGGL(attention_f32_kernel, dim3((a.M + 3) / 4, a.n_heads), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace wf
