// Bandwidth-bound kernels: ragged pack + hush append (with the row maps the convolutions need) and
// LayerNorm.  Both read and write every byte exactly once with 16-byte accesses.
#include "device_utils.h"
#include "kernels.h"

namespace wf {

namespace {

// ---------------------------------------------------------------------------------------------
// prep: (1) packed[r, :] = frame t of stream i  (t < T_i: the caller's frame; else hush[t - T_i]),
//           the concatenation x (+) h of every stream laid back to back without padding;
//       (2) conv1 row map: window of packed row r starts at row r-1; the first frame of a stream has
//           no left neighbour and the last no right neighbour (zero padding is per stream);
//       (3) conv2 row map: token j of stream i reads frames 2j-1, 2j, 2j+1 of that stream.
// One thread per 8 mel bins (threads [0, total_frames * n_mels/8)), then one thread per token.
template <typename TIN, typename TOUT>
__global__ void __launch_bounds__(256) prep_kernel(PrepArgs p) {
  const int cpr = p.n_mels >> 3;                       // 8-element chunks per frame
  const long n_pack = (long)p.total_frames * cpr;
  const long gid = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid < n_pack) {
    const int r = (int)(gid / cpr), c = (int)(gid % cpr);
    const int i = find_stream(p.cu_frames, p.B, r);
    const int t = r - p.cu_frames[i];
    const int T = p.n_frames[i];
    const int Tp = p.cu_frames[i + 1] - p.cu_frames[i];
    TOUT *dst = (TOUT *)p.packed + (size_t)r * p.n_mels + c * 8;
    if (t < T) {
      const TIN *src = (const TIN *)p.mel + ((size_t)p.frame_offset[i] + t) * p.n_mels + c * 8;
#pragma unroll
      for (int e = 0; e < 8; ++e) dst[e] = (TOUT)(float)src[e];
    } else {
      const TOUT *src = (const TOUT *)p.hush + (size_t)(t - T) * p.n_mels + c * 8;
#pragma unroll
      for (int e = 0; e < 8; ++e) dst[e] = src[e];
    }
    if (c == 0) {
      p.frame_src[r] = r - 1;
      p.frame_flags[r] = (t == 0 ? 1 : 0) | (t == Tp - 1 ? 2 : 0);
    }
    return;
  }
  const long m = gid - n_pack;
  if (m < p.M) {
    const int i = find_stream(p.cu_seqlens, p.B, (int)m);
    const int j = (int)m - p.cu_seqlens[i];
    const int Tp = p.cu_frames[i + 1] - p.cu_frames[i];
    p.tok_src[m] = p.cu_frames[i] + 2 * j - 1;
    p.tok_flags[m] = (j == 0 ? 1 : 0) | (2 * j + 1 >= Tp ? 2 : 0);
    p.tok_pos[m] = j;
  }
}

// ---------------------------------------------------------------------------------------------
// LayerNorm: one wave per row, the row lives in registers between the two statistics passes
// (mean, then centred variance -- the biased one), fp32 statistics.
template <typename TOUT, int MAXV>   // MAXV float4 per lane: d <= 256 * MAXV
__global__ void __launch_bounds__(256) layernorm_kernel(const float *__restrict__ x, const float *__restrict__ g,
                                                        const float *__restrict__ b, TOUT *__restrict__ out,
                                                        int M, int d, float eps) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= M) return;
  const int lane = threadIdx.x & 63;
  const int nv = d >> 2;                               // float4 per row
  const f32x4 *xr = (const f32x4 *)(x + (size_t)row * d);
  f32x4 v[MAXV];
  float sum = 0.0f;
#pragma unroll
  for (int i = 0; i < MAXV; ++i) {
    const int idx = lane + i * 64;
    if (idx < nv) {
      v[i] = xr[idx];
      sum += v[i][0] + v[i][1] + v[i][2] + v[i][3];
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
  const float mu = sum / (float)d;
  float sq = 0.0f;
#pragma unroll
  for (int i = 0; i < MAXV; ++i) {
    const int idx = lane + i * 64;
    if (idx < nv) {
#pragma unroll
      for (int e = 0; e < 4; ++e) { const float t = v[i][e] - mu; sq += t * t; }
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) sq += __shfl_xor(sq, off);
  const float rstd = rsqrtf(sq / (float)d + eps);
  const f32x4 *gr = (const f32x4 *)g, *br = (const f32x4 *)b;
#pragma unroll
  for (int i = 0; i < MAXV; ++i) {
    const int idx = lane + i * 64;
    if (idx < nv) {
      const f32x4 gg = gr[idx], bb = br[idx];
      f32x4 y;
#pragma unroll
      for (int e = 0; e < 4; ++e) y[e] = (v[i][e] - mu) * rstd * gg[e] + bb[e];
      if constexpr (sizeof(TOUT) == 2) {
        *(bf16x4 *)((__bf16 *)out + (size_t)row * d + idx * 4) = to_bf16x4(y);
      } else {
        *(f32x4 *)((float *)out + (size_t)row * d + idx * 4) = y;
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Decoder input: x[r, :] = table[tok[r], :] + pos[pos_idx[r], :], one thread per 4 features.
template <typename TTAB>
__global__ void __launch_bounds__(256) embed_kernel(const TTAB *__restrict__ table, const float *__restrict__ pos,
                                                    const int32_t *__restrict__ tok, const int32_t *__restrict__ pos_idx,
                                                    float *__restrict__ x, int rows, int d) {
  const int cpr = d >> 2;
  const long gid = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= (long)rows * cpr) return;
  const int r = (int)(gid / cpr), c = (int)(gid % cpr) * 4;
  const TTAB *t = table + (size_t)tok[r] * d + c;
  const f32x4 pe = *(const f32x4 *)(pos + (size_t)pos_idx[r] * d + c);
  f32x4 v;
#pragma unroll
  for (int e = 0; e < 4; ++e) v[e] = (float)t[e] + pe[e];
  *(f32x4 *)(x + (size_t)r * d + c) = v;
}

// dst[i, :] = src[row[i], :], 16 bytes per thread.
__global__ void __launch_bounds__(256) gather_rows_kernel(const unsigned char *__restrict__ src, const int32_t *__restrict__ row,
                                                          unsigned char *__restrict__ dst, int n, int row_bytes) {
  const int cpr = row_bytes >> 4;
  const long gid = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= (long)n * cpr) return;
  const int i = (int)(gid / cpr), c = (int)(gid % cpr);
  *(f32x4 *)(dst + (size_t)i * row_bytes + c * 16) = *(const f32x4 *)(src + (size_t)row[i] * row_bytes + c * 16);
}

}  // namespace

hipError_t launch_embed(const void *table, int table_bf16, const float *pos, const int32_t *tok, const int32_t *pos_idx,
                        float *x, int32_t rows, int32_t d, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  if (d % 4 != 0) return hipErrorInvalidValue;
  const long n = (long)rows * (d / 4);
  const dim3 grid((unsigned)((n + 255) / 256)), block(256);
  if (table_bf16) hipLaunchKernelGGL(embed_kernel<__bf16>, grid, block, 0, s, (const __bf16 *)table, pos, tok, pos_idx, x, rows, d);
  else hipLaunchKernelGGL(embed_kernel<float>, grid, block, 0, s, (const float *)table, pos, tok, pos_idx, x, rows, d);
  return hipGetLastError();
}

hipError_t launch_gather_rows(const void *src, const int32_t *row, void *dst, int32_t n, int32_t row_bytes, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  if (row_bytes % 16 != 0) return hipErrorInvalidValue;
  const long t = (long)n * (row_bytes / 16);
  hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)((t + 255) / 256)), dim3(256), 0, s, (const unsigned char *)src, row,
                     (unsigned char *)dst, n, row_bytes);
  return hipGetLastError();
}

hipError_t launch_layernorm(const float *x, const float *g, const float *b, void *out, int out_bf16,
                            int32_t M, int32_t d, float eps, hipStream_t s) {
  if (M <= 0) return hipSuccess;
  if (d % 4 != 0 || d > 256 * 8) return hipErrorInvalidValue;
  const dim3 grid((M + 3) / 4), block(256);
  if (d <= 256 * 2) {
    if (out_bf16) hipLaunchKernelGGL((layernorm_kernel<__bf16, 2>), grid, block, 0, s, x, g, b, (__bf16 *)out, M, d, eps);
    else hipLaunchKernelGGL((layernorm_kernel<float, 2>), grid, block, 0, s, x, g, b, (float *)out, M, d, eps);
  } else if (d <= 256 * 5) {
    if (out_bf16) hipLaunchKernelGGL((layernorm_kernel<__bf16, 5>), grid, block, 0, s, x, g, b, (__bf16 *)out, M, d, eps);
    else hipLaunchKernelGGL((layernorm_kernel<float, 5>), grid, block, 0, s, x, g, b, (float *)out, M, d, eps);
  } else {
    if (out_bf16) hipLaunchKernelGGL((layernorm_kernel<__bf16, 8>), grid, block, 0, s, x, g, b, (__bf16 *)out, M, d, eps);
    else hipLaunchKernelGGL((layernorm_kernel<float, 8>), grid, block, 0, s, x, g, b, (float *)out, M, d, eps);
  }
  return hipGetLastError();
}

hipError_t launch_prep(const PrepArgs &a, int packed_bf16, hipStream_t s) {
  const long n = (long)a.total_frames * (a.n_mels / 8) + a.M;
  if (n <= 0) return hipSuccess;
  const dim3 grid((unsigned)((n + 255) / 256)), block(256);
  if (packed_bf16) {
    if (a.mel_is_bf16) hipLaunchKernelGGL((prep_kernel<__bf16, __bf16>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((prep_kernel<float, __bf16>), grid, block, 0, s, a);
  } else {
    if (a.mel_is_bf16) hipLaunchKernelGGL((prep_kernel<__bf16, float>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((prep_kernel<float, float>), grid, block, 0, s, a);
  }
  return hipGetLastError();
}

}  // namespace wf
