// bf16 MFMA GEMM for SMALL row counts (a single stream's buffer, a few hundred tokens: the case the paper's
// method itself runs, Section "Operations"), where nothing is bound by the matrix pipe and everything by how long
// the chain of dependent steps of one workgroup is and by how many workgroups share the work.
//
//   out = epilogue(A . W^T),  A [M, K], W [N, K], fp32 accumulation, M up to about a thousand rows.
//
// Differences from the large-batch kernels of gemm_bf16.hip:
//   * 32-row output tiles, 32, 64 or 128 columns wide (NB column blocks of 32), so that even a 75-token batch spreads
//     over dozens of compute units (75 x 384: 36 workgroups instead of 3); the launcher takes the widest tile that
//     still leaves about 160 workgroups, because every column tile re-reads (and with A_LN re-normalises) the same
//     32 activation rows;
//   * the four waves of a workgroup split the reduction: in every 64-deep K step wave w multiplies the k slice
//     [16 w, 16 w + 16) with one 32x32x16 MFMA, and the four partial tiles are added in a fixed order through LDS
//     at the end (deterministic);
//   * operand chunks are requested eight (widest tile: four) K steps ahead into registers, so the K loop runs at the rate the chunks
//     arrive instead of one memory latency per step, and two K steps are staged in LDS per barrier;
//   * A_LN: the activation operand is LayerNorm(x) of an fp32 matrix x, normalised on the way into LDS.  The
//     workgroup first computes mean and 1/sqrt(var + eps) of its 32 rows (one pass, sums shifted by the row's first
//     element so that the variance does not cancel), then every chunk is (x - mean) * rstd * gamma + beta rounded
//     to bf16 -- exactly what the LayerNorm kernel would have stored.  This removes two kernels per transformer
//     block; with a few hundred tokens each kernel in the chain costs 5-7 us whatever it does.

#include "device_utils.h"
#include "kernels.h"

namespace wf {

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int SBM = 32, SBN = 32, SBK = 64;
constexpr int kMaxLnK = 2048;     // A_LN keeps the LayerNorm gain and shift of the whole row in LDS

template <int AMODE, int EPI, int NB>
__global__ void __launch_bounds__(256) gemm_small_kernel(GemmArgs p) {
  constexpr int TN = NB * SBN;                                               // tile width in columns
  constexpr int DEPTH = NB >= 4 ? 4 : 8;                                     // K steps in flight (register ring)
  // SPB K steps are staged in LDS per barrier, double-buffered (NS = 2 SPB stages per operand); the four waves'
  // partial tiles reuse the same memory after the K loop.
  constexpr int SPB = 2, NS = 2 * SPB;               // (four per barrier measured the same as two)
  constexpr int STAGE_BYTES = NS * (SBM + TN) * 128, PART_BYTES = 4 * SBM * (TN + 4) * 4;
  __shared__ __attribute__((aligned(16))) unsigned char sMem[STAGE_BYTES > PART_BYTES ? STAGE_BYTES : PART_BYTES];
  unsigned char(*sA)[SBM * 128] = (unsigned char(*)[SBM * 128])sMem;                     // [stage][row][64 bf16]
  unsigned char(*sW)[TN * 128] = (unsigned char(*)[TN * 128])(sMem + NS * SBM * 128);
  float(*sPart)[SBM][TN + 4] = (float(*)[SBM][TN + 4])sMem;
  __shared__ __attribute__((aligned(16))) float sGain[AMODE == A_LN ? kMaxLnK : 4], sShift[AMODE == A_LN ? kMaxLnK : 4];

  const int tiles_n = p.N / TN;
  const int m0 = (blockIdx.x / tiles_n) * SBM, n0 = (blockIdx.x % tiles_n) * TN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lg = lane >> 5;

  // ---- load descriptors: thread -> (row r, 16-byte chunk ch) of both operand tiles, fixed over the K loop
  const int r = tid >> 3, ch = tid & 7;
  int row = m0 + r;
  row = row < p.M ? row : p.M - 1;               // rows past M are computed but never stored
  const int lds_off = r * 128 + ((ch ^ ((r >> 1) & 7)) << 4);
  const __bf16 *W = (const __bf16 *)p.W;
  const __bf16 *wptr[NB];                        // weight rows n0 + 32 j + r
#pragma unroll
  for (int j = 0; j < NB; ++j) {
    const int n = n0 + j * SBN + r;
    wptr[j] = p.w_panels ? W + ((size_t)(n >> 8) * (p.K >> 6) << 14) + ((n & 255) << 6) + ch * 8 : W + (size_t)n * p.K + ch * 8;
  }
  const int wstep = p.w_panels ? 1 << 14 : SBK;
  const __bf16 *aptr = nullptr;
  const float *xptr = nullptr;
  int flags = 0;
  if constexpr (AMODE == A_PLAIN) aptr = (const __bf16 *)p.A + (size_t)row * p.lda + ch * 8;
  else if constexpr (AMODE == A_CONV3) {
    aptr = (const __bf16 *)p.A + (long)p.row_src[row] * p.C + ch * 8;
    flags = p.row_flags[row];
  } else xptr = (const float *)p.A + (size_t)row * p.lda + ch * 8;

  [[maybe_unused]] float mu = 0.0f, rstd = 0.0f;     // A_LN: statistics of this thread's row
  // ---- operand pipeline: chunks of K step kt + DEPTH - 1 are requested while step kt is multiplied
  u32x4 wreg[DEPTH][NB];
  [[maybe_unused]] u32x4 areg[DEPTH];
  [[maybe_unused]] f32x4 xreg[DEPTH][2];
  const int nk = p.K / SBK;
  auto request = [&](int kt, int slot) {
#pragma unroll
    for (int j = 0; j < NB; ++j) wreg[slot][j] = *(const u32x4 *)(wptr[j] + (size_t)kt * wstep);
    if constexpr (AMODE == A_PLAIN) {
      areg[slot] = *(const u32x4 *)(aptr + kt * SBK);
    } else if constexpr (AMODE == A_CONV3) {
      const int kk = kt * SBK + ch * 8;          // chunks never straddle taps: C % 8 == 0
      const int tap = kk / p.C;
      const bool ok = (kk < 3 * p.C) && !((tap == 0) && (flags & 1)) && !((tap == 2) && (flags & 2));
      u32x4 v = {0u, 0u, 0u, 0u};
      if (ok) v = *(const u32x4 *)(aptr + kt * SBK);
      areg[slot] = v;
    } else {
      xreg[slot][0] = *(const f32x4 *)(xptr + kt * SBK);
      xreg[slot][1] = *(const f32x4 *)(xptr + kt * SBK + 4);
    }
  };
  auto commit = [&](int kt, int slot) {          // registers -> LDS stage kt % NS
    unsigned char *dA = sA[kt & (NS - 1)] + lds_off, *dW = sW[kt & (NS - 1)] + lds_off;
#pragma unroll
    for (int j = 0; j < NB; ++j) *(u32x4 *)(dW + j * SBN * 128) = wreg[slot][j];
    if constexpr (AMODE == A_LN) {
      const int k = kt * SBK + ch * 8;
      const f32x4 g0 = *(const f32x4 *)&sGain[k], g1 = *(const f32x4 *)&sGain[k + 4];
      const f32x4 b0 = *(const f32x4 *)&sShift[k], b1 = *(const f32x4 *)&sShift[k + 4];
      f32x4 y0, y1;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        y0[e] = (xreg[slot][0][e] - mu) * rstd * g0[e] + b0[e];
        y1[e] = (xreg[slot][1][e] - mu) * rstd * g1[e] + b1[e];
      }
      const bf16x4 c0 = to_bf16x4(y0), c1 = to_bf16x4(y1);
      *(bf16x8 *)dA = __builtin_shufflevector(c0, c1, 0, 1, 2, 3, 4, 5, 6, 7);
    } else {
      *(u32x4 *)dA = areg[slot];
    }
  };

  f32x16 acc[NB];
#pragma unroll
  for (int j = 0; j < NB; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[j][i] = 0.0f;
#pragma unroll
  for (int d = 0; d < DEPTH; ++d)
    if (d < nk) request(d, d);
  // ---- A_LN: statistics of the tile's 32 rows (after the first operand requests, so that their latencies overlap).
  // Eight threads per row, each over every eighth 32-byte piece, eight pieces requested at a time.
  if constexpr (AMODE == A_LN) {
    for (int k = tid * 4; k < p.K; k += 1024) {   // gain and shift of the whole row -> LDS (a load per K step would sit
      *(f32x4 *)&sGain[k] = *(const f32x4 *)(p.ln_g + k);   // on the critical path of every step)
      *(f32x4 *)&sShift[k] = *(const f32x4 *)(p.ln_b + k);
    }
    const float *xr = (const float *)p.A + (size_t)row * p.lda;
    const float pivot = xr[0];
    float s1 = 0.0f, s2 = 0.0f;
    for (int k0 = ch * 8; k0 < p.K; k0 += 512) {
      f32x4 a[8], b[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int k = min(k0 + i * 64, p.K - 8);         // past the end: a valid address, the values are not used
        a[i] = *(const f32x4 *)(xr + k);
        b[i] = *(const f32x4 *)(xr + k + 4);
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        if (k0 + i * 64 < p.K) {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float da = a[i][e] - pivot, db = b[i][e] - pivot;
            s1 += da + db;
            s2 += da * da + db * db;
          }
        }
      }
    }
#pragma unroll
    for (int off = 4; off > 0; off >>= 1) {     // the eight threads of a row are neighbouring lanes
      s1 += __shfl_xor(s1, off);
      s2 += __shfl_xor(s2, off);
    }
    const float inv_k = 1.0f / (float)p.K;
    const float ms = s1 * inv_k;                 // mean - pivot
    const float var = fmaxf(s2 * inv_k - ms * ms, 0.0f);
    mu = pivot + ms;
    rstd = rsqrtf(var + p.ln_eps);
    __syncthreads();                             // gain / shift are in LDS
  }
  // fragment of wave `wave`: row l32, k slice 16 * wave + 8 * lg .. + 7 = chunk 2 * wave + lg
  const int frag_off = l32 * 128 + (((2 * wave + lg) ^ ((l32 >> 1) & 7)) << 4);
  // SPB K steps per barrier: they are written to their stages, their register slots are refilled with the steps
  // DEPTH further on, and after one barrier all of them are multiplied.  The group after the next one reuses these
  // stages; a wave gets there only through the next barrier, which every wave reaches after its reads of this group.
  auto multiply = [&](int kt) {
    const bf16x8 xf = *(const bf16x8 *)(sA[kt & (NS - 1)] + frag_off);
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      const bf16x8 wf = *(const bf16x8 *)(sW[kt & (NS - 1)] + j * SBN * 128 + frag_off);
      acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf, xf, acc[j], 0, 0, 0);
    }
  };
  static_assert(DEPTH % SPB == 0, "the ring is walked SPB slots at a time");
  for (int kt0 = 0; kt0 < nk; kt0 += DEPTH) {
#pragma unroll
    for (int d = 0; d < DEPTH; d += SPB) {       // unrolled by the ring depth: register slots are compile-time
      const int kt = kt0 + d;
      if (kt < nk) {
#pragma unroll
        for (int q = 0; q < SPB; ++q)
          if (kt + q < nk) commit(kt + q, d + q);
#pragma unroll
        for (int q = 0; q < SPB; ++q)
          if (kt + q + DEPTH < nk) request(kt + q + DEPTH, d + q);
        __syncthreads();                         // the stages of steps kt .. kt + SPB - 1 are complete
#pragma unroll
        for (int q = 0; q < SPB; ++q)
          if (kt + q < nk) multiply(kt + q);
      }
    }
  }
  __syncthreads();                               // every wave is done with the stages: the partial tiles may overwrite them

  // ---- the four k slices are added in wave order; lane holds token l32, features 8 (i / 4) + 4 lg + i % 4 of block j
#pragma unroll
  for (int j = 0; j < NB; ++j)
#pragma unroll
    for (int i = 0; i < 16; ++i) sPart[wave][l32][j * SBN + 8 * (i >> 2) + 4 * lg + (i & 3)] = acc[j][i];
  __syncthreads();
  // thread -> row er, 4 consecutive features from ec in each of the NB column blocks
  const int er = tid >> 3, m = m0 + er;
  if (m >= p.M) return;
  [[maybe_unused]] int prow = 0;
  if constexpr (EPI == EPI_BIAS_GELU_POS) prow = p.row_pos[m];
#pragma unroll
  for (int j = 0; j < NB; ++j) {
    const int ec = j * SBN + (tid & 7) * 4;
    f32x4 v = *(const f32x4 *)&sPart[0][er][ec];
#pragma unroll
    for (int w = 1; w < 4; ++w) {
      const f32x4 t = *(const f32x4 *)&sPart[w][er][ec];
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] += t[e];
    }
    const int nn = n0 + ec;
    const f32x4 b = *(const f32x4 *)(p.bias + nn);
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] += b[e];
    if constexpr (EPI == EPI_BIAS) {
      __bf16 *dst = (p.out2 && nn >= p.n_split) ? (__bf16 *)p.out2 + (size_t)m * p.ldo2 + (nn - p.n_split)
                                                 : (__bf16 *)p.out + (size_t)m * p.ldo + nn;
      *(bf16x4 *)dst = to_bf16x4(v);
    } else if constexpr (EPI == EPI_BIAS_GELU) {
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = gelu_fast(v[e]);
      *(bf16x4 *)((__bf16 *)p.out + (size_t)m * p.ldo + nn) = to_bf16x4(v);
    } else if constexpr (EPI == EPI_BIAS_RESID) {
      f32x4 *o = (f32x4 *)((float *)p.out + (size_t)m * p.ldo + nn);
      const f32x4 x = *o;
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] += x[e];
      *o = v;
    } else if constexpr (EPI == EPI_BIAS_F32) {
      *(f32x4 *)((float *)p.out + (size_t)m * p.ldo + nn) = v;
    } else {
      const f32x4 pe = *(const f32x4 *)(p.pos + (size_t)prow * p.N + nn);
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = gelu_fast(v[e]) + pe[e];
      *(f32x4 *)((float *)p.out + (size_t)m * p.ldo + nn) = v;
    }
  }
}

// Widest tile (in 32-column blocks) that divides N and still leaves at least 160 workgroups; 1 if even that gives fewer.
int pick_blocks(const GemmArgs &a) {
  constexpr int min_wgs = 160;     // measured: 425 tokens prefer 168-224 wide tiles to 336-448 narrower ones, 125 tokens 192-256 to 96-128
  const long rows = (a.M + SBM - 1) / SBM;
  for (int nb = 4; nb > 1; nb >>= 1)
    if (a.N % (nb * SBN) == 0 && rows * (a.N / (nb * SBN)) >= min_wgs) return nb;
  return 1;
}

template <int AMODE, int EPI>
hipError_t launch_small(const GemmArgs &a, hipStream_t s) {
  const int nb = pick_blocks(a);
  const dim3 grid((unsigned)((long)((a.M + SBM - 1) / SBM) * (a.N / (nb * SBN)))), block(256);
  if (nb == 4) hipLaunchKernelGGL((gemm_small_kernel<AMODE, EPI, 4>), grid, block, 0, s, a);
  else if (nb == 2) hipLaunchKernelGGL((gemm_small_kernel<AMODE, EPI, 2>), grid, block, 0, s, a);
  else hipLaunchKernelGGL((gemm_small_kernel<AMODE, EPI, 1>), grid, block, 0, s, a);
  return hipGetLastError();
}

}  // namespace

bool gemm_small_applies(int32_t M) { return M <= 1024; }

hipError_t launch_gemm_small(const GemmArgs &a, AMode amode, Epilogue epi, hipStream_t s) {
  if (a.M <= 0) return hipSuccess;
  if (a.N % SBN != 0 || a.K % SBK != 0 || a.K <= 0 || a.a_panels || a.out_panels) return hipErrorInvalidValue;
  if (a.out2 && (epi != EPI_BIAS || a.n_split % 4 != 0 || a.n_split <= 0 || a.n_split >= a.N)) return hipErrorInvalidValue;
  if (amode == A_PLAIN) {
    if (a.lda % 8 != 0) return hipErrorInvalidValue;
    switch (epi) {
      case EPI_BIAS: return launch_small<A_PLAIN, EPI_BIAS>(a, s);
      case EPI_BIAS_GELU: return launch_small<A_PLAIN, EPI_BIAS_GELU>(a, s);
      case EPI_BIAS_RESID: return launch_small<A_PLAIN, EPI_BIAS_RESID>(a, s);
      case EPI_BIAS_F32: return launch_small<A_PLAIN, EPI_BIAS_F32>(a, s);
      default: return hipErrorInvalidValue;
    }
  }
  if (amode == A_LN) {
    if (a.lda % 8 != 0 || !a.ln_g || !a.ln_b || !(a.ln_eps > 0.0f) || a.K > kMaxLnK) return hipErrorInvalidValue;
    switch (epi) {
      case EPI_BIAS: return launch_small<A_LN, EPI_BIAS>(a, s);
      case EPI_BIAS_GELU: return launch_small<A_LN, EPI_BIAS_GELU>(a, s);
      default: return hipErrorInvalidValue;
    }
  }
  if (a.C % 8 != 0 || 3 * a.C > a.K || !a.row_src || !a.row_flags) return hipErrorInvalidValue;
  switch (epi) {
    case EPI_BIAS_GELU: return launch_small<A_CONV3, EPI_BIAS_GELU>(a, s);
    case EPI_BIAS_GELU_POS:
      if (!a.pos || !a.row_pos) return hipErrorInvalidValue;
      return launch_small<A_CONV3, EPI_BIAS_GELU_POS>(a, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace wf
