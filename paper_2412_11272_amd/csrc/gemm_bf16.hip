// bf16 MFMA GEMMs for gfx950:  out = epilogue(A . W^T),  A [M, K] activations, W [N, K] weights, fp32
// accumulation.  launch_gemm_bf16 sends batches of up to about a thousand rows to the small-batch kernel of
// gemm_small.hip (latency-bound regime, LayerNorm fused into the operand); everything else runs here.  Two kernels
// share the tiling:
//
//   gemm_bf16_dl_kernel   (v_mfma_f32_16x16x32_bf16) the projections of a transformer block (QKV, out, fc1,
//                         fc2) and, when a tap is a whole number of K steps, the two convolutions of the
//                         stem.  Operand tiles go global -> LDS directly (global_load_lds_dwordx4),
//                         fragments are double-buffered in registers, the epilogue is transposed through
//                         LDS so that stores cover whole row segments.
//   gemm_bf16_kernel      (v_mfma_f32_32x32x16_bf16) the remaining convolution shapes: a width-3 convolution
//                         over a packed time-major matrix is a GEMM whose A row is the contiguous window
//                         of three frames, with the first / last tap zeroed at stream boundaries.  Here
//                         the masking is done in registers, so tiles go global -> registers -> LDS.
//
// Tiling: one workgroup computes a BM x BN tile and advances K by 64 through two LDS stages per operand
// (three for the activations of the row-major residual projections on 256-row tiles, which then run two steps
// ahead; four for both operands of a 128 x 128 launch with at most one tile per CU); each wave owns a
// (BM/WM) x (BN/WN) sub-tile.  Tiles: 320 x 256 or 256 x 256 on 8 waves for large batches (these kernels are
// bound by the operand lines they pull through L1, and 320 x 256 is the largest tile whose accumulators and
// fragments fit 256 registers: 576 lines per K step instead of 640 for the same work), 128 x 128 on 4 waves,
// two workgroups per CU, below that.  The weight fragment is the MFMA's first operand and the activation
// fragment the second, so a lane ends up holding four consecutive output features of one token.
// LDS rows are 128 bytes (64 bf16); the 16-byte chunk index is XOR-ed with (row >> 1) & 7.  The LDS
// has 64 four-byte banks and serves a 16-byte-per-lane read 16 lanes at a time, so the 16 rows a
// group of lanes touches must land on 16 distinct 16-byte bank groups: rows of equal parity share
// the 128-byte half, and (row >> 1) & 7 gives them 8 distinct chunk positions (measured: 209 B/clk
// per CU with this swizzle, 128 with XOR by row & 7, 32 with none).
//
// Workgroup -> tile: consecutive workgroup ids go to different XCDs (each with its own 4 MB L2), and every
// XCD gets a contiguous run of the tile order.  When a row of tiles is long (N >= 8 tiles) the order walks
// column groups of 4 tile columns, rows inside a group: the 32 tiles an XCD works on at a time then share 4
// weight panels and 8 activation panels instead of a whole row of weight panels, which cuts the L2 fill
// traffic (the dominant off-chip energy of these kernels on a power-limited part) by more than half:
// fc1 -7 %, QKV -2..-6 %.  Short rows (the 5 tile columns of the d x d and d x f projections) stay row-major.
#include <mutex>

#include "device_utils.h"
#include "kernels.h"

namespace wf {

namespace {

constexpr int BK = 64;

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// Global -> registers for one 64-wide K step of the tile (fully unrolled, values stay in VGPRs).
template <int XCH, int WCH, int NT, int AMODE>
__device__ __forceinline__ void load_tile(u32x4 (&xr)[XCH], u32x4 (&wr)[WCH], const __bf16 *const (&xptr)[XCH],
                                          const int (&xflags)[XCH], const __bf16 *const (&wptr)[WCH], int k0, int C, int tid) {
#pragma unroll
  for (int i = 0; i < XCH; ++i) {
    if (AMODE == A_PLAIN) {
      xr[i] = *(const u32x4 *)(xptr[i] + k0);
    } else {
      const int kk = k0 + ((i * NT + tid) & 7) * 8;   // chunks never straddle taps: C % 8 == 0
      const int tap = kk / C;
      const bool ok = (kk < 3 * C) && !((tap == 0) && (xflags[i] & 1)) && !((tap == 2) && (xflags[i] & 2));
      u32x4 v = {0u, 0u, 0u, 0u};
      if (ok) v = *(const u32x4 *)(xptr[i] + k0);
      xr[i] = v;
    }
  }
#pragma unroll
  for (int i = 0; i < WCH; ++i) wr[i] = *(const u32x4 *)(wptr[i] + k0);
}

template <int XCH, int WCH>
__device__ __forceinline__ void store_tile(const u32x4 (&xr)[XCH], const u32x4 (&wr)[WCH], unsigned char *dx, unsigned char *dw,
                                           const int (&xlds)[XCH], const int (&wlds)[WCH]) {
#pragma unroll
  for (int i = 0; i < XCH; ++i) *(u32x4 *)(dx + xlds[i]) = xr[i];
#pragma unroll
  for (int i = 0; i < WCH; ++i) *(u32x4 *)(dw + wlds[i]) = wr[i];
}

template <int BM, int BN, int WM, int WN, int AMODE, int EPI>
__global__ void __launch_bounds__(WM * WN * 64) gemm_bf16_kernel(GemmArgs p) {
  constexpr int NT = WM * WN * 64;
  constexpr int TM = BM / WM, TN = BN / WN;
  constexpr int IM = TM / 32, IN = TN / 32;
  constexpr int XCH = BM * 8 / NT;   // 16-byte chunks of the activation tile per thread
  constexpr int WCH = BN * 8 / NT;
  static_assert(BM * 8 % NT == 0 && BN * 8 % NT == 0, "tile/threads mismatch");

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char *sX = smem;                        // [2][BM][128 B]
  unsigned char *sW = smem + 2 * BM * 128;         // [2][BN][128 B]

  const int tiles_m = (p.M + BM - 1) / BM;
  const int tiles_n = p.N / BN;
  const int n_tiles = tiles_m * tiles_n;
  const int per_xcd = (n_tiles + 7) >> 3;
  const int tile = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);   // XCD x runs tiles [x*per_xcd, (x+1)*per_xcd)
  if (tile >= n_tiles) return;
  const int m0 = (tile / tiles_n) * BM;
  const int n0 = (tile % tiles_n) * BN;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int l32 = lane & 31, lg = lane >> 5;

  // ---- per-thread load descriptors (fixed over the K loop) ----
  const __bf16 *A = (const __bf16 *)p.A;
  const __bf16 *W = (const __bf16 *)p.W;
  const __bf16 *xptr[XCH];
  int xflags[XCH];
  int xlds[XCH];
#pragma unroll
  for (int i = 0; i < XCH; ++i) {
    const int c = i * NT + tid;
    const int r = c >> 3, ch = c & 7;
    int row = m0 + r;
    row = row < p.M ? row : p.M - 1;              // rows past M are computed but never stored
    if (AMODE == A_PLAIN) {
      xptr[i] = A + (size_t)row * p.lda + ch * 8;
      xflags[i] = 0;
    } else {
      xptr[i] = A + (long)p.row_src[row] * p.C + ch * 8;
      xflags[i] = p.row_flags[row];
    }
    xlds[i] = r * 128 + ((ch ^ ((r >> 1) & 7)) << 4);
  }
  const __bf16 *wptr[WCH];
  int wlds[WCH];
#pragma unroll
  for (int i = 0; i < WCH; ++i) {
    const int c = i * NT + tid;
    const int r = c >> 3, ch = c & 7;
    wptr[i] = W + (size_t)(n0 + r) * p.K + ch * 8;
    wlds[i] = r * 128 + ((ch ^ ((r >> 1) & 7)) << 4);
  }

  u32x4 xr[XCH], wr[WCH];
  f32x16 acc[IM][IN];
#pragma unroll
  for (int i = 0; i < IM; ++i)
#pragma unroll
    for (int j = 0; j < IN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  const int nk = p.K / BK;
  load_tile<XCH, WCH, NT, AMODE>(xr, wr, xptr, xflags, wptr, 0, p.C, tid);
  store_tile<XCH, WCH>(xr, wr, sX, sW, xlds, wlds);
  __syncthreads();

  // fragment read offsets: lane reads row (l32) of a 32-row group, chunk 2*ks + lg (swizzled)
  const int xrow0 = (wm * TM + l32) * 128;
  const int wrow0 = (wn * TN + l32) * 128;
  const int sw = (l32 >> 1) & 7;

  for (int kt = 0; kt < nk; ++kt) {
    const int stage = kt & 1;
    if (kt + 1 < nk) load_tile<XCH, WCH, NT, AMODE>(xr, wr, xptr, xflags, wptr, (kt + 1) * BK, p.C, tid);
    const unsigned char *cx = sX + stage * BM * 128 + xrow0;
    const unsigned char *cw = sW + stage * BN * 128 + wrow0;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int choff = ((2 * ks + lg) ^ sw) << 4;
      bf16x8 wf[IN], xf[IM];
#pragma unroll
      for (int j = 0; j < IN; ++j) wf[j] = *(const bf16x8 *)(cw + j * 32 * 128 + choff);
#pragma unroll
      for (int i = 0; i < IM; ++i) xf[i] = *(const bf16x8 *)(cx + i * 32 * 128 + choff);
#pragma unroll
      for (int i = 0; i < IM; ++i)
#pragma unroll
        for (int j = 0; j < IN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[j], xf[i], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) store_tile<XCH, WCH>(xr, wr, sX + (stage ^ 1) * BM * 128, sW + (stage ^ 1) * BN * 128, xlds, wlds);
    __syncthreads();
  }

  // ---- epilogue: lane holds, per 32x32 block, token m = l32 and features 8*g + 4*lg + (0..3), g = 0..3
#pragma unroll
  for (int i = 0; i < IM; ++i) {
    const int m = m0 + wm * TM + i * 32 + l32;
    if (m >= p.M) continue;
    int prow = 0;
    if (EPI == EPI_BIAS_GELU_POS) prow = p.row_pos[m];
#pragma unroll
    for (int j = 0; j < IN; ++j) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int n = n0 + wn * TN + j * 32 + g * 8 + lg * 4;
        const f32x4 b = *(const f32x4 *)(p.bias + n);
        f32x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = acc[i][j][g * 4 + e] + b[e];
        if (EPI == EPI_BIAS) {
          *(bf16x4 *)((__bf16 *)p.out + (size_t)m * p.ldo + n) = to_bf16x4(v);
        } else if (EPI == EPI_BIAS_GELU) {
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = gelu_fast(v[e]);
          *(bf16x4 *)((__bf16 *)p.out + (size_t)m * p.ldo + n) = to_bf16x4(v);
        } else if (EPI == EPI_BIAS_RESID) {
          f32x4 *o = (f32x4 *)((float *)p.out + (size_t)m * p.ldo + n);
          const f32x4 x = *o;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] += x[e];
          *o = v;
        } else {
          const f32x4 pe = *(const f32x4 *)(p.pos + (size_t)prow * p.N + n);
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = gelu_fast(v[e]) + pe[e];
          *(f32x4 *)((float *)p.out + (size_t)m * p.ldo + n) = v;
        }
      }
    }
  }
}

template <int BM, int BN, int WM, int WN, int AMODE, int EPI>
hipError_t launch_cfg(const GemmArgs &a, hipStream_t s) {
  constexpr int smem = 2 * (BM + BN) * 128;
  auto kern = gemm_bf16_kernel<BM, BN, WM, WN, AMODE, EPI>;
  static std::once_flag once;          // raised LDS limit: set once per process, by whichever thread gets here first
  static hipError_t attr_err = hipSuccess;
  std::call_once(once, [&] { attr_err = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, smem); });
  if (attr_err != hipSuccess) return attr_err;
  // one workgroup per tile, rounded up to whole groups of 8 (XCD x takes tiles [x*per_xcd, (x+1)*per_xcd); the
  // kernel drops the workgroups past the last tile)
  const int tiles = ((a.M + BM - 1) / BM) * (a.N / BN);
  const int grid = 8 * ((tiles + 7) / 8);
  hipLaunchKernelGGL(kern, dim3(grid), dim3(WM * WN * 64), smem, s, a);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Variant with direct global -> LDS loads (no VGPR staging) and register double-buffering of the
// MFMA fragments.  global_load_lds_dwordx4 writes lane l's 16 bytes at LDS base + 16*l, so a wave
// fills 8 consecutive 128-byte rows per instruction; the XOR swizzle is applied by choosing which
// global chunk each lane fetches (lane l of a row group fetches chunk (l & 7) ^ (l >> 3)).
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) void glb_void;

// Zero source for the masked taps of the convolution operand (device code takes its address directly).
__device__ __attribute__((aligned(16))) unsigned int g_zero16[4];

// One BM x BN output tile at (m0, n0), computed by the whole workgroup.  SMEM: bytes of LDS the kernel owns;
// NT: streaming stores for bf16 results; AMODE: plain or gathered convolution operand; DEEP: 3 = four LDS stages
// for both operands, requested three K steps ahead (for launches of at most one tile per CU); else which operand
// gets a third LDS stage and a prefetch distance of two K steps (0 none, 1 activations, 2 weights).
template <int BM, int BN, int WM, int WN, int EPI, int SMEM, bool NT, int AMODE, int DEEP>
__device__ __forceinline__ void dl_tile(const GemmArgs &p, unsigned char *smem, int m0, int n0) {
  constexpr int NW = WM * WN;
  constexpr int TM = BM / WM, TN = BN / WN;
  constexpr int XL = BM / 8 / NW;    // load instructions per wave for the activation tile (8 rows each)
  constexpr int WL = BN / 8 / NW;
  static_assert(BM % (8 * NW) == 0 && BN % (8 * NW) == 0 && TN % 32 == 0, "tile/waves mismatch");

  constexpr int XS = DEEP == 3 ? 4 : (DEEP == 1 ? 3 : 2), WS = DEEP == 3 ? 4 : (DEEP == 2 ? 3 : 2);   // LDS stages per operand
  unsigned char *sX = smem;                        // [XS][BM][128 B]
  unsigned char *sW = smem + XS * BM * 128;        // [WS][BN][128 B]

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;

  // lane -> row within the 8-row group written by one load instruction; the chunk it fetches is the
  // one that belongs at its LDS slot: (lane & 7) ^ swizzle(row)
  const int lrow = lane >> 3;
  const __bf16 *A = (const __bf16 *)p.A;
  const __bf16 *W = (const __bf16 *)p.W;
  // Plain operands are addressed as a uniform base plus a 32-bit byte offset per lane (half the registers of a
  // pointer per load instruction; the launcher keeps such operands under 4 GiB); the gathered convolution
  // operand keeps full pointers, since a masked tap redirects the whole address.
  constexpr bool OFFS = AMODE != A_CONV3;
  const __bf16 *xptr[OFFS ? 1 : XL];
  unsigned xoff[OFFS ? XL : 1], woff[WL];
  [[maybe_unused]] int xflags[XL];      // A_CONV3: bit 0 = first tap lies before the stream, bit 1 = last tap lies after it
#pragma unroll
  for (int i = 0; i < XL; ++i) {
    const int rt = (i * NW + wave) * 8 + lrow;
    const int lch = (lane & 7) ^ ((rt >> 1) & 7);
    int row = m0 + rt;
    row = row < p.M ? row : p.M - 1;              // rows past M are computed but never stored
    if constexpr (AMODE == A_CONV3) {
      // row = window of 3*C elements starting at frame row_src[row]; C % 64 == 0, so a K step lies in one tap
      xptr[i] = A + (long)p.row_src[row] * p.C + lch * 8;
      xflags[i] = p.row_flags[row];
    } else {
      xoff[i] = 2u * (p.a_panels ? (((unsigned)(row >> 8) * (unsigned)(p.K >> 6)) << 14) + ((row & 255) << 6) + lch * 8   // panel layout
                                 : (unsigned)row * (unsigned)p.lda + lch * 8);
    }
  }
#pragma unroll
  for (int i = 0; i < WL; ++i) {
    const int rt = (i * NW + wave) * 8 + lrow;
    const int lch = (lane & 7) ^ ((rt >> 1) & 7);
    const int n = n0 + rt;
    woff[i] = 2u * (p.w_panels ? (((unsigned)(n >> 8) * (unsigned)(p.K >> 6)) << 14) + ((n & 255) << 6) + lch * 8
                               : (unsigned)n * (unsigned)p.K + lch * 8);
  }

  [[maybe_unused]] const int kpt = AMODE == A_CONV3 ? p.C / BK : 0;     // K steps per tap
  auto issue_x = [&](int kt, int slot) {            // activation tile of K step kt into ring slot `slot` (= kt % 3)
    const int k0 = kt * BK;
    const int ka = p.a_panels ? kt << 14 : k0;     // panel layout: the next 64-column chunk is 256 * 64 elements on
    // A_CONV3: K steps [0, kpt) are tap 0, [2 kpt, 3 kpt) tap 2; the flag bit that zeroes this step's tap
    const int dead = AMODE == A_CONV3 ? (kt < kpt ? 1 : (kt >= 2 * kpt ? 2 : 0)) : 0;
    // the K offset goes into the 32-bit lane offset, so that the address stays "uniform base + zero-extended
    // 32-bit offset" inside the loop and the load takes the scalar-base form (one address register per load)
    const unsigned kb = 2u * (unsigned)ka;
#pragma unroll
    for (int i = 0; i < XL; ++i) {
      const void *src;
      if constexpr (AMODE == A_CONV3) src = (xflags[i] & dead) ? (const void *)g_zero16 : (const void *)(xptr[i] + ka);
      else src = (const unsigned char *)A + (unsigned)(xoff[i] + kb);
      __builtin_amdgcn_global_load_lds((const glb_void *)src,
                                       (lds_void *)(sX + slot * BM * 128 + (i * NW + wave) * 1024), 16, 0, 0);
    }
  };
  auto issue_w = [&](int kt, int slot) {
    const int kw = p.w_panels ? kt << 14 : kt * BK;
    const unsigned kb = 2u * (unsigned)kw;
#pragma unroll
    for (int i = 0; i < WL; ++i)
      __builtin_amdgcn_global_load_lds((const glb_void *)((const unsigned char *)W + (unsigned)(woff[i] + kb)),
                                       (lds_void *)(sW + slot * BN * 128 + (i * NW + wave) * 1024), 16, 0, 0);
  };

  // Accumulators: v_mfma_f32_16x16x32_bf16 blocks, TB token blocks x FB feature blocks of 16 x 16.  With
  // the weight fragment as first operand a lane holds, per block, token (lane % 16) and features
  // 4 * (lane / 16) + (0..3).  (This instruction shape does the same work per cycle as the 32x32x16 one but
  // draws less power: on random operands a register-only loop sustains 1.97 against 1.76 PFLOP/s.)
  constexpr int TB = TM / 16, FB = TN / 16, FBH = FB / 2;
  static_assert(TM % 16 == 0 && TN % 32 == 0, "wave tile must be a multiple of 16 x 32");
  // The accumulators start from the bias (a lane's four values of a block are four consecutive features), so the
  // epilogue has no bias add left.
  f32x4 acc[TB][FB];
#pragma unroll
  for (int j = 0; j < FB; ++j) {
    const f32x4 b = *(const f32x4 *)(p.bias + n0 + wn * TN + j * 16 + (lane >> 4) * 4);
#pragma unroll
    for (int i = 0; i < TB; ++i) acc[i][j] = b;
  }

  const int nk = p.K / BK;
  const int l16 = lane & 15, lq = lane >> 4;       // row inside a 16-row block; which 8 of the 32 reduction indices
  const int xrow0 = (wm * TM + l16) * 128;
  const int wrow0 = (wn * TN + l16) * 128;
  const int sw = (l16 >> 1) & 7;

  // Main loop.  A 64-deep LDS stage is two reduction steps of 32 (t = 0, 1); each step is split into the
  // lower and the upper half of the wave's feature blocks, so that a sub-step is TB*FBH MFMAs on one set of
  // activation fragments (xf) and one set of weight fragments (wlo / whi).  Fragments are prefetched one
  // sub-step ahead: under the MFMAs of (t, lo) the upper weight fragments of step t are read, under those
  // of (t, hi) the activation and lower weight fragments of step t+1.  The one barrier per stage sits right
  // after the LAST fragment read of the current stage: at that point (a) every wave has finished reading
  // this stage, so the loads of tile kt+2 may overwrite it, and (b) every wave has seen its own loads of
  // tile kt+1 land, so its first fragments can be read under the MFMAs of the last sub-step -- the matrix
  // pipe never drains at the barrier.  The two waves that share a SIMD issue their global loads at
  // different points (before / after those MFMAs), so one keeps the matrix pipe busy while the other is
  // held up handing loads to the memory pipeline.
  const bool early = (wave < NW / 2) || NW < 8;
  bf16x8 xf[2][TB], wlo[FBH], whi[FBH];
  auto rd_x = [&](int slot, int t, int buf) {
    const unsigned char *cx = sX + slot * BM * 128 + xrow0 + (((4 * t + lq) ^ sw) << 4);
#pragma unroll
    for (int i = 0; i < TB; ++i) xf[buf][i] = *(const bf16x8 *)(cx + i * 16 * 128);
  };
  auto rd_w = [&](int slot, int t, int half, bf16x8 (&dst)[FBH]) {
    const unsigned char *cw = sW + slot * BN * 128 + wrow0 + half * FBH * 16 * 128 + (((4 * t + lq) ^ sw) << 4);
#pragma unroll
    for (int j = 0; j < FBH; ++j) dst[j] = *(const bf16x8 *)(cw + j * 16 * 128);
  };
  auto mm = [&](int half, const bf16x8 (&w)[FBH], int buf) {
#pragma unroll
    for (int i = 0; i < TB; ++i)
#pragma unroll
      for (int j = 0; j < FBH; ++j)
        acc[i][half * FBH + j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[j], xf[buf][i], acc[i][half * FBH + j], 0, 0, 0);
  };
  // Scheduling hint for a sub-step with NRD fragment reads: alternate one MFMA with one LDS read, then the
  // remaining MFMAs -- the issue slots of the reads hide under the matrix pipe's occupancy.
#define WF_SCHED(NRD)                                                                                  \
  _Pragma("unroll") for (int q_ = 0; q_ < (NRD); ++q_) {                                              \
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                                \
    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                                \
  }                                                                                                   \
  __builtin_amdgcn_sched_group_barrier(0x008, (TB * FBH > (NRD) ? TB * FBH - (NRD) : 0), 0);          \
  __builtin_amdgcn_sched_barrier(0)

  // Operand pipeline.  Each operand has two LDS stages and is requested one K step ahead; with DEEP one of
  // them has three stages and is requested two steps ahead (the activations of a row-major tile order come
  // from further away than the weights, which stay in L2).  The deep operand is issued last: at the end of
  // step kt a wave has then issued ... shallow(kt+1), deep(kt+2) as its newest loads, and since vector-memory
  // operations complete in order, waiting until at most the loads of deep(kt+2) are outstanding means
  // everything step kt+1 reads has landed.  Slots: stage kt % 2, or kt % 3 for the deep operand.
  // DEEP == 3 (a launch of at most one tile per CU, where nothing but the tile's own requests hides the latency of
  // its operands): four stages for both, slot kt % 4; after the barrier that ends step kt the loads of step kt+4 go
  // into the slot just read, and the wait before that barrier lets the loads of steps kt+2 and kt+3 stay in flight.
  constexpr int NDEEP = DEEP == 1 ? XL : (DEEP == 2 ? WL : 0);       // load instructions of one deep tile
  constexpr int LPS = XL + WL;                                       // load instructions of one K step
  auto issue_next = [&](int kt, int s2, int s3) {    // after the barrier that ends step kt (s2 = kt % 2, s3 = kt % 3)
    if (DEEP == 3) {
      if (kt + 4 < nk) { issue_x(kt + 4, kt & 3); issue_w(kt + 4, kt & 3); }
    } else if (DEEP == 0) {
      if (kt + 2 < nk) { issue_x(kt + 2, s2); issue_w(kt + 2, s2); }
    } else if (DEEP == 1) {
      if (kt + 2 < nk) issue_w(kt + 2, s2);
      if (kt + 3 < nk) issue_x(kt + 3, s3);
    } else {
      if (kt + 2 < nk) issue_x(kt + 2, s2);
      if (kt + 3 < nk) issue_w(kt + 3, s3);
    }
  };
  issue_x(0, 0);
  issue_w(0, 0);
  __builtin_amdgcn_s_waitcnt(0x0F70);              // vmcnt(0)
  __builtin_amdgcn_s_barrier();
  if (1 < nk) { issue_x(1, 1); issue_w(1, 1); }
  if (DEEP == 1 && 2 < nk) issue_x(2, 2);
  if (DEEP == 2 && 2 < nk) issue_w(2, 2);
  if (DEEP == 3) {
    if (2 < nk) { issue_x(2, 2); issue_w(2, 2); }
    if (3 < nk) { issue_x(3, 3); issue_w(3, 3); }
  }
  rd_x(0, 0, 0);
  rd_w(0, 0, 0, wlo);
  int s3 = 0;                                      // kt % 3
  for (int kt = 0; kt < nk; ++kt) {
    const int s2 = kt & 1;
    const int s3n = s3 == 2 ? 0 : s3 + 1;
    const int xs = DEEP == 3 ? (kt & 3) : (DEEP == 1 ? s3 : s2), xs1 = DEEP == 3 ? ((kt + 1) & 3) : (DEEP == 1 ? s3n : s2 ^ 1);   // activation slots of steps kt, kt+1
    const int ws = DEEP == 3 ? (kt & 3) : (DEEP == 2 ? s3 : s2), ws1 = DEEP == 3 ? ((kt + 1) & 3) : (DEEP == 2 ? s3n : s2 ^ 1);   // weight slots
    __builtin_amdgcn_sched_barrier(0);
    // (t = 0, lo): read the upper weight fragments of step 0
    __builtin_amdgcn_s_waitcnt(0xC07F);            // lgkmcnt(0), placed BEFORE the next reads so it only waits for older ones
    __builtin_amdgcn_sched_barrier(0);
    rd_w(ws, 0, 1, whi);
    mm(0, wlo, 0);
    WF_SCHED(FBH);
    // (t = 0, hi): read the activation and lower weight fragments of step 1
    __builtin_amdgcn_s_waitcnt(0xC07F);
    __builtin_amdgcn_sched_barrier(0);
    rd_x(xs, 1, 1);
    rd_w(ws, 1, 0, wlo);
    mm(1, whi, 0);
    WF_SCHED(TB + FBH);
    // (t = 1, lo): read the upper weight fragments of step 1
    __builtin_amdgcn_s_waitcnt(0xC07F);
    __builtin_amdgcn_sched_barrier(0);
    rd_w(ws, 1, 1, whi);
    mm(0, wlo, 1);
    WF_SCHED(FBH);
    // this step's stages fully read; my part of the tiles of step kt+1 landed (deep(kt+2) may still be in flight)
    if (DEEP == 3) {                                  // loads of steps kt+2 and kt+3, as far as they exist, may stay in flight
      constexpr int W2 = 2 * LPS, W1 = LPS;           // vmcnt: bits 3:0 and 15:14 of the immediate
      if (kt + 3 < nk) __builtin_amdgcn_s_waitcnt(0x0070 | (W2 & 15) | ((W2 >> 4) << 14));
      else if (kt + 2 < nk) __builtin_amdgcn_s_waitcnt(0x0070 | (W1 & 15) | ((W1 >> 4) << 14));
      else __builtin_amdgcn_s_waitcnt(0x0070);
    } else if (DEEP != 0 && kt + 2 < nk) __builtin_amdgcn_s_waitcnt(0x0070 | NDEEP);   // vmcnt(NDEEP) lgkmcnt(0)
    else __builtin_amdgcn_s_waitcnt(0x0070);                                    // vmcnt(0) lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    if (early) issue_next(kt, s2, s3);
    __builtin_amdgcn_sched_barrier(0);
    if (kt + 1 < nk) {
      rd_x(xs1, 0, 0);
      rd_w(ws1, 0, 0, wlo);
    }
    __builtin_amdgcn_sched_barrier(0);
    mm(1, whi, 1);                                 // (t = 1, hi)
    __builtin_amdgcn_sched_barrier(0);
    if (!early) issue_next(kt, s2, s3);
    __builtin_amdgcn_sched_barrier(0);
    s3 = s3n;
  }
#undef WF_SCHED

  // ---- epilogue.  The accumulator layout gives a lane 4 consecutive features of ONE token, which would
  // make every store instruction touch 16 different rows.  Each wave therefore transposes its sub-tile
  // through its own 16 KB slice of the (now idle) LDS stages and writes whole 128/256-byte row
  // segments: 16-byte chunk c of row r sits at chunk position c ^ (r & (CPR-1)).
  __builtin_amdgcn_s_waitcnt(0x0F70);
  __builtin_amdgcn_s_barrier();                    // every wave is done reading the last K step
  unsigned char *stg = smem + wave * (TM * 256);   // TM rows x 256 bytes (<= 16 KB per wave)
  static_assert(NDEEP < 16 && 2 * LPS < 64 && NW * TM * 256 <= SMEM && (XS * BM + WS * BN) * 128 <= SMEM, "staging does not fit in the LDS stages");
  const int mw0 = m0 + wm * TM, nw0 = n0 + wn * TN;
  if (EPI == EPI_BIAS || EPI == EPI_BIAS_GELU) {
    constexpr int RB = TN * 2;                     // row bytes (bf16)
    constexpr int CPR = RB / 16;                   // 16-byte chunks per row
#pragma unroll
    for (int i = 0; i < TB; ++i) {
      const int r = i * 16 + l16;
#pragma unroll
      for (int j = 0; j < FB; ++j) {
        const int nl = j * 16 + lq * 4;            // feature inside the wave's sub-tile
        f32x4 v = acc[i][j];
        if (EPI == EPI_BIAS_GELU) {
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = gelu_fast(v[e]);
        }
        const int u = nl >> 2;                     // 8-byte unit inside the row
        *(bf16x4 *)(stg + r * RB + ((((u >> 1) ^ (r & (CPR - 1))) << 4) | ((u & 1) << 3))) = to_bf16x4(v);
      }
    }
    __builtin_amdgcn_s_waitcnt(0xC07F);            // lgkmcnt(0): the wave's own LDS writes have landed
    constexpr int RPI = 64 / CPR;                  // rows per store instruction
    const int rr = lane / CPR, c = lane % CPR;
#pragma unroll
    for (int it = 0; it < TM / RPI; ++it) {
      const int r = it * RPI + rr;
      const u32x4 v = *(const u32x4 *)(stg + r * RB + ((c ^ (r & (CPR - 1))) << 4));
      const int m = mw0 + r;
      if (m < p.M) {
        const int n = nw0 + c * 8;
        __bf16 *dst = p.out_panels ? (__bf16 *)p.out + ((((size_t)(m >> 8) * (p.N >> 6) + (n >> 6)) << 14) + ((m & 255) << 6) + (n & 63))
                      : (p.out2 && n >= p.n_split) ? (__bf16 *)p.out2 + (size_t)m * p.ldo2 + (n - p.n_split)
                                                   : (__bf16 *)p.out + (size_t)m * p.ldo + n;
        // Large bf16 results (QKV, the MLP's hidden activations) are written with the non-temporal hint:
        // they are far bigger than what the caches can hand to the consumer, and written plainly they
        // push the residual stream and the operands of the next kernels out of the memory-side cache.
        if constexpr (NT) __builtin_nontemporal_store(v, (u32x4 *)dst);
        else *(u32x4 *)dst = v;
      }
    }
  } else {
    // fp32 output: residual update in place (EPI_BIAS_RESID), GELU plus position row (EPI_BIAS_GELU_POS) or
    // plain store (EPI_BIAS_F32), PW features
    // (PW * 4 bytes per row) per pass
    constexpr int PW = TN >= 64 ? 64 : TN;         // features per pass
    constexpr int RB = PW * 4, CPR = RB / 16, RPI = 64 / CPR;
    const int rr = lane / CPR, c = lane % CPR;
    // The residual values a lane will update are requested well before they are needed, so that their
    // memory latency runs under the LDS transposition (and under the previous pass) instead of once per
    // row: half of a pass's rows before its staging writes, the other half right after them (when that
    // pass's accumulators are dead), and the first half of the NEXT pass before this pass's stores.
    constexpr int NIT = TM / RPI, NPS = TN / PW;
    f32x4 res[2][NIT];
    auto fetch_res = [&](int ps, int it) {
      int m = mw0 + it * RPI + rr;
      m = m < p.M ? m : p.M - 1;
      if constexpr (EPI == EPI_BIAS_GELU_POS)      // the addend is the token's position row instead of the old output
        res[ps & 1][it] = *(const f32x4 *)(p.pos + (size_t)p.row_pos[m] * p.N + nw0 + ps * PW + c * 4);
      else
        res[ps & 1][it] = *(const f32x4 *)((const float *)p.out + (size_t)m * p.ldo + nw0 + ps * PW + c * 4);
    };
    constexpr bool ADDEND = EPI == EPI_BIAS_RESID || EPI == EPI_BIAS_GELU_POS;
    if (ADDEND) {
#pragma unroll
      for (int it = 0; it < NIT / 2; ++it) fetch_res(0, it);
    }
#pragma unroll
    for (int ps = 0; ps < NPS; ++ps) {
#pragma unroll
      for (int i = 0; i < TB; ++i) {
        const int r = i * 16 + l16;
#pragma unroll
        for (int jj = 0; jj < PW / 16; ++jj) {
          const int j = ps * (PW / 16) + jj;
          const int nl = j * 16 + lq * 4;
          f32x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = EPI == EPI_BIAS_GELU_POS ? gelu_fast(acc[i][j][e]) : acc[i][j][e];
          const int ch = (nl % PW) >> 2;           // 16-byte chunk inside the pass
          *(f32x4 *)(stg + r * RB + ((ch ^ (r & (CPR - 1))) << 4)) = v;
        }
      }
      if (ADDEND) {
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int it = NIT / 2; it < NIT; ++it) fetch_res(ps, it);
        if (ps + 1 < NPS) {
#pragma unroll
          for (int it = 0; it < NIT / 2; ++it) fetch_res(ps + 1, it);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      __builtin_amdgcn_s_waitcnt(0xC07F);
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        const int r = it * RPI + rr;
        f32x4 v = *(const f32x4 *)(stg + r * RB + ((c ^ (r & (CPR - 1))) << 4));
        const int m = mw0 + r;
        if (ADDEND) {
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] += res[ps & 1][it][e];
        }
        if (m < p.M) *(f32x4 *)((float *)p.out + (size_t)m * p.ldo + nw0 + ps * PW + c * 4) = v;
      }
      __builtin_amdgcn_s_waitcnt(0xC07F);          // reads done before the next pass overwrites the slice
    }
  }
}

// Workgroup -> work unit.  Full BM x BN tiles first (in the tile order described at the top of the file);
// when the tiles left over after the last full round of the chip would occupy at most half of it, each of
// them is split into two BM x BN/2 units so that the last round takes half as long (620 tiles on 256 CUs:
// 2.5 rounds instead of 3).  Consecutive workgroup ids go to different XCDs; XCD x gets the full tiles at
// positions [x*full_per_xcd, ...) of the order and the half units [x*half_per_xcd, ...), full tiles first.
// Host and device share these two functions, so that the launcher's grid and the kernel's decoding of a workgroup id
// cannot drift apart (and a host test can enumerate the units of any shape: every tile exactly once).
struct DlUnit { int row, col, half; };   // tile row / column; half: 0 = whole tile, 1 / 2 = its left / right BN/2 columns

// Split of tiles_m x tiles_n tiles over the chip; fills the work-unit fields of b and returns the grid size.
__host__ inline int dl_plan(GemmArgs &b, int tiles_m, int tiles_n) {
  constexpr int kCUs = 256;
  const int tiles = tiles_m * tiles_n;
  const int rest = tiles % kCUs;
  const bool split = rest > 0 && 2 * rest <= kCUs;
  b.n_full = split ? tiles - rest : tiles;
  b.n_half = split ? 2 * rest : 0;
  b.full_per_xcd = (b.n_full + 7) / 8;
  b.half_per_xcd = (b.n_half + 7) / 8;
  b.group_n = tiles_n >= 8 ? 4 : tiles_n;     // column groups only pay when a row of tiles is long
  return 8 * (b.full_per_xcd + b.half_per_xcd);
}

// Workgroup id -> unit; false for the ids that round the grid up to whole groups of 8.
__host__ __device__ inline bool dl_unit(const GemmArgs &p, int bid, int tiles_m, int tiles_n, DlUnit &u) {
  // position t of the tile order -> (row, column): column groups of G tile columns, rows inside a group,
  // columns inside a row (the last group may be narrower)
  const int G = min(max(p.group_n, 1), tiles_n);
  auto locate = [&](int t) {
    const int gs = tiles_m * G;
    const int g = t / gs, rem = t - g * gs;
    const int gw = min(G, tiles_n - g * G);
    u.row = rem / gw;
    u.col = g * G + (rem - u.row * gw);
  };
  const int xcd = bid & 7, l = bid >> 3;
  if (l < p.full_per_xcd) {
    const int tile = xcd * p.full_per_xcd + l;
    if (tile >= p.n_full) return false;
    locate(tile);
    u.half = 0;
    return true;
  }
  const int hl = l - p.full_per_xcd;
  const int h = xcd * p.half_per_xcd + hl;
  if (hl >= p.half_per_xcd || h >= p.n_half) return false;
  locate(p.n_full + (h >> 1));
  u.half = 1 + (h & 1);
  return true;
}

// LDS bytes of a direct-load kernel: its operand stages, or the epilogue's per-wave transposition slices if those are larger.
constexpr int dl_smem_bytes(int bm, int bn, int nw, int tm, int deep) {
  const int stages = deep == 3 ? 4 * (bm + bn) * 128 : (2 * (bm + bn) + (deep == 1 ? bm : (deep == 2 ? bn : 0))) * 128;
  const int slices = nw * tm * 256;
  return stages > slices ? stages : slices;
}

template <int BM, int BN, int WM, int WN, int EPI, bool NT, int AMODE, int DEEP>
__global__ void __launch_bounds__(WM * WN * 64) gemm_bf16_dl_kernel(GemmArgs p) {
  constexpr int SMEM = dl_smem_bytes(BM, BN, WM * WN, BM / WM, DEEP);
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  DlUnit u;
  if (!dl_unit(p, blockIdx.x, (p.M + BM - 1) / BM, p.N / BN, u)) return;
  if (u.half == 0) dl_tile<BM, BN, WM, WN, EPI, SMEM, NT, AMODE, DEEP>(p, smem, u.row * BM, u.col * BN);
  else dl_tile<BM, BN / 2, WM, WN, EPI, SMEM, NT, AMODE, DEEP>(p, smem, u.row * BM, u.col * BN + (u.half - 1) * (BN / 2));
}

template <int BM, int BN, int WM, int WN, int EPI, bool NT = false, int AMODE = A_PLAIN, int DEEP = 0>
hipError_t launch_dl(const GemmArgs &a, hipStream_t s) {
  constexpr int smem = dl_smem_bytes(BM, BN, WM * WN, BM / WM, DEEP);
  auto kern = gemm_bf16_dl_kernel<BM, BN, WM, WN, EPI, NT, AMODE, DEEP>;
  static std::once_flag once;
  static hipError_t attr_err = hipSuccess;
  std::call_once(once, [&] { attr_err = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, smem); });
  if (attr_err != hipSuccess) return attr_err;
  GemmArgs b = a;
  const int grid = dl_plan(b, (a.M + BM - 1) / BM, a.N / BN);
  hipLaunchKernelGGL(kern, dim3(grid), dim3(WM * WN * 64), smem, s, b);
  return hipGetLastError();
}

// Large tile when it divides N and there is enough work for it: at least 160 tiles of 256 x 256.  That leaves up to
// 96 CUs idle in the tile's only round, but a CU's tile runs faster the fewer CUs are active, and from there on the
// large tile wins or ties on every shape of the benchmark configurations (below, the 128 x 128 tile wins).
bool use_large_tile(const GemmArgs &a) {
  return (a.N % 256 == 0) && ((long)((a.M + 255) / 256) * (a.N / 256) >= 160);
}

// Rows of the large tile: 320 or 256.  The 320-row tile fetches 10 % fewer operand lines per flop (the bound of
// these kernels) and measures about 7 % faster per flop, but a product is as slow as its last round of the chip,
// so the choice goes by the estimated makespan: rounds of 256 tiles (a last round cut into half units counts
// 0.5) times the measured per-tile time ratio of 1.18.
int large_tile_rows(int M, int N) {
  auto rounds = [](long tiles) {
    const long rest = tiles % 256;
    return (double)(tiles / 256) + (rest == 0 ? 0.0 : (2 * rest <= 256 ? 0.5 : 1.0));
  };
  const double t256 = rounds((long)((M + 255) / 256) * (N / 256));
  const double t320 = 1.18 * rounds((long)((M + 319) / 320) * (N / 256));
  return t320 < t256 ? 320 : 256;
}

}  // namespace

hipError_t launch_gemm_bf16(const GemmArgs &a, AMode amode, Epilogue epi, hipStream_t s) {
  if (a.M <= 0) return hipSuccess;
  if ((gemm_small_applies(a.M) || a.prefer_small) && !a.prefer_large && !a.a_panels && !a.out_panels) return launch_gemm_small(a, amode, epi, s);
  if (amode == A_LN) return hipErrorInvalidValue;      // the fused LayerNorm operand exists in the small-batch kernel only
  if (a.N % 128 != 0 || a.K % BK != 0 || a.K <= 0) return hipErrorInvalidValue;
  // operands are addressed with 32-bit byte offsets from their base
  const size_t a_rows = a.a_panels ? ((size_t)a.M + 255) / 256 * 256 : (size_t)a.M;
  const size_t a_bytes = amode == A_PLAIN ? a_rows * (size_t)(a.a_panels ? a.K : a.lda) * 2 : 0;
  if (a_bytes >= ((size_t)1 << 32) || (size_t)a.N * a.K * 2 >= ((size_t)1 << 32)) return hipErrorInvalidValue;
  const bool big = use_large_tile(a);
  if (amode == A_PLAIN) {
    if (a.lda % 8 != 0) return hipErrorInvalidValue;
    if (a.out_panels && epi != EPI_BIAS && epi != EPI_BIAS_GELU) return hipErrorInvalidValue;   // bf16 results only
    if (a.out2 && (epi != EPI_BIAS || a.out_panels || a.n_split % 8 != 0 || a.n_split <= 0 || a.n_split >= a.N)) return hipErrorInvalidValue;
    // streaming stores for bf16 results no cache level could hand on whole (threshold: twice the 32 MB of L2)
    const bool nt = big && (size_t)a.M * a.N * 2 >= ((size_t)64 << 20);
    if (big && large_tile_rows(a.M, a.N) == 320) {
      switch (epi) {
        case EPI_BIAS: return nt ? launch_dl<320, 256, 4, 2, EPI_BIAS, true>(a, s) : launch_dl<320, 256, 4, 2, EPI_BIAS>(a, s);
        case EPI_BIAS_GELU: return nt ? launch_dl<320, 256, 4, 2, EPI_BIAS_GELU, true>(a, s) : launch_dl<320, 256, 4, 2, EPI_BIAS_GELU>(a, s);
        case EPI_BIAS_RESID: return launch_dl<320, 256, 4, 2, EPI_BIAS_RESID>(a, s);
        default: break;     // fp32 store: the 256-row tile below
      }
    }
    // At most one 128 x 128 tile per CU: nothing but the tile's own requests hides the latency of its operands, and the
    // LDS of the second workgroup a CU could hold is free, so the operands get four stages.
    const bool lone = !big && (long)((a.M + 127) / 128) * (a.N / 128) <= 256 && a.K >= 4 * BK;
    if (lone) {
      switch (epi) {
        case EPI_BIAS: return launch_dl<128, 128, 2, 2, EPI_BIAS, false, A_PLAIN, 3>(a, s);
        case EPI_BIAS_GELU: return launch_dl<128, 128, 2, 2, EPI_BIAS_GELU, false, A_PLAIN, 3>(a, s);
        case EPI_BIAS_RESID: return launch_dl<128, 128, 2, 2, EPI_BIAS_RESID, false, A_PLAIN, 3>(a, s);
        case EPI_BIAS_F32: return launch_dl<128, 128, 2, 2, EPI_BIAS_F32, false, A_PLAIN, 3>(a, s);
        default: return hipErrorInvalidValue;
      }
    }
    switch (epi) {
      case EPI_BIAS:
        if (nt) return launch_dl<256, 256, 4, 2, EPI_BIAS, true>(a, s);
        return big ? launch_dl<256, 256, 4, 2, EPI_BIAS>(a, s) : launch_dl<128, 128, 2, 2, EPI_BIAS>(a, s);
      case EPI_BIAS_GELU:
        if (nt) return launch_dl<256, 256, 4, 2, EPI_BIAS_GELU, true>(a, s);
        return big ? launch_dl<256, 256, 4, 2, EPI_BIAS_GELU>(a, s) : launch_dl<128, 128, 2, 2, EPI_BIAS_GELU>(a, s);
      case EPI_BIAS_RESID:
        return big ? launch_dl<256, 256, 4, 2, EPI_BIAS_RESID, false, A_PLAIN, 1>(a, s) : launch_dl<128, 128, 2, 2, EPI_BIAS_RESID>(a, s);
      case EPI_BIAS_F32:
        return big ? launch_dl<256, 256, 4, 2, EPI_BIAS_F32>(a, s) : launch_dl<128, 128, 2, 2, EPI_BIAS_F32>(a, s);
      default: return hipErrorInvalidValue;
    }
  }
  if (a.C % 8 != 0 || 3 * a.C > a.K || !a.row_src || !a.row_flags) return hipErrorInvalidValue;
  // Taps that are whole K steps (C a multiple of 64, no padding after the third tap) go through the
  // direct-load kernel: a masked tap is then a whole 16-byte load redirected to a zero source.  Whether a shape
  // qualifies does not depend on M: all tile sizes of that kernel add up a row in the same order, so a row's bits
  // do not depend on how many rows share the launch (a batch cut into lanes gives the result of the whole batch).
  const bool direct = a.C % BK == 0 && 3 * a.C == a.K && !a.a_panels && !a.w_panels && !a.out_panels;
  switch (epi) {
    case EPI_BIAS_GELU:
      if (direct) return big ? launch_dl<256, 256, 4, 2, EPI_BIAS_GELU, false, A_CONV3>(a, s)
                             : launch_dl<128, 128, 2, 2, EPI_BIAS_GELU, false, A_CONV3>(a, s);
      return big ? launch_cfg<256, 256, 4, 2, A_CONV3, EPI_BIAS_GELU>(a, s) : launch_cfg<128, 128, 2, 2, A_CONV3, EPI_BIAS_GELU>(a, s);
    case EPI_BIAS_GELU_POS:
      if (!a.pos || !a.row_pos) return hipErrorInvalidValue;
      if (direct) return big ? launch_dl<256, 256, 4, 2, EPI_BIAS_GELU_POS, false, A_CONV3, 1>(a, s)
                             : launch_dl<128, 128, 2, 2, EPI_BIAS_GELU_POS, false, A_CONV3>(a, s);
      return big ? launch_cfg<256, 256, 4, 2, A_CONV3, EPI_BIAS_GELU_POS>(a, s)
                 : launch_cfg<128, 128, 2, 2, A_CONV3, EPI_BIAS_GELU_POS>(a, s);
    default: return hipErrorInvalidValue;
  }
}

// Diagnostic: tile rows x columns launch_gemm_bf16 picks for a plain M x N product (0 x 0: the small-batch kernel).
void gemm_tile_choice(int32_t M, int32_t N, int32_t *bm, int32_t *bn) {
  GemmArgs a{};
  a.M = M; a.N = N;
  if (gemm_small_applies(M)) { *bm = 0; *bn = 0; }
  else if (!use_large_tile(a)) { *bm = 128; *bn = 128; }
  else { *bm = large_tile_rows(M, N); *bn = 256; }
}

// Diagnostic: the work units the direct-load GEMM launches for an M x N result with bm x bn tiles, as
// (first row, first column, width in columns) triples in workgroup order.  Returns the count, or -1 if cap is too small.
int gemm_dl_tile_map(int32_t M, int32_t N, int32_t bm, int32_t bn, int32_t *units, int32_t cap) {
  GemmArgs b{};
  b.M = M; b.N = N;
  const int tiles_m = (M + bm - 1) / bm, tiles_n = N / bn;
  const int grid = dl_plan(b, tiles_m, tiles_n);
  int n = 0;
  for (int bid = 0; bid < grid; ++bid) {
    DlUnit u;
    if (!dl_unit(b, bid, tiles_m, tiles_n, u)) continue;
    if (n >= cap) return -1;
    units[3 * n] = u.row * bm;
    units[3 * n + 1] = u.col * bn + (u.half == 2 ? bn / 2 : 0);
    units[3 * n + 2] = u.half == 0 ? bn : bn / 2;
    ++n;
  }
  return n;
}

}  // namespace wf
