// Bidirectional multi-head attention over a ragged batch (head size 64) for gfx950, bf16 MFMA with
// fp32 accumulation and an online (running max / running sum) softmax in fp32.
//
// Tokens of all streams are packed back to back; cu_seqlens gives each stream's row range, and a
// query only ever sees the keys of its own stream.  One workgroup (4 waves) handles one work item
// = (stream, head, 128 consecutive queries); each wave owns 32 queries.  Keys/values are walked in
// tiles of 64, double-buffered in LDS.
//
// Both products are computed transposed: S^T = K Q^T and O^T = V^T P^T.  With
// v_mfma_f32_32x32x16_bf16 a lane then owns ONE query (column lane%32) in the S^T and O^T
// accumulators, so the row max, the rescale factor and the row sum are per-lane scalars, and the
// S^T accumulator registers are, as they stand, the second operand of the P.V MFMA: lane group
// g = lane/32 holds keys {8a + 4g + b}, and the V^T fragment is read with the same key order.
#include <algorithm>
#include <mutex>

#include "device_utils.h"
#include "kernels.h"

namespace wf {

namespace {

constexpr int BQ = 128;    // queries per work item
constexpr int BKV = 64;    // keys per tile

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) void glb_void;
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

// K and V tiles are both kept row-major in LDS, [key][64 features] = 128-byte rows, 16-byte chunk c of
// row r stored at chunk position c ^ swizzle(r) (K: (r >> 1) & 7; V: v_swizzle(r), see there), and are
// filled straight from global memory by
// global_load_lds_dwordx4 (lane l of a wave lands at LDS base + 16 l, so a wave fills 8 rows per
// instruction and applies the swizzle by choosing which chunk it fetches).
//
// The V^T fragment of the P.V product is read with ds_read_b64_tr_b16, which transposes a 16 x 4 block
// of 16-bit elements across a group of 16 lanes: lane r of the group supplies the address of 4
// consecutive elements, and lane i receives element i % 4 of the segments addressed by lanes
// i/4, i/4 + 4, i/4 + 8, i/4 + 12.  Pointing lane r = a + 4e at (key K0 + e, features F0 + 4a ..) gives lane i
// the four keys K0..K0+3 of feature F0 + i: four consecutive reduction indices of one V^T row.
//
// CAUSAL (self-attention among the prompt tokens of a decoder): query r sees keys 0..r.  Tiles that lie
// wholly in the future of a work item are never loaded, a wave skips the tiles that lie wholly in the
// future of its 32 queries (tile starts and wave starts are multiples of 32, so every tile a wave does
// process holds at least one visible key for each of its queries).
// Chunk swizzle of a V row.  A transposing read touches 4 consecutive keys x 64 bytes (4 chunks), so rows r and
// r + 2 -- same half of the 256-byte bank line -- must land in different groups of 4 chunks: the low bit of
// (r >> 1) goes to bit 2 of the XOR mask.  (K rows keep (r >> 1) & 7, which suits 16-row b128 reads.)
__device__ __forceinline__ int v_swizzle(int r) {
  const int q = (r >> 1) & 7;
  return ((q & 1) << 2) | (q >> 1);
}

template <bool CAUSAL>
__global__ void __launch_bounds__(256) attention_bf16_kernel(AttnArgs p) {
  __shared__ __attribute__((aligned(1024))) unsigned char sK[2][BKV * 128];
  __shared__ __attribute__((aligned(1024))) unsigned char sV[2][BKV * 128];

  // The grid has the head count rounded up to a multiple of 8.  Consecutive workgroups go to the 8 XCDs in
  // turn, so slot s of every work item lands on XCD s % 8; slot s holds head (s - rot) mod heads8, with rot
  // fixed per stream: every query block of one (stream, head) then finds its K and V in the same L2.  rot
  // advances by n_heads % 8 from one stream to the next in the (cost-sorted) work list, so the XCDs that get
  // one head more than the others change from stream to stream.  Slots without a head leave at once.
  const int heads8 = (p.n_heads + 7) & ~7;
  const int item = blockIdx.x / heads8;
  const int w1 = p.work[2 * item + 1];
  const int rot = (((w1 >> 20) & 7) * (p.n_heads & 7)) & 7;
  const int head = (blockIdx.x % heads8 + heads8 - rot) % heads8;
  if (head >= p.n_heads) return;
  const int stream = p.work[2 * item];
  const int q0 = w1 & 0xFFFFF;
  const int tok0 = p.cu_q[stream];
  const int Lq = p.cu_q[stream + 1] - tok0;
  const int ktok0 = p.cu_kv[stream];
  const int L = p.cu_kv[stream + 1] - ktok0;     // keys of this stream

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, lg = lane >> 5;
  const int ldq = p.ldq, ld = p.ldkv;
  const __bf16 *Qb = (const __bf16 *)p.q + (size_t)tok0 * ldq + head * 64;
  const __bf16 *Kb = (const __bf16 *)p.k + (size_t)ktok0 * ld + head * 64;
  const __bf16 *Vb = (const __bf16 *)p.v + (size_t)ktok0 * ld + head * 64;

  const int qw0 = q0 + wave * 32;              // first query of this wave
  const bool wave_active = qw0 < Lq;           // waves past the end still help with the loads
  int qrow = qw0 + l32;
  const bool q_valid = qrow < Lq;
  qrow = q_valid ? qrow : Lq - 1;

  // Q fragments for the whole loop: features 16*ks + 8*lg + (0..7) of this lane's query.
  bf16x8 qf[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) qf[ks] = *(const bf16x8 *)(Qb + (size_t)qrow * ldq + ks * 16 + lg * 8);

  f32x16 o[2];
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[t][r] = 0.0f;
  float m_run = -INFINITY;     // running max of the raw logits of this lane's query
  float l_run = 0.0f;          // this lane's share of the running sum (the lane^32 partner has the rest)
  const float c = p.scale * 1.4426950408889634f;   // exp(s*scale) = exp2(s*c)
  const float lazy = 8.0f / c;

  // Tile loads: 16 instructions of 8 rows per tile (8 for K, 8 for V), 4 per wave.
  const int lrow = lane >> 3;
  auto issue = [&](int kt) {
    const int buf = kt & 1;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int g = i * 4 + wave;                       // 0..7: K row group, 8..15: V row group
      const int rt = (g & 7) * 8 + lrow;                // row inside the tile
      int key = kt * BKV + rt;
      key = key < L ? key : L - 1;                      // clamped rows are masked out of the softmax below
      const int lch = (lane & 7) ^ (g < 8 ? (rt >> 1) & 7 : v_swizzle(rt));
      const __bf16 *src = (g < 8 ? Kb : Vb) + (size_t)key * ld + lch * 8;
      unsigned char *dst = (g < 8 ? sK[buf] : sV[buf]) + (g & 7) * 1024;
      __builtin_amdgcn_global_load_lds((const glb_void *)src, (lds_void *)dst, 16, 0, 0);
    }
  };

  // V^T fragment addressing (see above): inside its 16-lane group lane r = a + 4e addresses key e, features 4a..4a+3
  const int r16 = lane & 15;
  const int tr_key = r16 >> 2;                           // e
  const int tr_feat = ((lane >> 4) & 1) * 16 + (r16 & 3) * 4;   // feature offset inside a 32-feature block

  const int k_end = CAUSAL ? min(L, q0 + BQ) : L;          // keys this work item can see at all
  const int n_tiles = (k_end + BKV - 1) / BKV;
  issue(0);
  for (int kt = 0; kt < n_tiles; ++kt) {
    const int key0 = kt * BKV;
    __builtin_amdgcn_s_waitcnt(0x0F70);         // vmcnt(0): my share of tile kt has landed
    __builtin_amdgcn_s_barrier();               // everyone's has; the other buffer is no longer being read
    if (kt + 1 < n_tiles) issue(kt + 1);
    if (!wave_active) continue;
    if (CAUSAL && key0 > qw0 + 31) continue;
    const unsigned char *cK = sK[kt & 1], *cV = sV[kt & 1];

    // ---- S^T = K Q^T : two 32-key blocks, reduction over the 64 features in 4 steps
    f32x16 s[2];
#pragma unroll
    for (int kb2 = 0; kb2 < 2; ++kb2) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s[kb2][r] = 0.0f;
      const int row = kb2 * 32 + l32;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const bf16x8 kf = *(const bf16x8 *)(cK + row * 128 + (((2 * ks + lg) ^ ((row >> 1) & 7)) << 4));
        s[kb2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s[kb2], 0, 0, 0);
      }
    }
    // lane holds logits of query l32 against keys key0 + 32*kb2 + 8*(r/4) + 4*lg + r%4
    if (key0 + BKV > L) {
#pragma unroll
      for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = key0 + kb2 * 32 + 8 * (r >> 2) + 4 * lg + (r & 3);
          if (key >= L) s[kb2][r] = -INFINITY;
        }
    }
    if (CAUSAL && key0 + BKV - 1 > qw0) {
#pragma unroll
      for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = key0 + kb2 * 32 + 8 * (r >> 2) + 4 * lg + (r & 3);
          if (key > qrow) s[kb2][r] = -INFINITY;
        }
    }
    float tmax = s[0][0];
#pragma unroll
    for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
      for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, s[kb2][r]);
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
    const float m_new = fmaxf(m_run, tmax);       // finite: every tile has at least one valid key
    // The softmax reference m_run only has to bound the logits from below by a known margin: it follows the running
    // maximum when some query's maximum has moved up by more than 8 / c (weights up to 2^8 until then; fp32 sums and
    // bf16 weights have the range), which spares most rescales of the accumulators.
    if (__any(m_new > m_run + lazy)) {
      const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c);
      l_run *= alpha;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[t][r] *= alpha;
      m_run = m_new;
    }
    const float mc = m_run * c;
    float psum = 0.0f;
    bf16x8 pf[2][2];
#pragma unroll
    for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        f32x4 e0, e1;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          e0[e] = __builtin_amdgcn_exp2f(s[kb2][8 * h + e] * c - mc);
          e1[e] = __builtin_amdgcn_exp2f(s[kb2][8 * h + 4 + e] * c - mc);
          psum += e0[e] + e1[e];
        }
        const bf16x4 b0 = to_bf16x4(e0), b1 = to_bf16x4(e1);
        pf[kb2][h] = __builtin_shufflevector(b0, b1, 0, 1, 2, 3, 4, 5, 6, 7);
      }
    l_run += psum;

    // ---- O^T += V^T P^T.  Reduction step (kb2, h) covers the 16 keys the lane pair holds in
    // pf[kb2][h]: group lg has keys 32*kb2 + 16*h + 4*lg + (0..3) and the same + 8.
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int fchunk = (t * 32 + tr_feat) >> 3;           // 16-byte chunk of the features this lane addresses
      const int fin = ((t * 32 + tr_feat) & 7) * 2;         // byte offset inside the chunk
#pragma unroll
      for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const int k0 = kb2 * 32 + 16 * h + 4 * lg + tr_key;   // key row this lane addresses (first half)
          const int k1 = k0 + 8;
          const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (lds_s16x4 *)(cV + k0 * 128 + ((fchunk ^ v_swizzle(k0)) << 4) + fin));
          const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (lds_s16x4 *)(cV + k1 * 128 + ((fchunk ^ v_swizzle(k1)) << 4) + fin));
          const bf16x4 w0 = __builtin_bit_cast(bf16x4, v0), w1 = __builtin_bit_cast(bf16x4, v1);
          const bf16x8 vf = __builtin_shufflevector(w0, w1, 0, 1, 2, 3, 4, 5, 6, 7);
          o[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[kb2][h], o[t], 0, 0, 0);
        }
    }
  }

  if (!wave_active) return;
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  const float inv = 1.0f / l_tot;
  if (q_valid) {
    __bf16 *orow = (__bf16 *)p.out + (size_t)(tok0 + qrow) * p.d_model + head * 64;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        f32x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = o[t][g * 4 + e] * inv;
        *(bf16x4 *)(orow + t * 32 + g * 8 + lg * 4) = to_bf16x4(v);
      }
  }
}


// ---------------------------------------------------------------------------------------------
// Variant for batches too small to fill the chip with 128-query work items (one stream's buffer: a few hundred
// tokens).  There the kernel's duration is the length of one workgroup's chain of key tiles, so the chain is cut
// four ways: a workgroup takes 32 queries of one (stream, head) and its four waves walk the key tiles w, w + 4,
// w + 8, ... each with its own running maximum, sum and output accumulators, reading tiles it loads itself into
// LDS buffers of its own (no workgroup barrier inside the loop).  At the end the four partial results are rescaled
// to the common maximum and added in wave order through LDS (deterministic).  Same arithmetic per tile as
// attention_bf16_kernel; the grouping of the tiles differs, so results agree to fp32 rounding of the sums, not bit
// for bit.
__global__ void __launch_bounds__(256) attention_bf16_keysplit_kernel(AttnArgs p) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem_ks[];   // per wave: K[2][8 KB] then V[2][8 KB]

  const int heads8 = (p.n_heads + 7) & ~7;
  const int unit = blockIdx.x / heads8;               // (work item, quarter of its 128 queries)
  const int item = unit >> 2, sub = unit & 3;
  const int w1 = p.work[2 * item + 1];
  const int rot = (((w1 >> 20) & 7) * (p.n_heads & 7)) & 7;
  const int head = (blockIdx.x % heads8 + heads8 - rot) % heads8;
  if (head >= p.n_heads) return;
  const int stream = p.work[2 * item];
  const int q0 = (w1 & 0xFFFFF) + 32 * sub;
  const int tok0 = p.cu_q[stream];
  const int Lq = p.cu_q[stream + 1] - tok0;
  if (q0 >= Lq) return;
  const int ktok0 = p.cu_kv[stream];
  const int L = p.cu_kv[stream + 1] - ktok0;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, lg = lane >> 5;
  const int ldq = p.ldq, ld = p.ldkv;
  const __bf16 *Qb = (const __bf16 *)p.q + (size_t)tok0 * ldq + head * 64;
  const __bf16 *Kb = (const __bf16 *)p.k + (size_t)ktok0 * ld + head * 64;
  const __bf16 *Vb = (const __bf16 *)p.v + (size_t)ktok0 * ld + head * 64;
  unsigned char *myK = smem_ks + wave * 32768, *myV = myK + 16384;

  int qrow = q0 + l32;
  const bool q_valid = qrow < Lq;
  qrow = q_valid ? qrow : Lq - 1;
  bf16x8 qf[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) qf[ks] = *(const bf16x8 *)(Qb + (size_t)qrow * ldq + ks * 16 + lg * 8);

  f32x16 o[2];
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[t][r] = 0.0f;
  float m_run = -INFINITY, l_run = 0.0f;
  const float c = p.scale * 1.4426950408889634f;

  // one wave loads a whole tile: 8 instructions of 8 rows for K, 8 for V
  const int lrow = lane >> 3;
  auto issue = [&](int kt, int buf) {
#pragma unroll
    for (int g = 0; g < 8; ++g) {
      const int rt = g * 8 + lrow;
      int key = kt * BKV + rt;
      key = key < L ? key : L - 1;
      const __bf16 *srck = Kb + (size_t)key * ld + ((lane & 7) ^ ((rt >> 1) & 7)) * 8;
      const __bf16 *srcv = Vb + (size_t)key * ld + ((lane & 7) ^ v_swizzle(rt)) * 8;
      __builtin_amdgcn_global_load_lds((const glb_void *)srck, (lds_void *)(myK + buf * 8192 + g * 1024), 16, 0, 0);
      __builtin_amdgcn_global_load_lds((const glb_void *)srcv, (lds_void *)(myV + buf * 8192 + g * 1024), 16, 0, 0);
    }
  };
  const int r16 = lane & 15;
  const int tr_key = r16 >> 2;
  const int tr_feat = ((lane >> 4) & 1) * 16 + (r16 & 3) * 4;

  const int n_tiles = (L + BKV - 1) / BKV;
  int buf = 0;
  if (wave < n_tiles) issue(wave, 0);
  for (int kt = wave; kt < n_tiles; kt += 4, buf ^= 1) {
    const int key0 = kt * BKV;
    __builtin_amdgcn_s_waitcnt(0x0F70);         // vmcnt(0): this wave's tile kt has landed (nobody else touches these buffers)
    if (kt + 4 < n_tiles) issue(kt + 4, buf ^ 1);
    const unsigned char *cK = myK + buf * 8192, *cV = myV + buf * 8192;
    f32x16 s[2];
#pragma unroll
    for (int kb2 = 0; kb2 < 2; ++kb2) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s[kb2][r] = 0.0f;
      const int row = kb2 * 32 + l32;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const bf16x8 kf = *(const bf16x8 *)(cK + row * 128 + (((2 * ks + lg) ^ ((row >> 1) & 7)) << 4));
        s[kb2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s[kb2], 0, 0, 0);
      }
    }
    if (key0 + BKV > L) {
#pragma unroll
      for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = key0 + kb2 * 32 + 8 * (r >> 2) + 4 * lg + (r & 3);
          if (key >= L) s[kb2][r] = -INFINITY;
        }
    }
    float tmax = s[0][0];
#pragma unroll
    for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
      for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, s[kb2][r]);
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
    const float m_new = fmaxf(m_run, tmax);       // finite: every tile has at least one valid key
    if (__any(m_new > m_run)) {
      const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c);
      l_run *= alpha;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[t][r] *= alpha;
      m_run = m_new;
    }
    const float mc = m_run * c;
    float psum = 0.0f;
    bf16x8 pf[2][2];
#pragma unroll
    for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        f32x4 e0, e1;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          e0[e] = __builtin_amdgcn_exp2f(s[kb2][8 * h + e] * c - mc);
          e1[e] = __builtin_amdgcn_exp2f(s[kb2][8 * h + 4 + e] * c - mc);
          psum += e0[e] + e1[e];
        }
        const bf16x4 b0 = to_bf16x4(e0), b1 = to_bf16x4(e1);
        pf[kb2][h] = __builtin_shufflevector(b0, b1, 0, 1, 2, 3, 4, 5, 6, 7);
      }
    l_run += psum;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int fchunk = (t * 32 + tr_feat) >> 3;
      const int fin = ((t * 32 + tr_feat) & 7) * 2;
#pragma unroll
      for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const int k0 = kb2 * 32 + 16 * h + 4 * lg + tr_key;
          const int k1 = k0 + 8;
          const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(cV + k0 * 128 + ((fchunk ^ v_swizzle(k0)) << 4) + fin));
          const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(cV + k1 * 128 + ((fchunk ^ v_swizzle(k1)) << 4) + fin));
          const bf16x4 w0 = __builtin_bit_cast(bf16x4, v0), w1b = __builtin_bit_cast(bf16x4, v1);
          const bf16x8 vf = __builtin_shufflevector(w0, w1b, 0, 1, 2, 3, 4, 5, 6, 7);
          o[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[kb2][h], o[t], 0, 0, 0);
        }
    }
  }

  // ---- merge the four waves' partial results.  sM / sL: [wave][query]; sO: [wave][query][64 features] fp32, laid
  // over the tile buffers (every wave is past its last tile read once it reaches the barrier).
  __builtin_amdgcn_s_waitcnt(0x0F70);
  __syncthreads();
  float *sM = (float *)smem_ks;                   // 4 x 32
  float *sL = sM + 128;                           // 4 x 32
  float *sO = sL + 128;                           // 4 x 32 x 64
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  if (lg == 0) sM[wave * 32 + l32] = m_run;
  __syncthreads();
  float M = sM[l32];
#pragma unroll
  for (int w = 1; w < 4; ++w) M = fmaxf(M, sM[w * 32 + l32]);
  const float sc = __builtin_amdgcn_exp2f((m_run - M) * c);    // 0 for a wave that saw no tile (m_run = -inf)
  if (lg == 0) sL[wave * 32 + l32] = l_tot * sc;
  // lane holds, of query l32, features t*32 + 8*g + 4*lg + e  (o[t][4*g + e])
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      f32x4 v;
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = o[t][g * 4 + e] * sc;
      *(f32x4 *)(sO + (wave * 32 + l32) * 64 + t * 32 + g * 8 + lg * 4) = v;
    }
  __syncthreads();
  // thread -> query tid / 8, features (tid % 8) * 8 .. + 7
  const int qq = tid >> 3, f0 = (tid & 7) * 8;
  if (q0 + qq < Lq) {
    float lsum = sL[qq];
#pragma unroll
    for (int w = 1; w < 4; ++w) lsum += sL[w * 32 + qq];
    const float inv = 1.0f / lsum;
    f32x4 a0 = *(const f32x4 *)(sO + qq * 64 + f0), a1 = *(const f32x4 *)(sO + qq * 64 + f0 + 4);
#pragma unroll
    for (int w = 1; w < 4; ++w) {
      const f32x4 b0 = *(const f32x4 *)(sO + (w * 32 + qq) * 64 + f0), b1 = *(const f32x4 *)(sO + (w * 32 + qq) * 64 + f0 + 4);
#pragma unroll
      for (int e = 0; e < 4; ++e) { a0[e] += b0[e]; a1[e] += b1[e]; }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) { a0[e] *= inv; a1[e] *= inv; }
    const bf16x4 c0 = to_bf16x4(a0), c1 = to_bf16x4(a1);
    __bf16 *orow = (__bf16 *)p.out + (size_t)(tok0 + q0 + qq) * p.d_model + head * 64 + f0;
    *(bf16x8 *)orow = __builtin_shufflevector(c0, c1, 0, 1, 2, 3, 4, 5, 6, 7);
  }
}

}  // namespace

int attention_q_tile() { return BQ; }

hipError_t launch_attention_bf16(const AttnArgs &a, hipStream_t s) {
  if (a.n_work <= 0) return hipSuccess;
  if (a.d_model != a.n_heads * 64) return hipErrorInvalidValue;
  if (a.ldq % 8 != 0 || a.ldkv % 8 != 0 || !a.q || !a.k || !a.v || !a.cu_q || !a.cu_kv) return hipErrorInvalidValue;
  const dim3 grid(a.n_work * ((a.n_heads + 7) & ~7));
  if (a.causal) {
    if (a.cu_q != a.cu_kv) return hipErrorInvalidValue;
    hipLaunchKernelGGL(attention_bf16_kernel<true>, grid, dim3(256), 0, s, a);
  } else if (std::min<long>(4L * a.n_work, a.M / 32 + a.B) * a.n_heads <= 256) {
    // so few queries that even 32-query workgroups (one per compute unit: they take 128 KB of LDS) fit the chip in one go:
    // cut the key loop four ways instead.  (8 streams of 325 tokens x 16 heads = 1408 such workgroups ran 12 % slower.)
    constexpr int smem = 4 * 32768;
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [&] {
      attr_err = hipFuncSetAttribute((const void *)attention_bf16_keysplit_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    });
    if (attr_err != hipSuccess) return attr_err;
    hipLaunchKernelGGL(attention_bf16_keysplit_kernel, dim3(4 * grid.x), dim3(256), smem, s, a);
  } else {
    hipLaunchKernelGGL(attention_bf16_kernel<false>, grid, dim3(256), 0, s, a);
  }
  return hipGetLastError();
}

}  // namespace wf
