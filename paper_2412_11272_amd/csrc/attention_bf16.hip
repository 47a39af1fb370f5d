// Bidirectional multi-head attention over a ragged batch (head size 64) for gfx950, bf16 MFMA with
// fp32 accumulation and an online (running max / running sum) softmax in fp32.
//
// Tokens of all streams are packed back to back; cu_seqlens gives each stream's row range, and a
// query only ever sees the keys of its own stream.  One workgroup (4 waves) handles one work item
// = (stream, head, 128 consecutive queries); each wave owns 32 queries.  Keys/values are walked in
// tiles of 64: K goes to LDS row-major, V goes to LDS transposed ([feature][key]) so that both
// MFMA operands of the P.V product have their reduction index (the key) contiguous per lane.
//
// Both products are computed transposed: S^T = K Q^T and O^T = V^T P^T.  With
// v_mfma_f32_32x32x16_bf16 a lane then owns ONE query (column lane%32) in the S^T and O^T
// accumulators, so the row max, the rescale factor and the row sum are per-lane scalars, and the
// S^T accumulator registers are, as they stand, the second operand of the P.V MFMA: lane group
// g = lane/32 holds keys {8a + 4g + b}, and the V^T fragment is simply read with the same key order.
#include "device_utils.h"
#include "kernels.h"

namespace wf {

namespace {

constexpr int BQ = 128;    // queries per work item
constexpr int BKV = 64;    // keys per tile

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// Tile staging: K row-major [key][64 features] with the 16-byte chunk XOR-ed by (key >> 1) & 7, and
// V transposed [feature][64 keys] in 8-byte units (4 keys) XOR-ed by feature & 15.
__device__ __forceinline__ void stage_kv(unsigned char *sK, unsigned char *sVt, const u32x4 &k_a, const u32x4 &k_b,
                                         const u32x4 &v_a, const u32x4 &v_b, int kp, int ch) {
  const int r0 = 2 * kp, r1 = r0 + 1;
  *(u32x4 *)(sK + r0 * 128 + ((ch ^ ((r0 >> 1) & 7)) << 4)) = k_a;
  *(u32x4 *)(sK + r1 * 128 + ((ch ^ ((r1 >> 1) & 7)) << 4)) = k_b;
  // feature f = 8*ch + e; keys (2kp, 2kp+1) of that feature packed into one 32-bit word
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const uint32_t a = v_a[e >> 1], b = v_b[e >> 1];
    const uint32_t w = (e & 1) ? ((a >> 16) | (b & 0xffff0000u)) : ((a & 0xffffu) | (b << 16));
    const int f = 8 * ch + e;
    const int unit = (kp >> 1) ^ (f & 15);
    *(uint32_t *)(sVt + f * 128 + unit * 8 + (kp & 1) * 4) = w;
  }
}

__global__ void __launch_bounds__(256) attention_bf16_kernel(AttnArgs p) {
  __shared__ __attribute__((aligned(16))) unsigned char sK[2][BKV * 128];
  __shared__ __attribute__((aligned(16))) unsigned char sVt[2][64 * 128];

  const int item = blockIdx.x / p.n_heads;
  const int head = blockIdx.x % p.n_heads;
  const int stream = p.work[2 * item];
  const int q0 = p.work[2 * item + 1];
  const int tok0 = p.cu_seqlens[stream];
  const int L = p.cu_seqlens[stream + 1] - tok0;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lg = lane >> 5;
  const int ld = 3 * p.d_model;
  const __bf16 *qkv = (const __bf16 *)p.qkv;
  const __bf16 *Qb = qkv + (size_t)tok0 * ld + head * 64;
  const __bf16 *Kb = Qb + p.d_model;
  const __bf16 *Vb = Qb + 2 * p.d_model;

  const int qw0 = q0 + wave * 32;              // first query of this wave
  const bool wave_active = qw0 < L;            // waves past the end still help with the loads
  int qrow = qw0 + l32;
  const bool q_valid = qrow < L;
  qrow = q_valid ? qrow : L - 1;

  // Q fragments for the whole loop: features 16*ks + 8*lg + (0..7) of this lane's query.
  bf16x8 qf[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) qf[ks] = *(const bf16x8 *)(Qb + (size_t)qrow * ld + ks * 16 + lg * 8);

  f32x16 o[2];
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[t][r] = 0.0f;
  float m_run = -INFINITY;     // running max of the raw logits of this lane's query
  float l_run = 0.0f;          // this lane's share of the running sum (the lane^32 partner has the rest)
  const float c = p.scale * 1.4426950408889634f;   // exp(s*scale) = exp2(s*c)

  // cooperative load mapping: thread -> (key pair kp, 16-byte feature chunk ch)
  const int kp = tid >> 3, ch = tid & 7;
  u32x4 k_a, k_b, v_a, v_b;
  auto fetch = [&](int kt) {
    int ka = kt * BKV + 2 * kp, kb = ka + 1;
    ka = ka < L ? ka : L - 1;                   // clamped rows are masked out of the softmax below
    kb = kb < L ? kb : L - 1;
    k_a = *(const u32x4 *)(Kb + (size_t)ka * ld + ch * 8);
    k_b = *(const u32x4 *)(Kb + (size_t)kb * ld + ch * 8);
    v_a = *(const u32x4 *)(Vb + (size_t)ka * ld + ch * 8);
    v_b = *(const u32x4 *)(Vb + (size_t)kb * ld + ch * 8);
  };

  const int n_tiles = (L + BKV - 1) / BKV;
  fetch(0);
  stage_kv(sK[0], sVt[0], k_a, k_b, v_a, v_b, kp, ch);
  __syncthreads();
  for (int kt = 0; kt < n_tiles; ++kt) {
    const int key0 = kt * BKV;
    const unsigned char *cK = sK[kt & 1], *cVt = sVt[kt & 1];
    if (kt + 1 < n_tiles) fetch(kt + 1);        // in flight while this tile is being used
    if (wave_active) {
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
      float tmax = s[0][0];
#pragma unroll
      for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
        for (int r = 0; r < 16; ++r) tmax = fmaxf(tmax, s[kb2][r]);
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
      const float m_new = fmaxf(m_run, tmax);       // finite: every tile has at least one valid key
      if (__any(m_new > m_run)) {                   // rescale only when some query's maximum moved
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
        const int f = t * 32 + l32;
        const unsigned char *vrow = cVt + f * 128;
#pragma unroll
        for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            const int u0 = (kb2 * 32 + 16 * h + 4 * lg) >> 2;      // 8-byte unit of the first 4 keys
            const bf16x4 v0 = *(const bf16x4 *)(vrow + ((u0 ^ (f & 15)) << 3));
            const bf16x4 v1 = *(const bf16x4 *)(vrow + (((u0 + 2) ^ (f & 15)) << 3));
            const bf16x8 vf = __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
            o[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[kb2][h], o[t], 0, 0, 0);
          }
      }
    }
    if (kt + 1 < n_tiles) stage_kv(sK[(kt + 1) & 1], sVt[(kt + 1) & 1], k_a, k_b, v_a, v_b, kp, ch);
    __syncthreads();                            // next tile staged, this one no longer read
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

}  // namespace

int attention_q_tile() { return BQ; }

hipError_t launch_attention_bf16(const AttnArgs &a, hipStream_t s) {
  if (a.n_work <= 0) return hipSuccess;
  if (a.d_model != a.n_heads * 64) return hipErrorInvalidValue;
  hipLaunchKernelGGL(attention_bf16_kernel, dim3(a.n_work * a.n_heads), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace wf
