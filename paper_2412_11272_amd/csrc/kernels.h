// Internal launcher interface between the host runtime (encoder.hip) and the gfx950 kernels.
// Nothing here is part of the public ABI (include/wf_encoder.h is).
#pragma once
#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdint.h>

namespace wf {

typedef uint16_t bf16_raw;   // storage type of a bfloat16 value in host-visible structs

// How the GEMM reads its activation operand.
enum AMode : int {
  A_PLAIN = 0,   // row r of the operand is A + r * lda
  A_CONV3 = 1,   // row r is a contiguous window of 3*C elements starting at row_src[r] * C of a
                 // [rows, C] matrix: the three taps of a width-3 convolution.  row_flags[r] bit 0
                 // zeroes tap 0 (first frame of a stream), bit 1 zeroes tap 2 (last frame).
  A_LN = 2,      // small-batch kernel only: A is an fp32 matrix x (row stride lda) and the operand is LayerNorm(x) with
                 // ln_g / ln_b / ln_eps, normalised on the way in
};

// What the GEMM does with acc = A . W^T.
enum Epilogue : int {
  EPI_BIAS = 0,            // out = acc + bias                          (QKV projection)
  EPI_BIAS_GELU = 1,       // out = GELU(acc + bias)                    (fc1, first convolution)
  EPI_BIAS_RESID = 2,      // out(fp32) += acc + bias, in place         (out-projection, fc2)
  EPI_BIAS_GELU_POS = 3,   // out(fp32) = GELU(acc + bias) + pos[row_pos[r]]   (second convolution)
  EPI_BIAS_F32 = 4,        // out(fp32) = acc + bias                    (logits)
};

struct GemmArgs {
  const void *A;            // activations: bf16 (MFMA path) or fp32 (debug path)
  const void *W;            // weights [N, K] row-major, same element type as A; K zero-padded
  const float *bias;        // [N]
  void *out;                // [M, ldo]; bf16 for EPI_BIAS / EPI_BIAS_GELU on the MFMA path, else fp32
  int32_t M, N, K;          // K is the padded reduction length (multiple of 64 on the MFMA path)
  int32_t lda, ldo;
  // work-unit split of the direct-load GEMM (set by its launcher): full tiles, then half-width units
  int32_t n_full, n_half, full_per_xcd, half_per_xcd;
  int32_t group_n;          // tiles walk column groups of this many tile columns (>= tiles per row: plain row-major)
  // Panel layout (direct-load GEMM only): instead of row-major, a matrix is stored as [rows/256][cols/64][256][64],
  // i.e. every (256-row panel, 64-column chunk) is one contiguous 32 KB block -- exactly one K step of a
  // tile's operand.  a_panels: A is read in that layout; w_panels: W is (rows = output features, padded to a
  // multiple of 256); out_panels: a bf16 result is written in it.
  int32_t a_panels, w_panels, out_panels;
  // A_CONV3 only
  const int32_t *row_src;
  const int32_t *row_flags;
  int32_t C;                // channels per tap; 3*C <= K, elements at k >= 3*C read as zero
  // EPI_BIAS_GELU_POS only
  const float *pos;         // [n_pos, N]
  const int32_t *row_pos;   // [M]
  // A_LN only
  const float *ln_g, *ln_b; // [K]
  float ln_eps;
  // bf16 results only (EPI_BIAS on the MFMA path): columns [n_split, N) of the result go to out2 (row stride ldo2) instead
  // of out, starting at its column 0 -- one product feeding two buffers (queries | keys and values).  n_split % 8 == 0.
  void *out2;
  int32_t n_split, ldo2;
  int32_t prefer_large;     // stay on the large-batch kernels whatever M is (a product that streams a huge weight matrix)
  int32_t prefer_small;     // run on the small-batch kernel even if M is above its usual limit (the first convolution
                            // of a small batch has twice as many rows as the batch has tokens)
};

struct AttnArgs {
  // Head h owns columns [64h, 64h+64) counted from each of the three base pointers.  Queries of stream i
  // are rows [cu_q[i], cu_q[i+1]) of q (row stride ldq elements), its keys/values rows
  // [cu_kv[i], cu_kv[i+1]) of k and v (row stride ldkv).  Encoder self-attention: one [M, 3d] matrix
  // q | k | v and cu_q == cu_kv.  causal != 0 (needs cu_q == cu_kv): query r sees keys 0..r of its stream.
  const void *q, *k, *v;
  void *out;                // [Mq, d_model]
  int32_t ldq, ldkv;
  const int32_t *cu_q, *cu_kv;   // [B+1] each
  const int32_t *work;      // [n_work][2]: (stream, first query row inside the stream), longest first
  int32_t n_work, n_heads, d_model, B, M;   // M = total query rows
  int32_t causal;
  float scale;              // 1/sqrt(64)
};

struct PrepArgs {
  const void *mel;          // caller's frames [*, n_mels]
  const void *hush;         // [H, n_mels] same dtype as the packed output
  void *packed;             // [total_frames, n_mels]
  const int32_t *cu_frames, *cu_seqlens, *frame_offset, *n_frames;
  int32_t *frame_src, *frame_flags;            // [total_frames]  conv1 row map
  int32_t *tok_src, *tok_flags, *tok_pos;      // [M]             conv2 row map + position index
  int32_t B, n_mels, total_frames, M, mel_is_bf16;
};

// bf16 MFMA path -------------------------------------------------------------------------------
hipError_t launch_gemm_bf16(const GemmArgs &a, AMode amode, Epilogue epi, hipStream_t s);
// small row counts (gemm_small_applies(M)): 32 x 32 tiles, reduction split over the waves, optional fused LayerNorm
bool gemm_small_applies(int32_t M);
hipError_t launch_gemm_small(const GemmArgs &a, AMode amode, Epilogue epi, hipStream_t s);
hipError_t launch_attention_bf16(const AttnArgs &a, hipStream_t s);
hipError_t launch_layernorm(const float *x, const float *g, const float *b, void *out, int out_bf16,
                            int32_t M, int32_t d, float eps, hipStream_t s);
hipError_t launch_prep(const PrepArgs &a, int packed_bf16, hipStream_t s);
// x[r, :] = table[tok[r], :] + pos[pos_idx[r], :]  (fp32 out; table bf16 or fp32, pos fp32)
hipError_t launch_embed(const void *table, int table_bf16, const float *pos, const int32_t *tok, const int32_t *pos_idx,
                        float *x, int32_t rows, int32_t d, hipStream_t s);
// dst[i, :] = src[row[i], :] for rows of row_bytes bytes (multiple of 16)
hipError_t launch_gather_rows(const void *src, const int32_t *row, void *dst, int32_t n, int32_t row_bytes, hipStream_t s);
int attention_q_tile();     // query rows per attention work item
int gemm_dl_tile_map(int32_t M, int32_t N, int32_t bm, int32_t bn, int32_t *units, int32_t cap);   // diagnostic, host only
void gemm_tile_choice(int32_t M, int32_t N, int32_t *bm, int32_t *bn);                                                  // diagnostic, host only

// fp32 debug path ------------------------------------------------------------------------------
hipError_t launch_gemm_f32(const GemmArgs &a, AMode amode, Epilogue epi, hipStream_t s);
hipError_t launch_attention_f32(const AttnArgs &a, hipStream_t s);

// thread-local error text behind wf_last_error(), shared by all translation units
int set_error(int code, const char *fmt, va_list ap);
char *error_buffer();

// one-time per-process kernel attribute setup (dynamic LDS limits)
hipError_t init_kernels();

}  // namespace wf
