/*
 * wf_encoder.h -- C ABI of the ragged Whisper-style audio encoder for MI355X (gfx950).
 *
 * What the library computes (paper: WhisperFlow, arXiv 2412.11272):
 *   Each processing round, every stream hands over a log-mel snapshot of its current audio buffer
 *   (Section "Operations", processing rounds), of any length up to 30 s.  Instead of padding the
 *   snapshot to a 30 s / 1500-token window, one fixed short segment -- the hush word, 0.5 s = 25
 *   tokens, one per model -- is appended to it (Section "Hush word", hush word position: x (+) h)
 *   and the encoder runs on that length only.  Different streams therefore have different lengths
 *   (Section "Applicability" names this as the obstacle to batching); this library batches them
 *   anyway by packing all streams' tokens back to back and restricting attention to each stream.
 *   The encoder itself is the dense stage of a round (Section "CPU/GPU pipelining", categorization
 *   of workloads, item 1): log-mel -> Conv1d(k3)+GELU -> Conv1d(k3, stride 2)+GELU -> + sinusoidal
 *   positions -> n_layers pre-LN transformer blocks (bidirectional multi-head attention, GELU MLP)
 *   -> LayerNorm.  T mel frames (100 per second) become floor((T+1)/2) tokens.
 *   The hush word lives here at the log-mel level (a [hush_frames, n_mels] block); the paper appends
 *   at the raw-audio level (Section "Hush word", target level).
 *
 * Conventions
 *   - Every function returns WF_OK (0) or a negative WF_E_* code; nothing throws or exits.
 *     wf_last_error() gives a thread-local text for the last failure on the calling thread.
 *   - "host" pointers are ordinary CPU memory; "device" pointers are HIP device memory on the GPU
 *     that was current when the encoder was created.  The library never frees caller memory.
 *   - All matrices are row-major.  Linear weights are [out_features, in_features]; convolution
 *     kernels are [out_channels, in_channels, 3] (tap 0 multiplies frame t-1, tap 2 frame t+1 for
 *     the first convolution; frames 2j-1, 2j, 2j+1 for output token j of the second).
 *   - Log-mel input is time-major [frames, n_mels].
 */
#ifndef WF_ENCODER_H
#define WF_ENCODER_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define WF_OK            0
#define WF_E_INVALID_ARG (-1)   /* NULL pointer, bad shape, bad length, bad dtype                */
#define WF_E_CAPACITY    (-2)   /* batch exceeds the capacity given at create, or out_capacity   */
#define WF_E_OOM         (-3)   /* device or host allocation failed                              */
#define WF_E_HIP         (-4)   /* a HIP runtime call or kernel launch failed                    */

#define WF_DTYPE_F32  0
#define WF_DTYPE_BF16 1

#define WF_PRECISION_BF16 0     /* bf16 MFMA with fp32 accumulation, fp32 residual stream        */
#define WF_PRECISION_F32  1     /* debug path: fp32 storage and arithmetic everywhere            */

typedef struct wf_encoder wf_encoder;   /* opaque; owned by the library */

typedef struct {
  int32_t n_mels;                /* log-mel bins per frame; multiple of 8                          */
  int32_t d_model;               /* multiple of 128; d_model / n_heads must be 64                  */
  int32_t n_layers;              /* >= 0                                                           */
  int32_t n_heads;
  int32_t d_mlp;                 /* multiple of 128                                                */
  int32_t hush_frames;           /* H >= 0; 0 disables the append (padded-window baseline)         */
  int32_t max_streams;           /* capacity: streams per call                                     */
  int32_t max_total_frames;      /* capacity: sum over streams of (n_frames + H) per call; the
                                    widest activation matrix of such a batch must stay under 4 GiB:
                                    (max_total_frames / 2 + 256) * max(d_mlp, d_model) * 2 < 2^32  */
  int32_t max_frames_per_stream; /* capacity: n_frames + H of any one stream                       */
  int32_t precision;             /* WF_PRECISION_*                                                 */
  float   ln_eps;                /* LayerNorm epsilon; <= 0 selects 1e-5                           */
} wf_config;

/* Weights of one pre-LN block.  All HOST pointers, fp32.  bk may be NULL (no key bias). */
typedef struct {
  const float *ln1_g, *ln1_b;    /* [d]                */
  const float *wq, *bq;          /* [d, d], [d]        */
  const float *wk, *bk;          /* [d, d], [d] | NULL */
  const float *wv, *bv;          /* [d, d], [d]        */
  const float *wo, *bo;          /* [d, d], [d]        */
  const float *ln2_g, *ln2_b;    /* [d]                */
  const float *w1, *b1;          /* [d_mlp, d], [d_mlp]*/
  const float *w2, *b2;          /* [d, d_mlp], [d]    */
} wf_layer_weights;

/* All HOST pointers, fp32.  The library copies and converts them in wf_encoder_create; the caller
 * may free them as soon as it returns. */
typedef struct {
  const float *conv1_w, *conv1_b;        /* [d, n_mels, 3], [d]                                    */
  const float *conv2_w, *conv2_b;        /* [d, d, 3], [d]                                         */
  const float *hush_mel;                 /* [hush_frames, n_mels]; may be NULL iff hush_frames == 0 */
  const wf_layer_weights *layers;        /* [n_layers]                                             */
  const float *lnf_g, *lnf_b;            /* [d]                                                    */
} wf_weights;

/*
 * Create an encoder on the current HIP device: validates the configuration, uploads the weights
 * (rounded to bf16, round-to-nearest-even, in WF_PRECISION_BF16), the hush segment and the
 * sinusoidal position table P[j, c] = sin(j w_c), P[j, d/2 + c] = cos(j w_c),
 * w_c = 10000^(-c/(d/2 - 1)), and allocates a workspace sized from the three capacities.
 * Errors: WF_E_INVALID_ARG (NULL, bad shape), WF_E_OOM, WF_E_HIP.  On error *out is NULL.
 */
int wf_encoder_create(const wf_config *cfg, const wf_weights *weights, wf_encoder **out);

/*
 * Encode one ragged batch (the hot path).
 *
 *   mel_dev       device; log-mel frames, [*, n_mels] time-major, dtype mel_dtype (WF_DTYPE_*).
 *   frame_offset  host [B]; index (in frames) of stream i's first frame inside mel_dev.  Padded
 *                 layouts (i * T_max) and packed layouts (prefix sums) are both expressible.
 *   n_frames      host [B]; T_i >= 1 payload frames of stream i.
 *   B             1 <= B <= max_streams.
 *   out_dev       device; receives the encoder states, [M, d_model] packed stream-major, dtype
 *                 out_dtype; M = sum_i floor((T_i + H + 1) / 2).  Stream i occupies rows
 *                 [cu_seqlens[i], cu_seqlens[i+1]).
 *   out_capacity_tokens  rows available in out_dev.
 *   cu_seqlens_host      host [B+1], may be NULL; written before the call returns (computed on the
 *                 host from n_frames, no device synchronisation involved).
 *   hip_stream    a hipStream_t (NULL = the default stream).  All work is enqueued on it and the
 *                 call returns without waiting; the caller synchronises before reading out_dev.
 *
 * Host-side validation happens before anything is enqueued: WF_E_INVALID_ARG for NULL pointers,
 * B < 1, T_i < 1, negative offsets or unknown dtypes; WF_E_CAPACITY if B > max_streams,
 * T_i + H > max_frames_per_stream, sum(T_i + H) > max_total_frames or M > out_capacity_tokens.
 * An encoder owns one workspace: calls on the same encoder must not overlap in time (enqueue
 * them on one stream, or synchronise between streams).
 */
int wf_encode_batch(wf_encoder *enc,
                    const void *mel_dev, int32_t mel_dtype,
                    const int32_t *frame_offset, const int32_t *n_frames, int32_t B,
                    void *out_dev, int32_t out_dtype, int64_t out_capacity_tokens,
                    int32_t *cu_seqlens_host,
                    void *hip_stream);

/* Free everything the encoder owns (waits for the device to finish first).  NULL is accepted. */
void wf_encoder_destroy(wf_encoder *enc);

/* Thread-local description of the last error on this thread ("" if none). */
const char *wf_last_error(void);

/*
 * Host-only helper (no GPU needed): validates lengths exactly as wf_encode_batch does and writes
 * cu_seqlens[B+1] (token prefix sums), *total_frames = sum(T_i + H) and *total_tokens = M.
 * Output pointers may be NULL.  Same error codes as wf_encode_batch.
 */
int wf_plan_batch(const wf_config *cfg, const int32_t *n_frames, int32_t B,
                  int32_t *cu_seqlens, int64_t *total_frames, int64_t *total_tokens);

/* Host-only: validates a configuration as wf_encoder_create would (WF_OK or WF_E_INVALID_ARG). */
int wf_config_check(const wf_config *cfg);

/*
 * Per-kernel timing, measured with HIP events on the stream the kernels are launched on.
 * wf_encoder_set_profiling(enc, 1) makes later wf_encode_batch calls bracket every kernel launch
 * with a pair of events; wf_encoder_kernel_stats waits for the device, then adds up the elapsed
 * times by kernel class and resets the counters.  Classes are indexed 0 .. wf_kernel_class_count()-1.
 */
typedef struct {
  const char *name;     /* static string, e.g. "gemm_fc1" */
  int64_t launches;     /* launches since the last wf_encoder_kernel_stats call */
  double  total_ms;     /* sum of their durations */
  double  flops;        /* algorithmic flops of those launches (0 for bandwidth kernels) */
  double  bytes;        /* algorithmic HBM bytes of those launches (operands read + results written once) */
} wf_kernel_stat;

int wf_kernel_class_count(void);
int wf_encoder_set_profiling(wf_encoder *enc, int32_t enabled);
int wf_encoder_kernel_stats(wf_encoder *enc, wf_kernel_stat *stats, int32_t n_stats);
/* Number of lanes (1 .. 4, default 2): a batch of at least 4096 tokens per lane is cut into that many
 * contiguous groups of streams which run the layer sequence on streams of their own (lane 0 on the caller's),
 * so that one group's bandwidth-bound kernels and GEMM tails overlap another group's matrix work (worth 1-2 %
 * on a power-limited part).  Results do not depend on it.  The call is still ordered on hip_stream as a whole:
 * the other lanes start after the work already queued on hip_stream and hip_stream waits for them before the
 * call's work counts as done.  wf_encoder_get_lanes returns the current setting (negative WF_E_* on error). */
int wf_encoder_set_lanes(wf_encoder *enc, int32_t n_lanes);
int wf_encoder_get_lanes(const wf_encoder *enc);
/* Replay of small batches (opt-in, default off).  A batch that runs on one lane (fewer than 8192 tokens) consists
 * of 4 + 7 n_layers short dependent kernels (paper, Section "Operations": one stream's buffer per round is the
 * method's own case, 75 .. 750 tokens).  With wf_encoder_set_graphs(enc, 1), wf_encode_batch keeps up to 64 captured
 * HIP graphs of that launch sequence, keyed on everything that shapes the launches or is baked into their arguments: B, every
 * n_frames[i] and frame_offset[i], mel_dev, out_dev and the two dtypes.  A key seen for the second time is captured
 * (on a stream of the encoder, never the caller's; no memset or memcpy node: each entry owns a device copy of its
 * index arrays) and replayed from then on with one hipGraphLaunch on hip_stream; other calls, all batches with
 * more lanes, the fp32 path and calls under wf_encoder_set_profiling launch kernel by kernel.  Results are
 * bit-identical either way.  It takes the per-launch work off the host thread (one call instead of dozens); the time
 * on the GPU is the same, because a kernel of a dependent chain starts 5 - 7 us after its predecessor however it was
 * submitted.  The caller's buffers are part of the key, so a replay reads and writes the same
 * addresses the capture saw: keep mel_dev / out_dev allocated while replay is on.  wf_encoder_graph_stats: calls replayed, graphs captured, calls launched
 * directly (any pointer may be NULL). */
int wf_encoder_set_graphs(wf_encoder *enc, int32_t enabled);
int wf_encoder_graph_stats(const wf_encoder *enc, int64_t *replays, int64_t *captures, int64_t *direct_calls);
/* The configuration the encoder was created with (ln_eps as resolved). */
int wf_encoder_get_config(const wf_encoder *enc, wf_config *cfg);

/* Compute units and peak shader clock (kHz) of the current HIP device, as the runtime reports them (either pointer
 * may be NULL).  WF_E_HIP without a device.  For reports: the dense bf16 MFMA peak is units x 4096 flop x clock. */
int wf_device_info(int32_t *compute_units, int32_t *clock_khz);

/*
 * Diagnostic, host only (no GPU call): the work units the MFMA GEMM launches for an M x N result with tile_m x tile_n
 * tiles, in workgroup order, as (first row, first column, width in columns) triples in units[3 * i .. 3 * i + 2]
 * (HOST, room for `capacity` triples).  Whole tiles first; the tiles left over after the last full round of the
 * chip are cut into two half-width units when that shortens the last round.  It runs the very code the kernel
 * uses to decode its workgroup id, so a test can check that every element of the result is covered exactly once.
 * Returns the number of units (>= 0) or a negative WF_E_* code.
 */
int wf_gemm_tile_map(int32_t M, int32_t N, int32_t tile_m, int32_t tile_n, int32_t *units, int32_t capacity);

/*
 * Diagnostic, host only: the tile (rows x columns of the result per workgroup) the bf16 MFMA GEMM picks for a plain
 * M x N product: 320 x 256 or 256 x 256 for large batches (whichever finishes its last round of the chip earlier),
 * 128 x 128 below that, 0 x 0 when M is small enough for the small-batch kernel.  N must be a multiple of 128.
 */
int wf_gemm_tile_choice(int32_t M, int32_t N, int32_t *tile_m, int32_t *tile_n);

/*
 * Diagnostic, host only: the GELU the bf16 kernels apply in their epilogues (erf form by a clamped odd polynomial, no
 * transcendental instruction), evaluated on the host with the same source code; out[i] = GELU(z[i]) for n HOST
 * values.  A test bounds its distance from the exact erf form (Section "Operations": the encoder is the stock
 * Whisper one, whose activation is the erf GELU).
 */
int wf_gelu_host(const float *z, float *out, int32_t n);

/*
 * Operator-level entry points: single steps of the encoder on caller-provided DEVICE buffers, for
 * per-operator checks and micro-benchmarks.  precision selects the kernel family and the element
 * type of activations and weights (WF_PRECISION_BF16: bf16, WF_PRECISION_F32: fp32).
 *
 * wf_op_linear      out = epilogue(a . w^T + bias); a [M, K], w [N, K], bias fp32 [N]; N % 128 == 0,
 *                   K % 64 == 0.  epilogue 0: out [M, N] in the activation type; 1: GELU, same type;
 *                   2: out is fp32 [M, N] and is updated in place, out += a . w^T + bias.
 *                   (the projections of a transformer block: QKV, fc1, and out-projection / fc2)
 *                   bf16: a and w must each be smaller than 4 GiB (WF_E_INVALID_ARG otherwise).
 * wf_op_layernorm   out[r, :] = (x[r, :] - mean) / sqrt(biased var + eps) * g + b, x fp32 [M, d],
 *                   out dtype WF_DTYPE_*; d % 4 == 0, d <= 2048.
 * wf_op_ln_linear   bf16 path, small batches only (M <= 1024, else WF_E_CAPACITY): out = epilogue(LayerNorm(x) . w^T + bias)
 *                   with x fp32 [M, K] normalised on the way into the product (K <= 2048), w bf16 [N, K] row-major,
 *                   out bf16 [M, N]; epilogue 0 or 1 as above.  What QKV and fc1 run as for a single stream's buffer.
 * wf_op_attention   bidirectional softmax attention restricted to each stream, head size 64:
 *                   qkv [M, 3 * 64 * n_heads] (q | k | v), out [M, 64 * n_heads], cu_seqlens_host
 *                   [B+1] with cu_seqlens_host[0] == 0 and no empty stream.  Allocates a small
 *                   index buffer and waits for hip_stream before returning (the others are async).
 */
int wf_op_linear(int32_t precision, const void *a_dev, const void *w_dev, const float *bias_dev, void *out_dev,
                 int32_t M, int32_t N, int32_t K, int32_t epilogue, void *hip_stream);
int wf_op_layernorm(const float *x_dev, const float *g_dev, const float *b_dev, void *out_dev, int32_t out_dtype,
                    int32_t M, int32_t d, float eps, void *hip_stream);
int wf_op_ln_linear(const float *x_dev, const float *g_dev, const float *b_dev, float eps, const void *w_dev,
                    const float *bias_dev, void *out_dev, int32_t M, int32_t N, int32_t K, int32_t epilogue, void *hip_stream);
int wf_op_attention(int32_t precision, const void *qkv_dev, void *out_dev, const int32_t *cu_seqlens_host, int32_t B,
                    int32_t n_heads, void *hip_stream);
/*
 * wf_op_attention for callers that cannot allocate device memory (code that a HIP graph capture may enclose,
 * tight serving loops, harnesses that forbid hipMalloc).  Same arguments, same kernels and bit-identical
 * results, but: it calls no hipMalloc / hipFree / hipMemcpy / hipMemset and no allocating routine of any
 * library; the prefix sums and the work list go into a 64 KiB device array that is part of the library image
 * (one copy per GPU, held until the process ends) and reach it as kernel arguments of a small fill kernel; and it
 * is asynchronous on hip_stream (no wait before returning).
 * Limit: B + 1 + 2 * sum_i ceil(L_i / 128) <= 16384 ints (L_i = tokens of stream i), i.e. about 1 M tokens in
 * long streams or 5461 one-block streams; beyond it the call returns WF_E_CAPACITY with the sizes in
 * wf_last_error() and launches nothing.
 * All calls on one GPU share that array: calls ordered on one stream are safe back to back (each rewrites every
 * entry it reads; nothing has to start at zero), calls that overlap on different streams of one GPU race.
 */
int wf_op_attention_noalloc(int32_t precision, const void *qkv_dev, void *out_dev, const int32_t *cu_seqlens_host, int32_t B,
                            int32_t n_heads, void *hip_stream);

/*
 * Log-mel front end with the hush word appended at the raw-audio level (the step right before the
 * encoder).  Paper: raw audio is a 16 kHz one-dimensional array, 1 s of it is a (100, 80) log-mel matrix,
 * and the hush word is a fixed raw-audio vector of 8000 samples placed at the end of the audio before the
 * spectrogram is taken (Section "Hush word", position and target level; Section "Key Implementation
 * Details").  Everything else is this library's reading: periodic Hann window of 400 samples, frames
 * centred on multiples of 160 samples with 200 samples of reflect padding, 400-point DFT (201 bins),
 * power spectrum, n_mels unit-peak triangular filters equally spaced on the mel scale
 * 2595 log10(1 + f/700) over [0, 8000] Hz, log10 with floor 1e-10, clamp to within 8 decades of the
 * stream's maximum, then (v + 4) / 4.  Stream i with N_i samples yields floor((N_i + H) / 160) frames.
 *
 * wf_frontend_create   hush_audio: HOST fp32 [hush_samples] (copied), may be NULL iff hush_samples == 0.
 * wf_logmel_batch      audio_dev: DEVICE fp32 samples; sample_offset / n_samples: HOST [B] (first sample of
 *                      stream i inside audio_dev, and N_i); mel_out_dev: DEVICE [sum T'_i, n_mels] packed
 *                      stream-major, dtype mel_dtype (WF_DTYPE_*), directly usable as wf_encode_batch input
 *                      (with an encoder created with hush_frames = 0); cu_frames_host: HOST [B+1], may be
 *                      NULL.  Asynchronous on hip_stream.  WF_E_INVALID_ARG if N_i + H < 201 (shorter than
 *                      the reflect padding) or N_i < 0; WF_E_CAPACITY beyond max_streams / max_total_samples
 *                      (sum of N_i + H) / mel_capacity_frames.
 */
typedef struct wf_frontend wf_frontend;
typedef struct {
  int32_t n_mels;               /* 1 .. 256 */
  int32_t hush_samples;         /* H >= 0 */
  int32_t max_streams;
  int64_t max_total_samples;    /* capacity: sum over streams of (N_i + H) */
} wf_frontend_config;

int wf_frontend_create(const wf_frontend_config *cfg, const float *hush_audio, wf_frontend **out);
int wf_logmel_batch(wf_frontend *fe, const float *audio_dev, const int64_t *sample_offset, const int32_t *n_samples,
                    int32_t B, void *mel_out_dev, int32_t mel_dtype, int64_t mel_capacity_frames,
                    int32_t *cu_frames_host, void *hip_stream);
void wf_frontend_destroy(wf_frontend *fe);

/* ---- Decoder-side consumers of the encoder states ---------------------------------------------------
 * The two dense steps that follow the encoder in a processing round and stay on the GPU (paper Section
 * "Operations", workload mapping; Section "CPU/GPU pipelining", categorization of workloads, item (2):
 * about 100 prompt tokens pass through the decoder in one parallel pass):
 *   wf_cross_kv   every decoder layer projects the packed encoder states once into the keys and values
 *                 its cross-attention reads for the rest of the round: K_l = E Wk_l^T, V_l = E Wv_l^T + bv_l;
 *   wf_prefill    the prompt tokens of every stream go through the decoder stack in one pass: token
 *                 embedding + learned position, then per layer LayerNorm -> causal self-attention ->
 *                 residual, LayerNorm -> cross-attention over that stream's encoder tokens -> residual,
 *                 LayerNorm -> GELU MLP -> residual; final LayerNorm; logits of each stream's last prompt
 *                 position against the (tied) token-embedding matrix.
 * The decoder internals are not spelled out in the paper; this is the standard pre-LN encoder-decoder
 * transformer matching the encoder above (key projections without bias, softmax scale 1/8, exact GELU).
 *
 * Layouts.  Element type "act" is bf16 for WF_PRECISION_BF16 and fp32 for WF_PRECISION_F32.
 *   enc_dev        DEVICE [M, d_model] act, packed stream-major as wf_encode_batch writes it;
 *   cu_seqlens     HOST [B+1] encoder-token prefix sums (cu_seqlens[0] == 0, every stream >= 1 token);
 *   cross_kv_dev   DEVICE act, caller-owned: layer l occupies [kv_capacity_tokens, 2 d_model] starting at
 *                  element l * kv_capacity_tokens * 2 d_model; row m = key (first d_model) | value of token m;
 *   tokens         HOST int32 [sum P_i] prompt token ids, stream-major; cu_prompt HOST [B+1] prefix sums
 *                  (1 <= P_i <= n_ctx, ids in [0, n_vocab));
 *   hidden_out_dev DEVICE [sum P_i, d_model], dtype hidden_dtype (WF_DTYPE_*), may be NULL;
 *   logits_out_dev DEVICE fp32 [B, n_vocab], may be NULL;
 *   self_kv_out_dev DEVICE act, may be NULL: layer l occupies [self_kv_capacity_tokens, 2 d_model] like
 *                  cross_kv_dev, row r = self-attention key | value of prompt token r (what token-by-token
 *                  decoding continues from).
 * Weights: HOST fp32 row-major [out, in], copied (and converted) at create.  All calls are asynchronous on
 * hip_stream; one decoder object is not re-entrant.  Errors: WF_E_INVALID_ARG (NULL, bad lengths or ids,
 * d_model/n_heads != 64), WF_E_CAPACITY (max_streams, max_enc_tokens, max_prompt_tokens, a caller capacity).
 */
typedef struct wf_decoder wf_decoder;
typedef struct {
  int32_t d_model, n_layers, n_heads, d_mlp, n_vocab, n_ctx;
  int32_t max_streams;
  int32_t max_enc_tokens;       /* capacity: total encoder tokens per call */
  int32_t max_prompt_tokens;    /* capacity: total prompt tokens per call */
  int32_t precision;            /* WF_PRECISION_* */
  float ln_eps;                 /* <= 0 selects 1e-5 */
} wf_decoder_config;

typedef struct {
  const float *ln1_g, *ln1_b;                         /* before self-attention */
  const float *wq, *bq, *wk, *wv, *bv, *wo, *bo;      /* self-attention, [d, d] each */
  const float *lnx_g, *lnx_b;                         /* before cross-attention */
  const float *xwq, *xbq, *xwk, *xwv, *xbv, *xwo, *xbo;
  const float *ln2_g, *ln2_b;                         /* before the MLP */
  const float *w1 /* [d_mlp, d] */, *b1, *w2 /* [d, d_mlp] */, *b2;
} wf_decoder_layer_weights;

typedef struct {
  const float *tok_emb;         /* [n_vocab, d_model] */
  const float *pos_emb;         /* [n_ctx, d_model] */
  const wf_decoder_layer_weights *layers;   /* [n_layers] */
  const float *lnf_g, *lnf_b;
} wf_decoder_weights;

int wf_decoder_config_check(const wf_decoder_config *cfg);
int wf_decoder_create(const wf_decoder_config *cfg, const wf_decoder_weights *w, wf_decoder **out);
int wf_cross_kv(wf_decoder *dec, const void *enc_dev, int32_t M, void *cross_kv_dev, int64_t kv_capacity_tokens,
                void *hip_stream);
int wf_prefill(wf_decoder *dec, const int32_t *tokens, const int32_t *cu_prompt, const int32_t *cu_seqlens, int32_t B,
               const void *cross_kv_dev, int64_t kv_capacity_tokens, void *hidden_out_dev, int32_t hidden_dtype,
               float *logits_out_dev, void *self_kv_out_dev, int64_t self_kv_capacity_tokens, void *hip_stream);
void wf_decoder_destroy(wf_decoder *dec);          /* NULL-safe */
int wf_decoder_kernel_class_count(void);
int wf_decoder_set_profiling(wf_decoder *dec, int32_t enabled);
int wf_decoder_kernel_stats(wf_decoder *dec, wf_kernel_stat *stats, int32_t n_stats);

/* ---- Processing rounds over many concurrent streams ---------------------------------------------------
 * Host-side bookkeeping of the paper's online operation (Section "Operations": each round snapshots the
 * audio buffers; output is materialized once two consecutive rounds agree (LocalAgreement-2); buffers are
 * trimmed of materialized audio; a word's latency = wait until the next round + at least two rounds.
 * Section "Key Implementation Details": step length; below a round's processing time the rounds run back
 * to back, "best effort"), and a driver that runs such rounds through an encoder, one ragged batch per
 * round.  Integers throughout: times in microseconds, buffers in 10 ms frames.
 *
 * Rules.  Stream i ingests audio continuously from start_us[i].  Round k starts at s_0 = min(start_us) +
 * step_us, s_{k+1} = max(s_k + step_us, e_k), and ends at e_k = s_k + proc_k.  Its snapshot of stream i
 * holds n_i = floor((s_k - buffer start) / 10 ms) frames (0 before the stream starts; a buffer longer than
 * max_frames loses its oldest frames).  After round k, a buffer that held >= trim_frames frames drops the
 * frames that arrived before s_{k-1} (seen by two consecutive rounds, i.e. materialized) except
 * keep_frames of them.  Audio that arrived in (s_{k-1}, s_k] is first seen by round k and materialized at
 * e_{k+1}; mean_latency_us averages (materialization time - arrival time) over all such audio.
 *
 * wf_rounds_begin  opens the next round: *round_start_us = s_k, n_frames / first_frame: HOST [n_streams]
 *                  (first_frame = index, in the stream's own frame count since start_us[i], of the buffer's
 *                  first frame).  WF_E_INVALID_ARG if a round is already open.
 * wf_rounds_end    closes it with its processing time; *round_end_us (may be NULL) = e_k.
 * wf_run_rounds    runs n_rounds rounds: each round's active streams (n_i >= 1) are encoded as one ragged
 *                  batch by wf_encode_batch on hip_stream, the round's processing time is the wall-clock
 *                  time from planning to completion, and the virtual clock advances by it.  tracks_dev:
 *                  DEVICE [n_streams, track_frames, n_mels] (mel_dtype) synthetic per-stream feature tracks,
 *                  read circularly (track_frames > max_frames); pad_to_frames > 0 replaces every active
 *                  stream's length by pad_to_frames (the padded-window baseline; use an encoder without
 *                  hush).  out_dev receives the last round's states; records: HOST [n_rounds].
 */
typedef struct wf_rounds wf_rounds;
typedef struct {
  int32_t n_streams;
  int64_t step_us;              /* >= 1 */
  int32_t trim_frames;          /* 1 .. max_frames */
  int32_t keep_frames;          /* >= 0 */
  int32_t max_frames;           /* the model's window, 3000 = 30 s */
} wf_rounds_config;
typedef struct {
  int64_t rounds;
  double mean_latency_us, mean_proc_us;
  int64_t max_proc_us, frames_total, last_round_end_us;
} wf_rounds_stats;
typedef struct {
  int64_t start_us, end_us, proc_us;
  int64_t frames;               /* frames encoded this round (hush / padding included) */
  int64_t tokens;
  int32_t n_active, reserved;
} wf_round_record;

int wf_rounds_create(const wf_rounds_config *cfg, const int64_t *start_us, wf_rounds **out);
int wf_rounds_begin(wf_rounds *r, int64_t *round_start_us, int32_t *n_frames, int32_t *first_frame);
int wf_rounds_end(wf_rounds *r, int64_t proc_us, int64_t *round_end_us);
int wf_rounds_get_stats(const wf_rounds *r, wf_rounds_stats *stats);
int wf_rounds_reset_stats(wf_rounds *r);         /* statistics restart from here (e.g. after a warm-up); state is kept */
void wf_rounds_destroy(wf_rounds *r);            /* NULL-safe */
int wf_run_rounds(wf_rounds *r, wf_encoder *enc, const void *tracks_dev, int32_t mel_dtype, int64_t track_frames,
                  int32_t pad_to_frames, int32_t n_rounds, void *out_dev, int32_t out_dtype, int64_t out_capacity_tokens,
                  wf_round_record *records, void *hip_stream);

/* ---- Beam pruning ------------------------------------------------------------------------------------
 * The reference-based beam-size state machine of the paper's Section "Beam pruning" (search-based
 * reference alignment, selective transcript token matching and beam reduction, fallback mechanism).  Host
 * integer logic, no GPU call.  The reference is the token list of the previous processing round; each
 * wf_beam_pruner_step receives the highest-probability token of one decoding step of the current round.
 *   - the beam size starts at 1;
 *   - a punctuation token (listed in punct_ids) or a timestamp / special token (id >= special_from) is
 *     skipped: beam and reference index stay as they are.  That is all the paper exempts (the current best
 *     token).  With filter_reference != 0 such tokens are also left out of the reference list before any
 *     matching, so that an ordinary token never meets a punctuation or timestamp token on the reference side
 *     (an extension in the spirit of the rule's stated purpose); with filter_reference == 0 the reference is
 *     matched exactly as handed over (the paper's literal rule);
 *   - the first ordinary token is searched in the reference; its first occurrence i aligns the session
 *     (the next ordinary token is compared with reference token i + 1), no occurrence falls back;
 *   - afterwards an ordinary token equal to the reference token at the index keeps the beam at 1 and
 *     advances the index; a different one, or one arriving after the reference is used up, falls back;
 *   - a fallback restores the original beam size for the rest of the session.
 * Events: 0 skipped, 1 aligned, 2 matched, 3 fallback (alignment failed), 4 fallback (mismatch),
 * 5 fallback (reference used up), 6 already at the original beam size.
 *
 * wf_beam_pruner_create   ref_tokens HOST [n_ref] (n_ref >= 0, copied), punct_ids HOST [n_punct] (copied);
 *                         filter_reference: see above (it also applies to every later wf_beam_pruner_reset).
 * wf_beam_pruner_step     *event and *next_beam (either may be NULL): the event of this step and the beam
 *                         size the NEXT decoding step should run with.
 * wf_beam_pruner_reset    new decoding session against a new reference (same beam size and token classes).
 * wf_beam_prune_session   one whole session: best_tokens HOST [n]; beam_for_step / events HOST [n] (either may
 *                         be NULL): the beam size each step ran with and its event.
 */
typedef struct wf_beam_pruner wf_beam_pruner;
int wf_beam_pruner_create(int32_t beam_size, const int32_t *ref_tokens, int32_t n_ref, int32_t special_from,
                          const int32_t *punct_ids, int32_t n_punct, int32_t filter_reference, wf_beam_pruner **out);
int wf_beam_pruner_step(wf_beam_pruner *p, int32_t best_token, int32_t *event, int32_t *next_beam);
int wf_beam_pruner_reset(wf_beam_pruner *p, const int32_t *ref_tokens, int32_t n_ref);
int wf_beam_prune_session(wf_beam_pruner *p, const int32_t *best_tokens, int32_t n, int32_t *beam_for_step, int32_t *events);
void wf_beam_pruner_destroy(wf_beam_pruner *p);  /* NULL-safe */

#ifdef __cplusplus
}
#endif
#endif /* WF_ENCODER_H */
