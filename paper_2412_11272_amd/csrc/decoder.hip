// Host runtime of the decoder-side consumers of the encoder states: the per-layer cross-attention
// key/value projection and the prompt prefill (paper Section "Operations", workload mapping; Section
// "CPU/GPU pipelining", categorization of workloads, item (2)).  Both are sequences of the same
// kernels the encoder uses (GEMM with fused epilogues, LayerNorm, ragged attention) plus an embedding
// lookup and a row gather; this file validates the ragged batch on the host and sequences the launches
// on the caller's stream behind the C ABI declared in include/wf_encoder.h.
#include "host_runtime.h"

#include <new>

using namespace wf;
using namespace wf::host;

namespace {

enum DClass : int {
  DC_CROSS_KV = 0, DC_EMBED, DC_LN, DC_SELF_Q, DC_SELF_KV, DC_SELF_QKV, DC_SELF_ATTN, DC_SELF_OUT, DC_CROSS_Q, DC_CROSS_ATTN,
  DC_CROSS_OUT, DC_FC1, DC_FC2, DC_LNF, DC_LOGITS, DC_COUNT
};
const char *const kDecClassNames[DC_COUNT] = {
    "cross_kv_gemm", "embed", "layernorm", "gemm_self_q", "gemm_self_kv", "gemm_self_qkv", "attention_causal", "gemm_self_out_resid",
    "gemm_cross_q", "attention_cross", "gemm_cross_out_resid", "gemm_fc1_gelu", "gemm_fc2_resid", "layernorm_final",
    "gemm_logits"};

struct DecLayerDev {
  float *ln1_g, *ln1_b, *lnx_g, *lnx_b, *ln2_g, *ln2_b;
  void *wq, *wkv, *wo, *xwq, *xwkv, *xwo, *w1, *w2;     // act dtype; wkv / xwkv = [2d, d]: key rows then value rows
  float *bq, *bkv, *bo, *xbq, *xbkv, *xbo, *b1, *b2;    // bkv / xbkv = 0 | bv
  void *wqkv;                                           // bf16 path: [3d, d] = wq | wk | wv rows, one product for q, k and v
  float *bqkv;                                          //            bq | 0 | bv
};

}  // namespace

struct wf_decoder : DevCtx {
  wf_decoder_config cfg{};
  int vpad = 0;                         // n_vocab rounded up to the GEMM's tile width
  int64_t max_work = 0;
  void *tok_emb = nullptr;              // [vpad, d] act, zero rows beyond n_vocab
  float *pos_emb = nullptr, *zero_bias = nullptr, *lnf_g = nullptr, *lnf_b = nullptr;
  std::vector<DecLayerDev> layers;
  // workspace
  float *x = nullptr, *lbuf = nullptr;
  void *u = nullptr, *qbuf = nullptr, *skv = nullptr, *h = nullptr, *ulast = nullptr;
  int32_t *idx_dev = nullptr;
  int64_t idx_ints = 0;
};

namespace {

int check_dec_config(const wf_decoder_config *c) {
  if (!c) return fail(WF_E_INVALID_ARG, "cfg is NULL");
  if (c->d_model < 128 || c->d_model % 128 || c->d_model > 2048)
    return fail(WF_E_INVALID_ARG, "d_model = %d must be a multiple of 128 in [128, 2048]", c->d_model);
  if (c->n_heads < 1 || c->d_model != c->n_heads * 64)
    return fail(WF_E_INVALID_ARG, "d_model / n_heads must be 64 (d_model = %d, n_heads = %d)", c->d_model, c->n_heads);
  if (c->d_mlp < 128 || c->d_mlp % 128) return fail(WF_E_INVALID_ARG, "d_mlp = %d must be a positive multiple of 128", c->d_mlp);
  if (c->n_layers < 0) return fail(WF_E_INVALID_ARG, "n_layers = %d", c->n_layers);
  if (c->n_vocab < 1) return fail(WF_E_INVALID_ARG, "n_vocab = %d", c->n_vocab);
  if (c->n_ctx < 1 || c->n_ctx > (1 << 20)) return fail(WF_E_INVALID_ARG, "n_ctx = %d (supported: 1 .. %d)", c->n_ctx, 1 << 20);
  if (c->max_streams < 1) return fail(WF_E_INVALID_ARG, "max_streams = %d", c->max_streams);
  if (c->max_enc_tokens < 1) return fail(WF_E_INVALID_ARG, "max_enc_tokens = %d", c->max_enc_tokens);
  if (c->max_prompt_tokens < 1) return fail(WF_E_INVALID_ARG, "max_prompt_tokens = %d", c->max_prompt_tokens);
  if (c->precision != WF_PRECISION_BF16 && c->precision != WF_PRECISION_F32) return fail(WF_E_INVALID_ARG, "precision = %d", c->precision);
  return WF_OK;
}

// [2d, d] = rows of wk then rows of wv; bias 0 | bv.
int upload_kv(wf_decoder *e, void **w_dst, float **b_dst, const float *wk, const float *wv, const float *bv) {
  const size_t d = e->cfg.d_model;
  std::vector<float> w(2 * d * d), b(2 * d, 0.0f);
  memcpy(w.data(), wk, d * d * 4);
  memcpy(w.data() + d * d, wv, d * d * 4);
  memcpy(b.data() + d, bv, d * 4);
  int rc = upload_w(e, w_dst, w);
  if (rc) return rc;
  return upload_f32(e, b_dst, b.data(), b.size());
}

int dec_create_impl(wf_decoder *e, const wf_decoder_config *cfg, const wf_decoder_weights *w) {
  e->cfg = *cfg;
  e->class_names = kDecClassNames;
  e->n_classes = DC_COUNT;
  if (e->cfg.ln_eps <= 0.0f) e->cfg.ln_eps = 1e-5f;
  e->bf16 = cfg->precision == WF_PRECISION_BF16;
  e->es = e->bf16 ? 2 : 4;
  WF_HIP_TRY(hipGetDevice(&e->device));
  const size_t d = cfg->d_model, f = cfg->d_mlp, V = cfg->n_vocab;
  e->vpad = (int)round_up(cfg->n_vocab, 256);
  int rc;
  {
    std::vector<float> t((size_t)e->vpad * d, 0.0f);
    memcpy(t.data(), w->tok_emb, V * d * 4);
    if ((rc = upload_w(e, &e->tok_emb, t))) return rc;
    std::vector<float> z((size_t)e->vpad, 0.0f);
    if ((rc = upload_f32(e, &e->zero_bias, z.data(), z.size()))) return rc;
  }
  if ((rc = upload_f32(e, &e->pos_emb, w->pos_emb, (size_t)cfg->n_ctx * d))) return rc;
  if ((rc = upload_f32(e, &e->lnf_g, w->lnf_g, d))) return rc;
  if ((rc = upload_f32(e, &e->lnf_b, w->lnf_b, d))) return rc;
  e->layers.resize(cfg->n_layers);
  for (int l = 0; l < cfg->n_layers; ++l) {
    const wf_decoder_layer_weights &s = w->layers[l];
    DecLayerDev &t = e->layers[l];
    const float *req[] = {s.ln1_g, s.ln1_b, s.wq, s.bq, s.wk, s.wv, s.bv, s.wo, s.bo, s.lnx_g, s.lnx_b, s.xwq, s.xbq, s.xwk,
                          s.xwv, s.xbv, s.xwo, s.xbo, s.ln2_g, s.ln2_b, s.w1, s.b1, s.w2, s.b2};
    for (const float *p : req)
      if (!p) return fail(WF_E_INVALID_ARG, "decoder layer %d: a weight pointer is NULL", l);
    t.wq = t.wkv = t.wqkv = nullptr;
    t.bq = t.bkv = t.bqkv = nullptr;
    if (!e->bf16) {
      if ((rc = upload_w(e, &t.wq, s.wq, d * d)) || (rc = upload_f32(e, &t.bq, s.bq, d))) return rc;
      if ((rc = upload_kv(e, &t.wkv, &t.bkv, s.wk, s.wv, s.bv))) return rc;
    } else {
      std::vector<float> wf(3 * d * d), bf(3 * d, 0.0f);
      memcpy(wf.data(), s.wq, d * d * 4);
      memcpy(wf.data() + d * d, s.wk, d * d * 4);
      memcpy(wf.data() + 2 * d * d, s.wv, d * d * 4);
      memcpy(bf.data(), s.bq, d * 4);
      memcpy(bf.data() + 2 * d, s.bv, d * 4);
      if ((rc = upload_w(e, &t.wqkv, wf)) || (rc = upload_f32(e, &t.bqkv, bf.data(), bf.size()))) return rc;
    }
    if ((rc = upload_w(e, &t.wo, s.wo, d * d)) || (rc = upload_f32(e, &t.bo, s.bo, d))) return rc;
    if ((rc = upload_w(e, &t.xwq, s.xwq, d * d)) || (rc = upload_f32(e, &t.xbq, s.xbq, d))) return rc;
    if ((rc = upload_kv(e, &t.xwkv, &t.xbkv, s.xwk, s.xwv, s.xbv))) return rc;
    if ((rc = upload_w(e, &t.xwo, s.xwo, d * d)) || (rc = upload_f32(e, &t.xbo, s.xbo, d))) return rc;
    if ((rc = upload_w(e, &t.w1, s.w1, f * d)) || (rc = upload_f32(e, &t.b1, s.b1, f))) return rc;
    if ((rc = upload_w(e, &t.w2, s.w2, d * f)) || (rc = upload_f32(e, &t.b2, s.b2, d))) return rc;
    if ((rc = upload_f32(e, &t.ln1_g, s.ln1_g, d)) || (rc = upload_f32(e, &t.ln1_b, s.ln1_b, d))) return rc;
    if ((rc = upload_f32(e, &t.lnx_g, s.lnx_g, d)) || (rc = upload_f32(e, &t.lnx_b, s.lnx_b, d))) return rc;
    if ((rc = upload_f32(e, &t.ln2_g, s.ln2_g, d)) || (rc = upload_f32(e, &t.ln2_b, s.ln2_b, d))) return rc;
  }
  const size_t P = cfg->max_prompt_tokens, S = cfg->max_streams;
  if ((rc = dev_alloc(e, (void **)&e->x, P * d * 4))) return rc;
  if ((rc = dev_alloc(e, &e->u, P * d * e->es))) return rc;
  if ((rc = dev_alloc(e, &e->qbuf, P * d * e->es))) return rc;
  if ((rc = dev_alloc(e, &e->skv, P * 2 * d * e->es))) return rc;
  if ((rc = dev_alloc(e, &e->h, P * f * e->es))) return rc;
  if ((rc = dev_alloc(e, &e->ulast, S * d * e->es))) return rc;
  if ((rc = dev_alloc(e, (void **)&e->lbuf, S * (size_t)e->vpad * 4))) return rc;
  e->max_work = (int64_t)P / attention_q_tile() + (int64_t)S + 1;
  e->idx_ints = 2 * (int64_t)P + 3 * ((int64_t)S + 1) + 2 * e->max_work;
  if ((rc = dev_alloc(e, (void **)&e->idx_dev, (size_t)e->idx_ints * 4))) return rc;
  if ((rc = staging_create(e, (size_t)e->idx_ints))) return rc;
  WF_HIP_TRY(hipDeviceSynchronize());
  return WF_OK;
}

int run_attention(wf_decoder *e, hipStream_t s, int cls, const AttnArgs &a, double flops, double bytes) {
  Scope sc(e, s, cls, flops, bytes);
  hipError_t err = e->bf16 ? launch_attention_bf16(a, s) : launch_attention_f32(a, s);
  if (err != hipSuccess) return fail(WF_E_HIP, "%s launch: %s", kDecClassNames[cls], hipGetErrorString(err));
  return WF_OK;
}

}  // namespace

extern "C" {

int wf_decoder_config_check(const wf_decoder_config *cfg) { return check_dec_config(cfg); }

int wf_decoder_kernel_class_count(void) { return DC_COUNT; }

void wf_decoder_destroy(wf_decoder *e) {
  if (!e) return;
  release(e);
  delete e;
}

int wf_decoder_create(const wf_decoder_config *cfg, const wf_decoder_weights *w, wf_decoder **out) {
  if (!out) return fail(WF_E_INVALID_ARG, "out is NULL");
  *out = nullptr;
  int rc = check_dec_config(cfg);
  if (rc) return rc;
  if (!w) return fail(WF_E_INVALID_ARG, "weights is NULL");
  if (!w->tok_emb || !w->pos_emb || !w->lnf_g || !w->lnf_b) return fail(WF_E_INVALID_ARG, "an embedding or final-LayerNorm pointer is NULL");
  if (cfg->n_layers > 0 && !w->layers) return fail(WF_E_INVALID_ARG, "layers is NULL but n_layers = %d", cfg->n_layers);
  wf_decoder *e = new (std::nothrow) wf_decoder();
  if (!e) return fail(WF_E_OOM, "host allocation failed");
  rc = dec_create_impl(e, cfg, w);
  if (rc) {
    char keep[512];
    snprintf(keep, sizeof(keep), "%s", error_buffer());
    wf_decoder_destroy(e);
    snprintf(error_buffer(), 512, "%s", keep);
    return rc;
  }
  *out = e;
  return WF_OK;
}

int wf_decoder_set_profiling(wf_decoder *e, int32_t enabled) {
  if (!e) return fail(WF_E_INVALID_ARG, "decoder is NULL");
  e->profiling = enabled != 0;
  return WF_OK;
}

int wf_decoder_kernel_stats(wf_decoder *e, wf_kernel_stat *stats, int32_t n_stats) {
  if (!e || !stats) return fail(WF_E_INVALID_ARG, "decoder or stats is NULL");
  return collect_stats(e, stats, n_stats);
}

int wf_cross_kv(wf_decoder *e, const void *enc_dev, int32_t M, void *cross_kv_dev, int64_t kv_capacity_tokens, void *hip_stream) {
  if (!e) return fail(WF_E_INVALID_ARG, "decoder is NULL");
  if (!enc_dev || !cross_kv_dev) return fail(WF_E_INVALID_ARG, "enc_dev or cross_kv_dev is NULL");
  if (M < 1) return fail(WF_E_INVALID_ARG, "M = %d, need M >= 1", M);
  if (M > e->cfg.max_enc_tokens) return fail(WF_E_CAPACITY, "M = %d exceeds max_enc_tokens = %d", M, e->cfg.max_enc_tokens);
  if (M > kv_capacity_tokens) return fail(WF_E_CAPACITY, "M = %d exceeds kv_capacity_tokens = %lld", M, (long long)kv_capacity_tokens);
  hipStream_t s = (hipStream_t)hip_stream;
  const int d = e->cfg.d_model;
  for (int l = 0; l < e->cfg.n_layers; ++l) {
    const DecLayerDev &w = e->layers[l];
    char *dst = (char *)cross_kv_dev + (size_t)l * kv_capacity_tokens * 2 * d * e->es;
    int rc = run_linear(e, s, DC_CROSS_KV, enc_dev, d, w.xwkv, w.xbkv, dst, 2 * d, M, 2 * d, d, EPI_BIAS);
    if (rc) return rc;
  }
  return WF_OK;
}

int wf_prefill(wf_decoder *e, const int32_t *tokens, const int32_t *cu_prompt, const int32_t *cu_seqlens, int32_t B,
               const void *cross_kv_dev, int64_t kv_capacity_tokens, void *hidden_out_dev, int32_t hidden_dtype,
               float *logits_out_dev, void *self_kv_out_dev, int64_t self_kv_capacity_tokens, void *hip_stream) {
  if (!e) return fail(WF_E_INVALID_ARG, "decoder is NULL");
  if (!tokens || !cu_prompt || !cu_seqlens || !cross_kv_dev) return fail(WF_E_INVALID_ARG, "tokens, cu_prompt, cu_seqlens or cross_kv_dev is NULL");
  const wf_decoder_config &c = e->cfg;
  if (B < 1) return fail(WF_E_INVALID_ARG, "B = %d, need B >= 1", B);
  if (B > c.max_streams) return fail(WF_E_CAPACITY, "B = %d exceeds max_streams = %d", B, c.max_streams);
  if (hidden_out_dev && hidden_dtype != WF_DTYPE_F32 && hidden_dtype != WF_DTYPE_BF16) return fail(WF_E_INVALID_ARG, "hidden_dtype = %d", hidden_dtype);
  if (cu_prompt[0] != 0 || cu_seqlens[0] != 0) return fail(WF_E_INVALID_ARG, "cu_prompt[0] and cu_seqlens[0] must be 0");
  for (int i = 0; i < B; ++i) {
    const int64_t P = (int64_t)cu_prompt[i + 1] - cu_prompt[i], L = (int64_t)cu_seqlens[i + 1] - cu_seqlens[i];
    if (P < 1 || P > c.n_ctx) return fail(WF_E_INVALID_ARG, "stream %d: %lld prompt tokens, need 1 .. n_ctx = %d", i, (long long)P, c.n_ctx);
    if (L < 1) return fail(WF_E_INVALID_ARG, "stream %d has no encoder tokens", i);
    if (cu_prompt[i + 1] > c.max_prompt_tokens)
      return fail(WF_E_CAPACITY, "prompt tokens exceed max_prompt_tokens = %d (at stream %d)", c.max_prompt_tokens, i);
    if (cu_seqlens[i + 1] > c.max_enc_tokens)
      return fail(WF_E_CAPACITY, "encoder tokens exceed max_enc_tokens = %d (at stream %d)", c.max_enc_tokens, i);
  }
  const int Pt = cu_prompt[B], M = cu_seqlens[B];
  if (M > kv_capacity_tokens) return fail(WF_E_CAPACITY, "%d encoder tokens exceed kv_capacity_tokens = %lld", M, (long long)kv_capacity_tokens);
  if (self_kv_out_dev && Pt > self_kv_capacity_tokens)
    return fail(WF_E_CAPACITY, "%d prompt tokens exceed self_kv_capacity_tokens = %lld", Pt, (long long)self_kv_capacity_tokens);
  for (int r = 0; r < Pt; ++r)
    if (tokens[r] < 0 || tokens[r] >= c.n_vocab) return fail(WF_E_INVALID_ARG, "tokens[%d] = %d outside [0, %d)", r, tokens[r], c.n_vocab);

  // ---- index arrays: tok | pos | cu_prompt | cu_seqlens | last row | attention work list
  int slot;
  int32_t *hs;
  int rc = staging_acquire(e, &slot, &hs);
  if (rc) return rc;
  const int S1 = B + 1;
  int32_t *h_tok = hs, *h_pos = hs + Pt, *h_cup = hs + 2 * Pt, *h_cus = h_cup + S1, *h_last = h_cus + S1, *h_work = h_last + S1;
  memcpy(h_tok, tokens, (size_t)Pt * 4);
  memcpy(h_cup, cu_prompt, (size_t)S1 * 4);
  memcpy(h_cus, cu_seqlens, (size_t)S1 * 4);
  std::vector<int64_t> cost(B);
  double self_flops = 0.0, cross_flops = 0.0;
  const int d = c.d_model, f = c.d_mlp;
  for (int i = 0; i < B; ++i) {
    const int P = cu_prompt[i + 1] - cu_prompt[i], L = cu_seqlens[i + 1] - cu_seqlens[i];
    for (int t = 0; t < P; ++t) h_pos[cu_prompt[i] + t] = t;
    h_last[i] = cu_prompt[i + 1] - 1;
    cost[i] = (int64_t)P * L;
    self_flops += 2.0 * P * (P + 1.0) * d;        // each query sees (its position + 1) keys: 4 d sum_r (r+1)
    cross_flops += 4.0 * P * L * d;
  }
  h_last[B] = 0;
  const int n_work = build_work(h_cup, B, attention_q_tile(), h_work, cost.data());
  const size_t idx_ints = (size_t)2 * Pt + 3 * S1 + 2 * (size_t)n_work;
  hipStream_t s = (hipStream_t)hip_stream;
  if ((rc = staging_submit(e, slot, e->idx_dev, idx_ints * 4, s))) return rc;
  const int32_t *d_tok = e->idx_dev, *d_pos = d_tok + Pt, *d_cup = d_tok + 2 * Pt, *d_cus = d_cup + S1, *d_last = d_cus + S1,
                *d_work = d_last + S1;

  const int act_bf16 = e->bf16 ? 1 : 0;
  const size_t es = e->es;
  {
    Scope sc(e, s, DC_EMBED, 0.0, (double)Pt * d * (es + 4 + 4));
    hipError_t err = launch_embed(e->tok_emb, act_bf16, e->pos_emb, d_tok, d_pos, e->x, Pt, d, s);
    if (err != hipSuccess) return fail(WF_E_HIP, "embed launch: %s", hipGetErrorString(err));
  }
  for (int l = 0; l < c.n_layers; ++l) {
    const DecLayerDev &w = e->layers[l];
    char *skv = self_kv_out_dev ? (char *)self_kv_out_dev + (size_t)l * self_kv_capacity_tokens * 2 * d * es : (char *)e->skv;
    const char *xkv = (const char *)cross_kv_dev + (size_t)l * kv_capacity_tokens * 2 * d * es;
    // causal self-attention among the prompt tokens
    if ((rc = run_ln(e, s, DC_LN, e->x, w.ln1_g, w.ln1_b, e->u, act_bf16, Pt, d, c.ln_eps))) return rc;
    if (e->bf16) {     // one product for q | k | v: the first d result columns go to the query buffer, the rest to the K/V cache
      GemmArgs a{};
      a.A = e->u; a.W = w.wqkv; a.bias = w.bqkv; a.out = e->qbuf; a.M = Pt; a.N = 3 * d; a.K = d; a.lda = d; a.ldo = d;
      a.out2 = skv; a.n_split = d; a.ldo2 = 2 * d;
      if ((rc = run_gemm(e, s, DC_SELF_QKV, a, A_PLAIN, EPI_BIAS, d, (int)es, Pt, d))) return rc;
    } else {
      if ((rc = run_linear(e, s, DC_SELF_Q, e->u, d, w.wq, w.bq, e->qbuf, d, Pt, d, d, EPI_BIAS))) return rc;
      if ((rc = run_linear(e, s, DC_SELF_KV, e->u, d, w.wkv, w.bkv, skv, 2 * d, Pt, 2 * d, d, EPI_BIAS))) return rc;
    }
    {
      AttnArgs a{};
      a.q = e->qbuf; a.ldq = d; a.k = skv; a.v = skv + (size_t)d * es; a.ldkv = 2 * d; a.out = e->u;
      a.cu_q = d_cup; a.cu_kv = d_cup; a.work = d_work; a.n_work = n_work; a.n_heads = c.n_heads; a.d_model = d;
      a.B = B; a.M = Pt; a.causal = 1; a.scale = 0.125f;
      if ((rc = run_attention(e, s, DC_SELF_ATTN, a, self_flops, (double)Pt * 4 * d * es))) return rc;
    }
    if ((rc = run_linear(e, s, DC_SELF_OUT, e->u, d, w.wo, w.bo, e->x, d, Pt, d, d, EPI_BIAS_RESID))) return rc;
    // cross-attention over the stream's encoder tokens
    if ((rc = run_ln(e, s, DC_LN, e->x, w.lnx_g, w.lnx_b, e->u, act_bf16, Pt, d, c.ln_eps))) return rc;
    if ((rc = run_linear(e, s, DC_CROSS_Q, e->u, d, w.xwq, w.xbq, e->qbuf, d, Pt, d, d, EPI_BIAS))) return rc;
    {
      AttnArgs a{};
      a.q = e->qbuf; a.ldq = d; a.k = xkv; a.v = xkv + (size_t)d * es; a.ldkv = 2 * d; a.out = e->u;
      a.cu_q = d_cup; a.cu_kv = d_cus; a.work = d_work; a.n_work = n_work; a.n_heads = c.n_heads; a.d_model = d;
      a.B = B; a.M = Pt; a.causal = 0; a.scale = 0.125f;
      if ((rc = run_attention(e, s, DC_CROSS_ATTN, a, cross_flops, ((double)Pt * 2 + (double)M * 2) * d * es))) return rc;
    }
    if ((rc = run_linear(e, s, DC_CROSS_OUT, e->u, d, w.xwo, w.xbo, e->x, d, Pt, d, d, EPI_BIAS_RESID))) return rc;
    // MLP
    if ((rc = run_ln(e, s, DC_LN, e->x, w.ln2_g, w.ln2_b, e->u, act_bf16, Pt, d, c.ln_eps))) return rc;
    if ((rc = run_linear(e, s, DC_FC1, e->u, d, w.w1, w.b1, e->h, f, Pt, f, d, EPI_BIAS_GELU))) return rc;
    if ((rc = run_linear(e, s, DC_FC2, e->h, f, w.w2, w.b2, e->x, d, Pt, d, f, EPI_BIAS_RESID))) return rc;
  }
  if ((rc = run_ln(e, s, DC_LNF, e->x, e->lnf_g, e->lnf_b, e->u, act_bf16, Pt, d, c.ln_eps))) return rc;
  if (hidden_out_dev &&
      (rc = run_ln(e, s, DC_LNF, e->x, e->lnf_g, e->lnf_b, hidden_out_dev, hidden_dtype == WF_DTYPE_BF16, Pt, d, c.ln_eps)))
    return rc;
  if (logits_out_dev) {
    hipError_t err = launch_gather_rows(e->u, d_last, e->ulast, B, (int)(d * es), s);
    if (err != hipSuccess) return fail(WF_E_HIP, "gather launch: %s", hipGetErrorString(err));
    // (the weight-streaming logits product keeps the 128-wide tile even for a handful of rows: measured 46 us against
    // 63 us on the small-batch kernel for 64 x 51866 x 1280)
    {
      GemmArgs a{};
      a.A = e->ulast; a.W = e->tok_emb; a.bias = e->zero_bias; a.out = e->lbuf; a.M = B; a.N = e->vpad; a.K = d; a.lda = d; a.ldo = e->vpad;
      a.prefer_large = 1;
      if ((rc = run_gemm(e, s, DC_LOGITS, a, A_PLAIN, EPI_BIAS_F32, d, 4, B, d))) return rc;
      WF_HIP_TRY(hipMemcpy2DAsync(logits_out_dev, (size_t)c.n_vocab * 4, e->lbuf, (size_t)e->vpad * 4, (size_t)c.n_vocab * 4, B,
                                  hipMemcpyDeviceToDevice, s));
    }
  }
  return WF_OK;
}

}  // extern "C"
