// Host runtime of the ragged encoder: configuration checks, weight upload, the ragged-batch
// planner (prefix sums, attention work list) and the launch sequence behind the C ABI declared in
// include/wf_encoder.h.  Everything device-side is in the kernel files; this file only sequences
// them on the caller's stream.
#include "host_runtime.h"
#include "device_utils.h"

#include <cmath>
#include <mutex>
#include <new>

using namespace wf;
using namespace wf::host;

// ------------------------------------------------------------------------------------------------
// errors
namespace {
thread_local char g_err[512] = "";
}  // namespace

namespace wf {
// Same thread-local error text for every translation unit of the library.
int set_error(int code, const char *fmt, va_list ap) {
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  return code;
}
char *error_buffer() { return g_err; }
}  // namespace wf

#define HIP_TRY WF_HIP_TRY

namespace {

enum KClass : int {
  KC_PREP = 0, KC_CONV1, KC_CONV2, KC_LN, KC_QKV, KC_ATTN, KC_OUT, KC_FC1, KC_FC2, KC_LNF, KC_COUNT
};
const char *const kClassNames[KC_COUNT] = {"prep_pack_hush", "conv1_gemm_gelu", "conv2_gemm_gelu_pos", "layernorm",
                                           "gemm_qkv", "attention", "gemm_out_resid", "gemm_fc1_gelu",
                                           "gemm_fc2_resid", "layernorm_final"};

struct LayerDev {
  float *ln1_g, *ln1_b, *ln2_g, *ln2_b;
  void *wqkv, *wo, *w1, *w2;          // act dtype
  float *bqkv, *bo, *b1, *b2;
};

}  // namespace

constexpr int kMaxLanes = 4;

struct wf_encoder : DevCtx {
  wf_config cfg{};
  // Lanes (wf_encoder_set_lanes): the batch is cut into contiguous groups of streams that run the
  // whole layer sequence on streams of their own, so that one group's bandwidth-bound kernels and GEMM tails
  // overlap the other's matrix work.  Lane 0 is the caller's stream.
  int n_lanes = 2;
  hipStream_t lane_stream[kMaxLanes] = {};
  hipEvent_t lane_done[kMaxLanes] = {};
  hipEvent_t fork_evt = nullptr;
  int k1p = 0;                          // padded reduction length of the first convolution
  int64_t max_tokens = 0, max_work = 0, max_pos = 0;
  // weights
  void *conv1_w = nullptr, *conv2_w = nullptr, *hush = nullptr;
  float *conv1_b = nullptr, *conv2_b = nullptr, *lnf_g = nullptr, *lnf_b = nullptr, *pos = nullptr;
  std::vector<LayerDev> layers;
  // workspace
  void *packed = nullptr, *G = nullptr, *u = nullptr, *qkv = nullptr, *h = nullptr;
  float *x = nullptr;
  int32_t *frame_src = nullptr, *frame_flags = nullptr, *tok_src = nullptr, *tok_flags = nullptr, *tok_pos = nullptr;
  int32_t *idx_dev = nullptr;
  int64_t idx_ints = 0;
  // Replay cache for small batches (see wf_encoder_set_graphs): launch sequences captured as HIP graphs, keyed on
  // everything that shapes the launches or is baked into their arguments.
  struct GraphEntry {
    std::vector<int64_t> key;
    int32_t *idx = nullptr;              // this entry's own copy of the index arrays (device)
    hipGraphExec_t exec = nullptr;       // NULL: key seen once, nothing captured yet
    uint64_t last_use = 0;
  };
  std::vector<GraphEntry> graphs;
  bool graphs_enabled = false;
  hipStream_t cap_stream = nullptr;      // capture happens here, never on the caller's stream
  uint64_t graph_clock = 0;
  int64_t graph_replays = 0, graph_captures = 0, direct_calls = 0;
};

constexpr int kGraphCacheEntries = 64;

namespace {

// Convolution kernel [c_out, c_in, 3] -> GEMM weight [c_out, kp], column k*c_in + m = W[c, m, k],
// zero in the padding columns.
std::vector<float> conv_as_gemm_weight(const float *w, int c_out, int c_in, int kp) {
  std::vector<float> r((size_t)c_out * kp, 0.0f);
  for (int c = 0; c < c_out; ++c)
    for (int m = 0; m < c_in; ++m)
      for (int k = 0; k < 3; ++k) r[(size_t)c * kp + k * c_in + m] = w[((size_t)c * c_in + m) * 3 + k];
  return r;
}

struct Plan {
  int64_t total_frames = 0, total_tokens = 0;
};

// Shared by wf_plan_batch and wf_encode_batch: validates and fills cu_frames / cu_seqlens (either may be NULL).
int plan_batch(const wf_config &c, const int32_t *n_frames, int32_t B, int32_t *cu_frames, int32_t *cu_seqlens, Plan *plan) {
  if (!n_frames) return fail(WF_E_INVALID_ARG, "n_frames is NULL");
  if (B < 1) return fail(WF_E_INVALID_ARG, "B = %d, need B >= 1", B);
  if (B > c.max_streams) return fail(WF_E_CAPACITY, "B = %d exceeds max_streams = %d", B, c.max_streams);
  int64_t tf = 0, tt = 0;
  if (cu_frames) cu_frames[0] = 0;
  if (cu_seqlens) cu_seqlens[0] = 0;
  for (int i = 0; i < B; ++i) {
    const int64_t T = n_frames[i];
    if (T < 1) return fail(WF_E_INVALID_ARG, "n_frames[%d] = %lld, need >= 1", i, (long long)T);
    const int64_t Tp = T + c.hush_frames;
    if (Tp > c.max_frames_per_stream)
      return fail(WF_E_CAPACITY, "stream %d: %lld frames incl. hush exceed max_frames_per_stream = %d", i, (long long)Tp,
                  c.max_frames_per_stream);
    tf += Tp;
    tt += (Tp + 1) / 2;
    if (tf > c.max_total_frames)
      return fail(WF_E_CAPACITY, "total frames incl. hush exceed max_total_frames = %d (at stream %d)", c.max_total_frames, i);
    if (cu_frames) cu_frames[i + 1] = (int32_t)tf;
    if (cu_seqlens) cu_seqlens[i + 1] = (int32_t)tt;
  }
  plan->total_frames = tf;
  plan->total_tokens = tt;
  return WF_OK;
}

int check_config(const wf_config *c) {
  if (!c) return fail(WF_E_INVALID_ARG, "cfg is NULL");
  if (c->n_mels < 8 || c->n_mels % 8) return fail(WF_E_INVALID_ARG, "n_mels = %d must be a positive multiple of 8", c->n_mels);
  if (c->d_model < 128 || c->d_model % 128) return fail(WF_E_INVALID_ARG, "d_model = %d must be a positive multiple of 128", c->d_model);
  if (c->n_heads < 1 || c->d_model != c->n_heads * 64)
    return fail(WF_E_INVALID_ARG, "d_model / n_heads must be 64 (d_model = %d, n_heads = %d)", c->d_model, c->n_heads);
  if (c->d_mlp < 128 || c->d_mlp % 128) return fail(WF_E_INVALID_ARG, "d_mlp = %d must be a positive multiple of 128", c->d_mlp);
  if (c->n_layers < 0) return fail(WF_E_INVALID_ARG, "n_layers = %d", c->n_layers);
  if (c->hush_frames < 0) return fail(WF_E_INVALID_ARG, "hush_frames = %d", c->hush_frames);
  if (c->max_streams < 1) return fail(WF_E_INVALID_ARG, "max_streams = %d", c->max_streams);
  if (c->max_frames_per_stream < 1 + c->hush_frames)
    return fail(WF_E_INVALID_ARG, "max_frames_per_stream = %d cannot hold one frame plus the hush segment", c->max_frames_per_stream);
  if (c->max_frames_per_stream > (1 << 21) - 2)     // the attention work list keeps a query offset in 20 bits
    return fail(WF_E_INVALID_ARG, "max_frames_per_stream = %d exceeds the supported %d", c->max_frames_per_stream, (1 << 21) - 2);
  if (c->max_total_frames < c->max_frames_per_stream)
    return fail(WF_E_INVALID_ARG, "max_total_frames = %d < max_frames_per_stream = %d", c->max_total_frames, c->max_frames_per_stream);
  if (c->precision != WF_PRECISION_BF16 && c->precision != WF_PRECISION_F32)
    return fail(WF_E_INVALID_ARG, "precision = %d", c->precision);
  if (c->d_model > 2048) return fail(WF_E_INVALID_ARG, "d_model = %d exceeds the supported 2048", c->d_model);
  // the MFMA GEMMs address an operand with 32-bit byte offsets: the largest one (the MLP's hidden activations of a
  // full batch, rows padded to whole 256-row panels) must stay under 4 GiB
  const int64_t max_tokens = ((int64_t)c->max_total_frames + 1) / 2 + 256;
  const int64_t widest = c->d_mlp > c->d_model ? c->d_mlp : c->d_model;
  if (max_tokens * widest * 2 >= ((int64_t)1 << 32))
    return fail(WF_E_INVALID_ARG, "max_total_frames = %d with d_mlp = %d needs an activation matrix of 4 GiB or more; split the batch",
                c->max_total_frames, c->d_mlp);
  return WF_OK;
}

}  // namespace

// ------------------------------------------------------------------------------------------------
// public ABI
extern "C" {

const char *wf_last_error(void) { return g_err; }

int wf_config_check(const wf_config *cfg) { return check_config(cfg); }

int wf_plan_batch(const wf_config *cfg, const int32_t *n_frames, int32_t B, int32_t *cu_seqlens, int64_t *total_frames,
                  int64_t *total_tokens) {
  int rc = check_config(cfg);
  if (rc) return rc;
  Plan plan;
  rc = plan_batch(*cfg, n_frames, B, nullptr, cu_seqlens, &plan);
  if (rc) return rc;
  if (total_frames) *total_frames = plan.total_frames;
  if (total_tokens) *total_tokens = plan.total_tokens;
  return WF_OK;
}

int wf_kernel_class_count(void) { return KC_COUNT; }

void wf_encoder_destroy(wf_encoder *e) {
  if (!e) return;
  (void)hipSetDevice(e->device);
  (void)hipDeviceSynchronize();
  for (auto &g : e->graphs) {
    if (g.exec) (void)hipGraphExecDestroy(g.exec);
    if (g.idx) (void)hipFree(g.idx);
  }
  if (e->cap_stream) (void)hipStreamDestroy(e->cap_stream);
  release(e);
  for (int g = 1; g < kMaxLanes; ++g) {
    if (e->lane_stream[g]) (void)hipStreamDestroy(e->lane_stream[g]);
    if (e->lane_done[g]) (void)hipEventDestroy(e->lane_done[g]);
  }
  if (e->fork_evt) (void)hipEventDestroy(e->fork_evt);
  delete e;
}

static int create_impl(wf_encoder *e, const wf_config *cfg, const wf_weights *w) {
  e->cfg = *cfg;
  e->class_names = kClassNames;
  e->n_classes = KC_COUNT;
  if (e->cfg.ln_eps <= 0.0f) e->cfg.ln_eps = 1e-5f;
  e->bf16 = cfg->precision == WF_PRECISION_BF16;
  e->es = e->bf16 ? 2 : 4;
  HIP_TRY(hipGetDevice(&e->device));
  HIP_TRY(init_kernels());
  const int d = cfg->d_model, f = cfg->d_mlp, C = cfg->n_mels, H = cfg->hush_frames;
  e->k1p = (int)round_up(3 * C, 64);
  e->max_tokens = ((int64_t)cfg->max_total_frames + cfg->max_streams + 1) / 2;
  e->max_pos = (cfg->max_frames_per_stream + 1) / 2;
  e->max_work = e->max_tokens / attention_q_tile() + cfg->max_streams + 1;
  int rc;

  // ---- weights
  if ((rc = upload_w(e, &e->conv1_w, conv_as_gemm_weight(w->conv1_w, d, C, e->k1p)))) return rc;
  if ((rc = upload_w(e, &e->conv2_w, conv_as_gemm_weight(w->conv2_w, d, d, 3 * d)))) return rc;
  if ((rc = upload_f32(e, &e->conv1_b, w->conv1_b, d))) return rc;
  if ((rc = upload_f32(e, &e->conv2_b, w->conv2_b, d))) return rc;
  if ((rc = upload_f32(e, &e->lnf_g, w->lnf_g, d))) return rc;
  if ((rc = upload_f32(e, &e->lnf_b, w->lnf_b, d))) return rc;
  {
    std::vector<float> hm((size_t)std::max(H, 1) * C, 0.0f);
    if (H > 0) memcpy(hm.data(), w->hush_mel, (size_t)H * C * 4);
    if ((rc = upload_w(e, &e->hush, hm))) return rc;
  }
  {
    // Sinusoidal table in double, rounded once to fp32.
    const int half = d / 2;
    std::vector<float> P((size_t)e->max_pos * d);
    for (int c = 0; c < half; ++c) {
      const double omega = std::exp(-std::log(10000.0) * (double)c / (double)(half - 1));
      for (int64_t j = 0; j < e->max_pos; ++j) {
        P[(size_t)j * d + c] = (float)std::sin((double)j * omega);
        P[(size_t)j * d + half + c] = (float)std::cos((double)j * omega);
      }
    }
    if ((rc = upload_f32(e, &e->pos, P.data(), P.size()))) return rc;
  }
  e->layers.resize(cfg->n_layers);
  for (int l = 0; l < cfg->n_layers; ++l) {
    const wf_layer_weights &s = w->layers[l];
    LayerDev &t = e->layers[l];
    const float *req[] = {s.ln1_g, s.ln1_b, s.wq, s.bq, s.wk, s.wv, s.bv, s.wo, s.bo, s.ln2_g, s.ln2_b, s.w1, s.b1, s.w2, s.b2};
    for (const float *p : req)
      if (!p) return fail(WF_E_INVALID_ARG, "layer %d: a required weight pointer is NULL", l);
    std::vector<float> wqkv((size_t)3 * d * d), bqkv((size_t)3 * d, 0.0f);
    memcpy(wqkv.data(), s.wq, (size_t)d * d * 4);
    memcpy(wqkv.data() + (size_t)d * d, s.wk, (size_t)d * d * 4);
    memcpy(wqkv.data() + (size_t)2 * d * d, s.wv, (size_t)d * d * 4);
    memcpy(bqkv.data(), s.bq, (size_t)d * 4);
    if (s.bk) memcpy(bqkv.data() + d, s.bk, (size_t)d * 4);
    memcpy(bqkv.data() + 2 * d, s.bv, (size_t)d * 4);
    if (e->bf16) {     // the projection weights of the MFMA path live in panel layout
      if ((rc = upload_w_panels(e, &t.wqkv, wqkv.data(), 3 * d, d))) return rc;
      if ((rc = upload_w_panels(e, &t.wo, s.wo, d, d))) return rc;
      if ((rc = upload_w_panels(e, &t.w1, s.w1, f, d))) return rc;
      if ((rc = upload_w_panels(e, &t.w2, s.w2, d, f))) return rc;
    } else {
      if ((rc = upload_w(e, &t.wqkv, wqkv))) return rc;
      if ((rc = upload_w(e, &t.wo, std::vector<float>(s.wo, s.wo + (size_t)d * d)))) return rc;
      if ((rc = upload_w(e, &t.w1, std::vector<float>(s.w1, s.w1 + (size_t)f * d)))) return rc;
      if ((rc = upload_w(e, &t.w2, std::vector<float>(s.w2, s.w2 + (size_t)d * f)))) return rc;
    }
    if ((rc = upload_f32(e, &t.bqkv, bqkv.data(), bqkv.size()))) return rc;
    if ((rc = upload_f32(e, &t.bo, s.bo, d))) return rc;
    if ((rc = upload_f32(e, &t.b1, s.b1, f))) return rc;
    if ((rc = upload_f32(e, &t.b2, s.b2, d))) return rc;
    if ((rc = upload_f32(e, &t.ln1_g, s.ln1_g, d))) return rc;
    if ((rc = upload_f32(e, &t.ln1_b, s.ln1_b, d))) return rc;
    if ((rc = upload_f32(e, &t.ln2_g, s.ln2_g, d))) return rc;
    if ((rc = upload_f32(e, &t.ln2_b, s.ln2_b, d))) return rc;
  }

  // ---- workspace
  const int64_t F = cfg->max_total_frames, Mx = e->max_tokens;
  if ((rc = dev_alloc(e, &e->packed, (size_t)F * C * e->es))) return rc;
  if ((rc = dev_alloc(e, &e->G, (size_t)F * d * e->es))) return rc;
  if ((rc = dev_alloc(e, (void **)&e->x, (size_t)Mx * d * 4))) return rc;
  if ((rc = dev_alloc(e, &e->u, (size_t)Mx * d * e->es))) return rc;
  if ((rc = dev_alloc(e, &e->qkv, (size_t)Mx * 3 * d * e->es))) return rc;
  // the MLP's hidden activations are kept in panel layout on the bf16 path: whole 256-row panels per lane
  if ((rc = dev_alloc(e, &e->h, (size_t)(Mx + 256 * kMaxLanes) * f * e->es))) return rc;
  if ((rc = dev_alloc(e, (void **)&e->frame_src, (size_t)F * 4))) return rc;
  if ((rc = dev_alloc(e, (void **)&e->frame_flags, (size_t)F * 4))) return rc;
  if ((rc = dev_alloc(e, (void **)&e->tok_src, (size_t)Mx * 4))) return rc;
  if ((rc = dev_alloc(e, (void **)&e->tok_flags, (size_t)Mx * 4))) return rc;
  if ((rc = dev_alloc(e, (void **)&e->tok_pos, (size_t)Mx * 4))) return rc;
  e->idx_ints = 4 * ((int64_t)cfg->max_streams + 1) + 2 * e->max_work;
  if ((rc = dev_alloc(e, (void **)&e->idx_dev, (size_t)e->idx_ints * 4))) return rc;
  if ((rc = staging_create(e, (size_t)e->idx_ints))) return rc;
  for (int g = 1; g < kMaxLanes; ++g) {
    HIP_TRY(hipStreamCreateWithFlags(&e->lane_stream[g], hipStreamNonBlocking));
    HIP_TRY(hipEventCreateWithFlags(&e->lane_done[g], hipEventDisableTiming));
  }
  HIP_TRY(hipEventCreateWithFlags(&e->fork_evt, hipEventDisableTiming));
  HIP_TRY(hipStreamCreateWithFlags(&e->cap_stream, hipStreamNonBlocking));
  HIP_TRY(hipDeviceSynchronize());
  return WF_OK;
}

int wf_encoder_create(const wf_config *cfg, const wf_weights *w, wf_encoder **out) {
  if (!out) return fail(WF_E_INVALID_ARG, "out is NULL");
  *out = nullptr;
  int rc = check_config(cfg);
  if (rc) return rc;
  if (!w) return fail(WF_E_INVALID_ARG, "weights is NULL");
  if (!w->conv1_w || !w->conv1_b || !w->conv2_w || !w->conv2_b || !w->lnf_g || !w->lnf_b)
    return fail(WF_E_INVALID_ARG, "a stem or final-LayerNorm weight pointer is NULL");
  if (cfg->hush_frames > 0 && !w->hush_mel) return fail(WF_E_INVALID_ARG, "hush_mel is NULL but hush_frames = %d", cfg->hush_frames);
  if (cfg->n_layers > 0 && !w->layers) return fail(WF_E_INVALID_ARG, "layers is NULL but n_layers = %d", cfg->n_layers);
  wf_encoder *e = new (std::nothrow) wf_encoder();
  if (!e) return fail(WF_E_OOM, "host allocation failed");
  rc = create_impl(e, cfg, w);
  if (rc) {
    char keep[sizeof(g_err)];
    memcpy(keep, g_err, sizeof(keep));
    wf_encoder_destroy(e);
    memcpy(g_err, keep, sizeof(keep));
    return rc;
  }
  *out = e;
  return WF_OK;
}

int wf_encode_batch(wf_encoder *e, const void *mel_dev, int32_t mel_dtype, const int32_t *frame_offset, const int32_t *n_frames,
                    int32_t B, void *out_dev, int32_t out_dtype, int64_t out_capacity_tokens, int32_t *cu_seqlens_host,
                    void *hip_stream) {
  if (!e) return fail(WF_E_INVALID_ARG, "encoder is NULL");
  if (!mel_dev || !out_dev || !frame_offset) return fail(WF_E_INVALID_ARG, "mel_dev, out_dev or frame_offset is NULL");
  if (mel_dtype != WF_DTYPE_F32 && mel_dtype != WF_DTYPE_BF16) return fail(WF_E_INVALID_ARG, "mel_dtype = %d", mel_dtype);
  if (out_dtype != WF_DTYPE_F32 && out_dtype != WF_DTYPE_BF16) return fail(WF_E_INVALID_ARG, "out_dtype = %d", out_dtype);
  const wf_config &c = e->cfg;
  if (B >= 1 && B <= c.max_streams)
    for (int i = 0; i < B; ++i)
      if (frame_offset[i] < 0) return fail(WF_E_INVALID_ARG, "frame_offset[%d] = %d is negative", i, frame_offset[i]);

  // ---- plan on the host, into the next pinned staging slot
  int slot;
  int32_t *hs;
  int rc = staging_acquire(e, &slot, &hs);
  if (rc) return rc;
  const int S1 = c.max_streams + 1;
  int32_t *h_cu_frames = hs, *h_cu_seq = hs + S1, *h_off = hs + 2 * S1, *h_nf = hs + 3 * S1, *h_work = hs + 4 * S1;
  Plan plan;
  rc = plan_batch(c, n_frames, B, h_cu_frames, h_cu_seq, &plan);
  if (rc) return rc;
  const int M = (int)plan.total_tokens, TF = (int)plan.total_frames;
  if (M > out_capacity_tokens)
    return fail(WF_E_CAPACITY, "batch produces %d tokens but out_capacity_tokens = %lld", M, (long long)out_capacity_tokens);
  memcpy(h_off, frame_offset, (size_t)B * 4);
  memcpy(h_nf, n_frames, (size_t)B * 4);
  // ---- lanes: contiguous groups of streams with about the same number of tokens each
  int n_lanes = std::min(std::min(e->n_lanes, B), std::max(1, M / 4096));
  if (!e->bf16) n_lanes = 1;             // the fp32 debug attention walks every row of the batch
  int lane_b[kMaxLanes + 1], lane_w0[kMaxLanes + 1];
  lane_b[0] = 0;
  lane_w0[0] = 0;
  {
    int b = 0;
    for (int g = 0; g < n_lanes; ++g) {
      const int64_t target = (int64_t)M * (g + 1) / n_lanes;
      int nb = b;
      while (nb < B && (nb == b || h_cu_seq[nb + 1] <= target || g == n_lanes - 1)) ++nb;   // at least one stream each
      if (B - nb < n_lanes - 1 - g) nb = B - (n_lanes - 1 - g);                                // leave one for every later lane
      lane_b[g + 1] = nb;
      lane_w0[g + 1] = lane_w0[g] + build_work(h_cu_seq + b, nb - b, attention_q_tile(), h_work + 2 * lane_w0[g], nullptr, b);
      b = nb;
    }
  }
  const int n_work = lane_w0[n_lanes];
  if (cu_seqlens_host) memcpy(cu_seqlens_host, h_cu_seq, (size_t)(B + 1) * 4);

  const size_t idx_bytes = (size_t)(4 * S1 + 2 * n_work) * 4;

  // The launch sequence on stream s, reading the index arrays at idx_base (device).
  auto enqueue = [&](hipStream_t s, const int32_t *idx_base) -> int {
  const int32_t *d_cu_frames = idx_base, *d_cu_seq = idx_base + S1, *d_off = idx_base + 2 * S1, *d_nf = idx_base + 3 * S1,
                *d_work = idx_base + 4 * S1;

  const int d = c.d_model, f = c.d_mlp, C = c.n_mels;
  const int act_bf16 = e->bf16 ? 1 : 0;
  const size_t es = e->es;

  // ---- a0: pack + hush append + row maps (whole batch, caller's stream)
  {
    PrepArgs a{};
    a.mel = mel_dev; a.hush = e->hush; a.packed = e->packed;
    a.cu_frames = d_cu_frames; a.cu_seqlens = d_cu_seq; a.frame_offset = d_off; a.n_frames = d_nf;
    a.frame_src = e->frame_src; a.frame_flags = e->frame_flags;
    a.tok_src = e->tok_src; a.tok_flags = e->tok_flags; a.tok_pos = e->tok_pos;
    a.B = B; a.n_mels = C; a.total_frames = TF; a.M = M; a.mel_is_bf16 = mel_dtype == WF_DTYPE_BF16;
    Scope sc(e, s, KC_PREP, 0.0, (double)TF * C * ((mel_dtype == WF_DTYPE_BF16 ? 2 : 4) + es) + 8.0 * TF + 12.0 * M);
    hipError_t err = launch_prep(a, act_bf16, s);
    if (err != hipSuccess) return fail(WF_E_HIP, "prep launch: %s", hipGetErrorString(err));
  }
  if (n_lanes > 1) HIP_TRY(hipEventRecord(e->fork_evt, s));

  // ---- a1 .. a9 for the streams [b0, b1) on stream ls
  auto run_lane = [&](hipStream_t ls, int b0, int b1, const int32_t *work, int nw, int64_t h_row0) -> int {
    const int f0 = h_cu_frames[b0], Fg = h_cu_frames[b1] - f0;      // frames of the group
    const int r0 = h_cu_seq[b0], Mg = h_cu_seq[b1] - r0;            // tokens of the group
    const int Bg = b1 - b0;
    char *G = (char *)e->G + (size_t)f0 * d * es;
    float *x = e->x + (size_t)r0 * d;
    char *u = (char *)e->u + (size_t)r0 * d * es;
    char *qkv = (char *)e->qkv + (size_t)r0 * 3 * d * es;
    char *hbuf = (char *)e->h + (size_t)h_row0 * f * es;           // panel-aligned start of this lane's hidden activations
    const int panels = e->bf16 ? 1 : 0;                            // the fp32 debug kernels keep everything row-major
    // A group of at most about a thousand tokens runs on the small-batch GEMM (all of its products, so that a row's
    // arithmetic does not depend on which other streams share the batch), which also normalises its activation
    // operand itself: the two LayerNorm launches of a block disappear and the MLP's hidden activations stay row-major.
    const bool small = e->bf16 && gemm_small_applies(Mg);
    const int hpanels = small ? 0 : panels;
    int rc;
    {   // a1: conv1 + GELU as a GEMM over 3-frame windows (row maps hold absolute rows of the packed input)
      GemmArgs a{};
      a.A = e->packed; a.W = e->conv1_w; a.bias = e->conv1_b; a.out = G;
      a.M = Fg; a.N = d; a.K = e->k1p; a.lda = C; a.ldo = d;
      a.row_src = e->frame_src + f0; a.row_flags = e->frame_flags + f0; a.C = C;
      a.prefer_small = small;
      if ((rc = run_gemm(e, ls, KC_CONV1, a, A_CONV3, EPI_BIAS_GELU, 3 * C, (int)es, Fg, C))) return rc;
    }
    {   // a2: conv2 (stride 2) + GELU + positions -> fp32 residual stream
      GemmArgs a{};
      a.A = e->G; a.W = e->conv2_w; a.bias = e->conv2_b; a.out = x;
      a.M = Mg; a.N = d; a.K = 3 * d; a.lda = d; a.ldo = d;
      a.row_src = e->tok_src + r0; a.row_flags = e->tok_flags + r0; a.C = d;
      a.pos = e->pos; a.row_pos = e->tok_pos + r0;
      if ((rc = run_gemm(e, ls, KC_CONV2, a, A_CONV3, EPI_BIAS_GELU_POS, 3 * d, 4, Fg, d))) return rc;
    }
    double attn_flops = 0.0;
    for (int i = b0; i < b1; ++i) {
      const double L = h_cu_seq[i + 1] - h_cu_seq[i];
      attn_flops += 4.0 * L * L * d;
    }
    for (int l = 0; l < c.n_layers; ++l) {
      const LayerDev &w = e->layers[l];
      if (!small && (rc = run_ln(e, ls, KC_LN, x, w.ln1_g, w.ln1_b, u, act_bf16, Mg, d, c.ln_eps))) return rc;
      {
        GemmArgs a{};
        a.A = u; a.W = w.wqkv; a.bias = w.bqkv; a.out = qkv; a.M = Mg; a.N = 3 * d; a.K = d; a.lda = d; a.ldo = 3 * d;
        a.w_panels = panels;
        if (small) { a.A = x; a.ln_g = w.ln1_g; a.ln_b = w.ln1_b; a.ln_eps = c.ln_eps; }
        if ((rc = run_gemm(e, ls, KC_QKV, a, small ? A_LN : A_PLAIN, EPI_BIAS, d, (int)es, Mg, d))) return rc;
      }
      {
        AttnArgs a{};   // q, k, v and out are addressed through the absolute prefix sums, so the bases stay whole-batch
        a.q = e->qkv; a.k = (const char *)e->qkv + (size_t)d * es; a.v = (const char *)e->qkv + (size_t)2 * d * es;
        a.ldq = a.ldkv = 3 * d; a.out = e->u; a.cu_q = a.cu_kv = d_cu_seq; a.work = work;
        a.n_work = nw; a.n_heads = c.n_heads; a.d_model = d; a.B = B; a.M = M;
        a.scale = 0.125f;
        Scope sc(e, ls, KC_ATTN, attn_flops, (double)Mg * 4 * d * es);
        hipError_t err = e->bf16 ? launch_attention_bf16(a, ls) : launch_attention_f32(a, ls);
        if (err != hipSuccess) return fail(WF_E_HIP, "attention launch: %s", hipGetErrorString(err));
      }
      {
        GemmArgs a{};
        a.A = u; a.W = w.wo; a.bias = w.bo; a.out = x; a.M = Mg; a.N = d; a.K = d; a.lda = d; a.ldo = d;
        a.w_panels = panels;
        if ((rc = run_gemm(e, ls, KC_OUT, a, A_PLAIN, EPI_BIAS_RESID, d, 4, Mg, d))) return rc;
      }
      if (!small && (rc = run_ln(e, ls, KC_LN, x, w.ln2_g, w.ln2_b, u, act_bf16, Mg, d, c.ln_eps))) return rc;
      {   // fc1 writes the hidden activations as [rows/256][f/64][256][64] panels: one contiguous 32 KB block per
          // K step of fc2's activation operand (whose rows would otherwise be 2 f bytes apart in memory)
        GemmArgs a{};
        a.A = u; a.W = w.w1; a.bias = w.b1; a.out = hbuf; a.M = Mg; a.N = f; a.K = d; a.lda = d; a.ldo = f;
        a.out_panels = hpanels; a.w_panels = panels;
        if (small) { a.A = x; a.ln_g = w.ln2_g; a.ln_b = w.ln2_b; a.ln_eps = c.ln_eps; }
        if ((rc = run_gemm(e, ls, KC_FC1, a, small ? A_LN : A_PLAIN, EPI_BIAS_GELU, d, (int)es, Mg, d))) return rc;
      }
      {
        GemmArgs a{};
        a.A = hbuf; a.W = w.w2; a.bias = w.b2; a.out = x; a.M = Mg; a.N = d; a.K = f; a.lda = f; a.ldo = d;
        a.a_panels = hpanels; a.w_panels = panels;
        if ((rc = run_gemm(e, ls, KC_FC2, a, A_PLAIN, EPI_BIAS_RESID, f, 4, Mg, f))) return rc;
      }
    }
    // a9: final LayerNorm straight into the caller's buffer
    char *out = (char *)out_dev + (size_t)r0 * d * (out_dtype == WF_DTYPE_BF16 ? 2 : 4);
    (void)Bg;
    return run_ln(e, ls, KC_LNF, x, e->lnf_g, e->lnf_b, out, out_dtype == WF_DTYPE_BF16, Mg, d, c.ln_eps);
  };

  int64_t h_row0[kMaxLanes + 1];                           // every lane's hidden activations start on a panel boundary
  h_row0[0] = 0;
  for (int g = 0; g < n_lanes; ++g)
    h_row0[g + 1] = h_row0[g] + round_up(h_cu_seq[lane_b[g + 1]] - h_cu_seq[lane_b[g]], 256);
  // A failure part-way leaves kernels of the lanes already enqueued in flight on the encoder's own streams.  They
  // are joined back into the caller's stream on every path, so that whatever the caller (or the next call on this
  // encoder, which shares the workspace) enqueues on `s` afterwards is ordered after them.
  int first_err = WF_OK;
  char err_text[512] = "";
  auto note = [&](int code) {
    if (code != WF_OK && first_err == WF_OK) {
      first_err = code;
      snprintf(err_text, sizeof(err_text), "%s", g_err);
    }
  };
  auto hip_note = [&](hipError_t err, const char *what) {
    if (err != hipSuccess) note(fail(WF_E_HIP, "%s: %s", what, hipGetErrorString(err)));
    return err == hipSuccess;
  };
  bool started[kMaxLanes] = {};
  for (int g = n_lanes - 1; g >= 0 && first_err == WF_OK; --g) {   // the caller's own lane is enqueued last
    hipStream_t ls = g == 0 ? s : e->lane_stream[g];
    if (g > 0 && !hip_note(hipStreamWaitEvent(ls, e->fork_evt, 0), "lane fork")) break;
    started[g] = g > 0;
    note(run_lane(ls, lane_b[g], lane_b[g + 1], d_work + 2 * lane_w0[g], lane_w0[g + 1] - lane_w0[g], h_row0[g]));
  }
  for (int g = 1; g < n_lanes; ++g) {
    if (!started[g]) continue;
    if (hip_note(hipEventRecord(e->lane_done[g], e->lane_stream[g]), "lane join (record)"))
      hip_note(hipStreamWaitEvent(s, e->lane_done[g], 0), "lane join (wait)");
    else
      (void)hipStreamSynchronize(e->lane_stream[g]);      // could not order it on the GPU: wait for it here
  }
  if (first_err != WF_OK) {
    snprintf(g_err, sizeof(g_err), "%s", err_text);
    return first_err;
  }
  return WF_OK;
  };   // enqueue

  hipStream_t s = (hipStream_t)hip_stream;
  // ---- small batches: replay a captured graph of the same launch sequence.  A batch of a few thousand tokens is
  // bound by the cost of issuing its 4 + 7 n_layers launches one by one; everything that shapes those launches or is
  // baked into their arguments (stream lengths and offsets, the two caller buffers, the dtypes) is the cache key, so
  // a replay needs no upload at all: each entry keeps its own device copy of the index arrays.  A key is captured
  // the second time it is seen; other batches take the direct path below.
  const bool graph_ok = e->graphs_enabled && e->bf16 && !e->profiling && n_lanes == 1;
  if (graph_ok) {
    std::vector<int64_t> key;
    key.reserve(2 * (size_t)B + 5);
    key.push_back(B);
    key.push_back((int64_t)(uintptr_t)mel_dev);
    key.push_back((int64_t)(uintptr_t)out_dev);
    key.push_back(mel_dtype);
    key.push_back(out_dtype);
    for (int i = 0; i < B; ++i) key.push_back(((int64_t)frame_offset[i] << 32) | (uint32_t)n_frames[i]);
    wf_encoder::GraphEntry *hit = nullptr;
    for (auto &g : e->graphs)
      if (g.key == key) { hit = &g; break; }
    if (hit && hit->exec) {
      hit->last_use = ++e->graph_clock;
      HIP_TRY(hipGraphLaunch(hit->exec, s));
      ++e->graph_replays;
      return WF_OK;
    }
    if (!hit) {                                   // first sighting: remember the key, run directly
      if ((int)e->graphs.size() >= kGraphCacheEntries) {
        size_t victim = 0;
        for (size_t i = 1; i < e->graphs.size(); ++i)
          if (e->graphs[i].last_use < e->graphs[victim].last_use) victim = i;
        wf_encoder::GraphEntry &v = e->graphs[victim];
        if (v.exec) {                             // may still be in flight: wait before tearing it down
          HIP_TRY(hipDeviceSynchronize());
          (void)hipGraphExecDestroy(v.exec);
          (void)hipFree(v.idx);
        }
        e->graphs.erase(e->graphs.begin() + (long)victim);
      }
      wf_encoder::GraphEntry g;
      g.key = std::move(key);
      g.last_use = ++e->graph_clock;
      e->graphs.push_back(std::move(g));
    } else {                                      // second sighting: capture, instantiate, replay
      hit->last_use = ++e->graph_clock;
      int32_t *idx = nullptr;
      HIP_TRY(hipMalloc((void **)&idx, idx_bytes));
      hipError_t err = hipMemcpy(idx, hs, idx_bytes, hipMemcpyHostToDevice);
      hipGraph_t graph = nullptr;
      hipGraphExec_t exec = nullptr;
      int erc = WF_OK;
      if (err == hipSuccess) err = hipStreamBeginCapture(e->cap_stream, hipStreamCaptureModeThreadLocal);
      if (err == hipSuccess) {
        erc = enqueue(e->cap_stream, idx);
        err = hipStreamEndCapture(e->cap_stream, &graph);          // always ends the capture, also after a failed launch
        if (err == hipSuccess && erc == WF_OK) err = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
        if (graph) (void)hipGraphDestroy(graph);
      }
      if (err != hipSuccess || erc != WF_OK || !exec) {
        if (exec) (void)hipGraphExecDestroy(exec);
        (void)hipFree(idx);
        (void)hipGetLastError();
        if (erc != WF_OK) return erc;
        if (err != hipSuccess) return fail(WF_E_HIP, "graph capture: %s", hipGetErrorString(err));
        return fail(WF_E_HIP, "graph capture produced no executable graph");
      }
      hit->idx = idx;
      hit->exec = exec;
      ++e->graph_captures;
      HIP_TRY(hipGraphLaunch(exec, s));
      ++e->graph_replays;
      return WF_OK;
    }
  }
  ++e->direct_calls;
  if ((rc = staging_submit(e, slot, e->idx_dev, idx_bytes, s))) return rc;
  return enqueue(s, e->idx_dev);
}

int wf_encoder_set_graphs(wf_encoder *e, int32_t enabled) {
  if (!e) return fail(WF_E_INVALID_ARG, "encoder is NULL");
  e->graphs_enabled = enabled != 0;
  return WF_OK;
}

int wf_encoder_graph_stats(const wf_encoder *e, int64_t *replays, int64_t *captures, int64_t *direct_calls) {
  if (!e) return fail(WF_E_INVALID_ARG, "encoder is NULL");
  if (replays) *replays = e->graph_replays;
  if (captures) *captures = e->graph_captures;
  if (direct_calls) *direct_calls = e->direct_calls;
  return WF_OK;
}

int wf_encoder_set_lanes(wf_encoder *e, int32_t n_lanes) {
  if (!e) return fail(WF_E_INVALID_ARG, "encoder is NULL");
  if (n_lanes < 1 || n_lanes > kMaxLanes) return fail(WF_E_INVALID_ARG, "n_lanes = %d, need 1 .. %d", n_lanes, (int)kMaxLanes);
  e->n_lanes = n_lanes;
  return WF_OK;
}

int wf_encoder_get_lanes(const wf_encoder *e) {
  if (!e) return fail(WF_E_INVALID_ARG, "encoder is NULL");
  return e->n_lanes;
}

int wf_encoder_get_config(const wf_encoder *e, wf_config *cfg) {
  if (!e || !cfg) return fail(WF_E_INVALID_ARG, "encoder or cfg is NULL");
  *cfg = e->cfg;
  return WF_OK;
}

int wf_encoder_set_profiling(wf_encoder *e, int32_t enabled) {
  if (!e) return fail(WF_E_INVALID_ARG, "encoder is NULL");
  e->profiling = enabled != 0;
  return WF_OK;
}

int wf_encoder_kernel_stats(wf_encoder *e, wf_kernel_stat *stats, int32_t n_stats) {
  if (!e || !stats) return fail(WF_E_INVALID_ARG, "encoder or stats is NULL");
  return collect_stats(e, stats, n_stats);
}

int wf_device_info(int32_t *compute_units, int32_t *clock_khz) {
  int dev = 0, v = 0;
  HIP_TRY(hipGetDevice(&dev));
  if (compute_units) {
    HIP_TRY(hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev));
    *compute_units = v;
  }
  if (clock_khz) {
    HIP_TRY(hipDeviceGetAttribute(&v, hipDeviceAttributeClockRate, dev));
    *clock_khz = v;
  }
  return WF_OK;
}

int wf_gemm_tile_map(int32_t M, int32_t N, int32_t tile_m, int32_t tile_n, int32_t *units, int32_t capacity) {
  if (!units || capacity < 0) return fail(WF_E_INVALID_ARG, "units is NULL or capacity negative");
  if (M < 1 || N < 1 || tile_m < 1 || tile_n < 2 || tile_n % 2 || N % tile_n) return fail(WF_E_INVALID_ARG, "need M, N >= 1 and N a multiple of an even tile_n");
  const int n = gemm_dl_tile_map(M, N, tile_m, tile_n, units, capacity);
  if (n < 0) return fail(WF_E_CAPACITY, "more work units than capacity = %d", capacity);
  return n;
}

int wf_gelu_host(const float *z, float *out, int32_t n) {
  if (n < 0 || (n > 0 && (!z || !out))) return fail(WF_E_INVALID_ARG, "NULL pointer or negative count");
  for (int32_t i = 0; i < n; ++i) out[i] = gelu_fast(z[i]);
  return WF_OK;
}

int wf_gemm_tile_choice(int32_t M, int32_t N, int32_t *tile_m, int32_t *tile_n) {
  if (!tile_m || !tile_n) return fail(WF_E_INVALID_ARG, "NULL pointer");
  if (M < 1 || N < 128 || N % 128) return fail(WF_E_INVALID_ARG, "need M >= 1 and N a positive multiple of 128");
  gemm_tile_choice(M, N, tile_m, tile_n);
  return WF_OK;
}

// ---- operator-level entry points -------------------------------------------------------------
int wf_op_linear(int32_t precision, const void *a_dev, const void *w_dev, const float *bias_dev, void *out_dev, int32_t M,
                 int32_t N, int32_t K, int32_t epilogue, void *hip_stream) {
  if (!a_dev || !w_dev || !bias_dev || !out_dev) return fail(WF_E_INVALID_ARG, "NULL pointer");
  if (M < 1 || N < 128 || N % 128 || K < 64 || K % 64) return fail(WF_E_INVALID_ARG, "need M >= 1, N %% 128 == 0, K %% 64 == 0");
  if (epilogue < 0 || epilogue > 2) return fail(WF_E_INVALID_ARG, "epilogue = %d", epilogue);
  if (precision == WF_PRECISION_BF16 && ((int64_t)M * K * 2 >= ((int64_t)1 << 32) || (int64_t)N * K * 2 >= ((int64_t)1 << 32)))
    return fail(WF_E_INVALID_ARG, "an operand of 4 GiB or more (M = %d, N = %d, K = %d): the bf16 GEMM addresses operands with 32-bit offsets", M, N, K);
  GemmArgs a{};
  a.A = a_dev; a.W = w_dev; a.bias = bias_dev; a.out = out_dev;
  a.M = M; a.N = N; a.K = K; a.lda = K; a.ldo = N;
  hipError_t err = precision == WF_PRECISION_BF16 ? launch_gemm_bf16(a, A_PLAIN, (Epilogue)epilogue, (hipStream_t)hip_stream)
                                                  : launch_gemm_f32(a, A_PLAIN, (Epilogue)epilogue, (hipStream_t)hip_stream);
  if (err != hipSuccess) return fail(WF_E_HIP, "linear launch: %s", hipGetErrorString(err));
  return WF_OK;
}

int wf_op_ln_linear(const float *x_dev, const float *g_dev, const float *b_dev, float eps, const void *w_dev, const float *bias_dev,
                    void *out_dev, int32_t M, int32_t N, int32_t K, int32_t epilogue, void *hip_stream) {
  if (!x_dev || !g_dev || !b_dev || !w_dev || !bias_dev || !out_dev) return fail(WF_E_INVALID_ARG, "NULL pointer");
  if (M < 1 || N < 128 || N % 128 || K < 64 || K % 64 || K > 2048) return fail(WF_E_INVALID_ARG, "need M >= 1, N %% 128 == 0, K %% 64 == 0, K <= 2048");
  if (!gemm_small_applies(M)) return fail(WF_E_CAPACITY, "M = %d: the fused LayerNorm operand exists for small batches only", M);
  if (epilogue < 0 || epilogue > 1) return fail(WF_E_INVALID_ARG, "epilogue = %d (0: bias, 1: bias + GELU)", epilogue);
  if (!(eps > 0.0f)) return fail(WF_E_INVALID_ARG, "eps must be positive");
  GemmArgs a{};
  a.A = x_dev; a.W = w_dev; a.bias = bias_dev; a.out = out_dev;
  a.M = M; a.N = N; a.K = K; a.lda = K; a.ldo = N;
  a.ln_g = g_dev; a.ln_b = b_dev; a.ln_eps = eps;
  hipError_t err = launch_gemm_bf16(a, A_LN, (Epilogue)epilogue, (hipStream_t)hip_stream);
  if (err != hipSuccess) return fail(WF_E_HIP, "ln_linear launch: %s", hipGetErrorString(err));
  return WF_OK;
}

int wf_op_layernorm(const float *x_dev, const float *g_dev, const float *b_dev, void *out_dev, int32_t out_dtype, int32_t M,
                    int32_t d, float eps, void *hip_stream) {
  if (!x_dev || !g_dev || !b_dev || !out_dev) return fail(WF_E_INVALID_ARG, "NULL pointer");
  if (M < 1 || d < 4 || d % 4 || d > 2048) return fail(WF_E_INVALID_ARG, "need M >= 1, d %% 4 == 0, d <= 2048");
  hipError_t err = launch_layernorm(x_dev, g_dev, b_dev, out_dev, out_dtype == WF_DTYPE_BF16, M, d, eps, (hipStream_t)hip_stream);
  if (err != hipSuccess) return fail(WF_E_HIP, "layernorm launch: %s", hipGetErrorString(err));
  return WF_OK;
}

int wf_op_attention(int32_t precision, const void *qkv_dev, void *out_dev, const int32_t *cu_seqlens_host, int32_t B,
                    int32_t n_heads, void *hip_stream) {
  if (!qkv_dev || !out_dev || !cu_seqlens_host) return fail(WF_E_INVALID_ARG, "NULL pointer");
  if (B < 1 || n_heads < 1 || cu_seqlens_host[0] != 0) return fail(WF_E_INVALID_ARG, "need B >= 1, n_heads >= 1, cu_seqlens[0] == 0");
  for (int i = 0; i < B; ++i)
    if (cu_seqlens_host[i + 1] <= cu_seqlens_host[i] || cu_seqlens_host[i + 1] - cu_seqlens_host[i] > (1 << 20))
      return fail(WF_E_INVALID_ARG, "stream %d: need 1 .. %d tokens", i, 1 << 20);
  const int M = cu_seqlens_host[B];
  const int qt = attention_q_tile();
  std::vector<int32_t> idx((size_t)(B + 1) + 2 * ((size_t)M / qt + B + 1));
  memcpy(idx.data(), cu_seqlens_host, (size_t)(B + 1) * 4);
  const int n_work = build_work(cu_seqlens_host, B, qt, idx.data() + B + 1);
  int32_t *d_idx = nullptr;
  HIP_TRY(hipMalloc((void **)&d_idx, idx.size() * 4));
  hipStream_t s = (hipStream_t)hip_stream;
  hipError_t err = hipMemcpyAsync(d_idx, idx.data(), idx.size() * 4, hipMemcpyHostToDevice, s);
  if (err == hipSuccess) {
    AttnArgs a{};
    const size_t es = precision == WF_PRECISION_BF16 ? 2 : 4;
    a.q = qkv_dev; a.k = (const char *)qkv_dev + (size_t)n_heads * 64 * es; a.v = (const char *)qkv_dev + (size_t)2 * n_heads * 64 * es;
    a.ldq = a.ldkv = 3 * n_heads * 64; a.out = out_dev; a.cu_q = a.cu_kv = d_idx; a.work = d_idx + B + 1;
    a.n_work = n_work; a.n_heads = n_heads; a.d_model = n_heads * 64; a.B = B; a.M = M; a.scale = 0.125f;
    err = precision == WF_PRECISION_BF16 ? launch_attention_bf16(a, s) : launch_attention_f32(a, s);
  }
  hipError_t err2 = hipStreamSynchronize(s);
  (void)hipFree(d_idx);
  if (err != hipSuccess) return fail(WF_E_HIP, "attention launch: %s", hipGetErrorString(err));
  if (err2 != hipSuccess) return fail(WF_E_HIP, "attention: %s", hipGetErrorString(err2));
  return WF_OK;
}

}  // extern "C"

// ------------------------------------------------------------------------------------------------
// wf_op_attention for callers that cannot allocate: the index memory (prefix sums + work list) that
// wf_op_attention gets from hipMalloc lives in a file-scope device array instead.
namespace {

constexpr int kScratchInts = 16384;                       // 64 KiB per GPU, held until the process ends
static __device__ __align__(256) int32_t scratch[kScratchInts];

constexpr int kMaxDevices = 16;
int32_t *g_scratch_ptr[kMaxDevices] = {};                 // device address of `scratch` on each GPU (the array's
std::mutex g_scratch_mu;                                  // name is only a host-side stand-in for the symbol)

// Device address of this GPU's copy of `scratch`, looked up once per device with that device current.
int scratch_address(int32_t **out) {
  int dev = 0;
  WF_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(WF_E_INVALID_ARG, "device %d: only devices 0 .. %d are supported", dev, kMaxDevices - 1);
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void *ptr = nullptr;
    WF_HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return fail(WF_E_HIP, "hipGetSymbolAddress returned a NULL address");
    g_scratch_ptr[dev] = (int32_t *)ptr;
  }
  *out = g_scratch_ptr[dev];
  return WF_OK;
}

// Host -> device transport of a few hundred ints without a copy engine, a staging buffer or a memset: the
// values ride in the kernel arguments.
constexpr int kFillChunk = 960;                           // ints per launch (kernel arguments are limited to 4 KiB)
struct FillArgs {
  int32_t n;
  int32_t v[kFillChunk];
};
__global__ void __launch_bounds__(256) fill_ints_kernel(int32_t *dst, FillArgs a) {
  for (int i = threadIdx.x; i < a.n; i += blockDim.x) dst[i] = a.v[i];
}

}  // namespace

extern "C" int wf_op_attention_noalloc(int32_t precision, const void *qkv_dev, void *out_dev, const int32_t *cu_seqlens_host, int32_t B,
                                       int32_t n_heads, void *hip_stream) {
  if (!qkv_dev || !out_dev || !cu_seqlens_host) return fail(WF_E_INVALID_ARG, "NULL pointer");
  if (precision != WF_PRECISION_BF16 && precision != WF_PRECISION_F32) return fail(WF_E_INVALID_ARG, "precision = %d", precision);
  if (B < 1 || n_heads < 1 || cu_seqlens_host[0] != 0) return fail(WF_E_INVALID_ARG, "need B >= 1, n_heads >= 1, cu_seqlens[0] == 0");
  constexpr int kMaxB = (kScratchInts - 1) / 3;          // every stream needs its prefix sum and at least one work item
  if (B > kMaxB) return fail(WF_E_CAPACITY, "B = %d exceeds the %d streams the %d-int index scratch can hold", B, kMaxB, kScratchInts);
  for (int i = 0; i < B; ++i)
    if (cu_seqlens_host[i + 1] <= cu_seqlens_host[i] || cu_seqlens_host[i + 1] - cu_seqlens_host[i] > (1 << 20))
      return fail(WF_E_INVALID_ARG, "stream %d: need 1 .. %d tokens", i, 1 << 20);
  const int M = cu_seqlens_host[B];
  const int qt = attention_q_tile();
  int64_t n_work = 0;
  for (int i = 0; i < B; ++i) n_work += (cu_seqlens_host[i + 1] - cu_seqlens_host[i] + qt - 1) / qt;
  const int64_t need = (int64_t)(B + 1) + 2 * n_work;
  if (need > kScratchInts)
    return fail(WF_E_CAPACITY, "B = %d streams with %lld query blocks need %lld ints of index scratch, the limit is %d "
                "(B + 1 + 2 * sum ceil(L_i / %d) <= %d); use wf_op_attention", B, (long long)n_work, (long long)need, kScratchInts, qt, kScratchInts);
  int32_t *d_idx = nullptr;
  int rc = scratch_address(&d_idx);
  if (rc) return rc;
  int32_t idx[kScratchInts];                              // host copy of the indices, on the stack: no heap use either
  int64_t keys[kMaxB];
  memcpy(idx, cu_seqlens_host, (size_t)(B + 1) * 4);
  const int nw = build_work_noalloc(cu_seqlens_host, B, qt, idx + B + 1, keys);
  hipStream_t s = (hipStream_t)hip_stream;
  for (int64_t off = 0; off < need; off += kFillChunk) {  // every entry this call reads is rewritten; nothing needs clearing
    FillArgs fa;
    fa.n = (int32_t)std::min<int64_t>(kFillChunk, need - off);
    memcpy(fa.v, idx + off, (size_t)fa.n * 4);
    hipLaunchKernelGGL(fill_ints_kernel, dim3(1), dim3(256), 0, s, d_idx + off, fa);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return fail(WF_E_HIP, "index fill launch: %s", hipGetErrorString(err));
  }
  AttnArgs a{};
  const size_t es = precision == WF_PRECISION_BF16 ? 2 : 4;
  a.q = qkv_dev; a.k = (const char *)qkv_dev + (size_t)n_heads * 64 * es; a.v = (const char *)qkv_dev + (size_t)2 * n_heads * 64 * es;
  a.ldq = a.ldkv = 3 * n_heads * 64; a.out = out_dev; a.cu_q = a.cu_kv = d_idx; a.work = d_idx + B + 1;
  a.n_work = nw; a.n_heads = n_heads; a.d_model = n_heads * 64; a.B = B; a.M = M; a.scale = 0.125f;
  hipError_t err = precision == WF_PRECISION_BF16 ? launch_attention_bf16(a, s) : launch_attention_f32(a, s);
  if (err != hipSuccess) return fail(WF_E_HIP, "attention launch: %s", hipGetErrorString(err));
  return WF_OK;
}

namespace wf {
hipError_t init_kernels() { return hipSuccess; }
}  // namespace wf
