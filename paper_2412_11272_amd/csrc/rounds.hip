// Processing rounds over many concurrent streams: the integer bookkeeping of snapshots, trimming and
// LocalAgreement-2 latency (paper Section "Operations"; Section "Key Implementation Details", step
// length and best-effort mode), and the driver that pushes each round's ragged batch through the
// encoder.  Host code only; the rules are stated with the declarations in include/wf_encoder.h.
#include "host_runtime.h"

#include <chrono>
#include <cmath>
#include <new>

using namespace wf::host;

namespace {
constexpr int64_t kFrameUs = 10000;
struct Interval { int64_t lo, hi; };
}  // namespace

struct wf_rounds {
  wf_rounds_config cfg{};
  std::vector<int64_t> start, buf_start;
  std::vector<int32_t> n_cur;
  std::vector<Interval> pending;       // arrivals of the previous round, materialized when the open round ends
  int64_t k = 0, s_prev = 0, e_prev = 0, s_cur = 0;
  bool open = false;
  unsigned __int128 lat2 = 0;          // sum of len * (2 e - lo - hi)
  int64_t len_total = 0, frames_total = 0, proc_total = 0, proc_max = 0;
  int64_t stat_k0 = 0;                 // rounds before the last wf_rounds_reset_stats
  // scratch for wf_run_rounds
  std::vector<int32_t> nf, ff, act_off, act_n, cu;
};

extern "C" {

int wf_rounds_create(const wf_rounds_config *cfg, const int64_t *start_us, wf_rounds **out) {
  if (!out) return fail(WF_E_INVALID_ARG, "out is NULL");
  *out = nullptr;
  if (!cfg || !start_us) return fail(WF_E_INVALID_ARG, "cfg or start_us is NULL");
  if (cfg->n_streams < 1) return fail(WF_E_INVALID_ARG, "n_streams = %d", cfg->n_streams);
  if (cfg->step_us < 1) return fail(WF_E_INVALID_ARG, "step_us = %lld, need >= 1", (long long)cfg->step_us);
  if (cfg->max_frames < 1 || cfg->trim_frames < 1 || cfg->trim_frames > cfg->max_frames || cfg->keep_frames < 0)
    return fail(WF_E_INVALID_ARG, "need 1 <= trim_frames <= max_frames and keep_frames >= 0 (got %d, %d, %d)", cfg->trim_frames,
                cfg->max_frames, cfg->keep_frames);
  for (int i = 0; i < cfg->n_streams; ++i)
    if (start_us[i] < 0) return fail(WF_E_INVALID_ARG, "start_us[%d] is negative", i);
  wf_rounds *r = new (std::nothrow) wf_rounds();
  if (!r) return fail(WF_E_OOM, "host allocation failed");
  r->cfg = *cfg;
  r->start.assign(start_us, start_us + cfg->n_streams);
  r->buf_start = r->start;
  r->n_cur.assign(cfg->n_streams, 0);
  *out = r;
  return WF_OK;
}

void wf_rounds_destroy(wf_rounds *r) { delete r; }

int wf_rounds_begin(wf_rounds *r, int64_t *round_start_us, int32_t *n_frames, int32_t *first_frame) {
  if (!r || !n_frames || !first_frame) return fail(WF_E_INVALID_ARG, "rounds, n_frames or first_frame is NULL");
  if (r->open) return fail(WF_E_INVALID_ARG, "a round is already open");
  const int S = r->cfg.n_streams;
  int64_t s;
  if (r->k == 0) {
    s = *std::min_element(r->start.begin(), r->start.end()) + r->cfg.step_us;
  } else {
    s = std::max(r->s_prev + r->cfg.step_us, r->e_prev);
  }
  for (int i = 0; i < S; ++i) {
    int64_t cnt = s > r->buf_start[i] ? (s - r->buf_start[i]) / kFrameUs : 0;
    if (cnt > r->cfg.max_frames) {
      r->buf_start[i] += (cnt - r->cfg.max_frames) * kFrameUs;
      cnt = r->cfg.max_frames;
    }
    n_frames[i] = r->n_cur[i] = (int32_t)cnt;
    first_frame[i] = (int32_t)((r->buf_start[i] - r->start[i]) / kFrameUs);
  }
  r->s_cur = s;
  r->open = true;
  if (round_start_us) *round_start_us = s;
  return WF_OK;
}

int wf_rounds_end(wf_rounds *r, int64_t proc_us, int64_t *round_end_us) {
  if (!r) return fail(WF_E_INVALID_ARG, "rounds is NULL");
  if (!r->open) return fail(WF_E_INVALID_ARG, "no round is open");
  if (proc_us < 0) return fail(WF_E_INVALID_ARG, "proc_us is negative");
  const int S = r->cfg.n_streams;
  const int64_t s = r->s_cur, e = s + proc_us;
  for (const Interval &iv : r->pending) {
    r->lat2 += (unsigned __int128)(iv.hi - iv.lo) * (unsigned __int128)(2 * e - iv.lo - iv.hi);
    r->len_total += iv.hi - iv.lo;
  }
  r->pending.clear();
  for (int i = 0; i < S; ++i) {
    const int64_t lo = r->k > 0 ? std::max(r->s_prev, r->start[i]) : r->start[i];
    if (s > lo) r->pending.push_back({lo, s});
  }
  if (r->k > 0) {
    for (int i = 0; i < S; ++i) {
      if (r->n_cur[i] < r->cfg.trim_frames) continue;
      const int64_t committed = r->s_prev > r->buf_start[i] ? (r->s_prev - r->buf_start[i]) / kFrameUs : 0;
      const int64_t drop = std::max<int64_t>(0, committed - r->cfg.keep_frames);
      r->buf_start[i] += drop * kFrameUs;
    }
  }
  for (int i = 0; i < S; ++i) r->frames_total += r->n_cur[i];
  r->proc_total += proc_us;
  r->proc_max = std::max(r->proc_max, proc_us);
  r->s_prev = s;
  r->e_prev = e;
  r->open = false;
  r->k += 1;
  if (round_end_us) *round_end_us = e;
  return WF_OK;
}

int wf_rounds_get_stats(const wf_rounds *r, wf_rounds_stats *st) {
  if (!r || !st) return fail(WF_E_INVALID_ARG, "rounds or stats is NULL");
  st->rounds = r->k - r->stat_k0;
  st->mean_latency_us = r->len_total > 0 ? (double)((long double)r->lat2 / (2.0L * (long double)r->len_total)) : 0.0;
  st->mean_proc_us = st->rounds > 0 ? (double)r->proc_total / (double)st->rounds : 0.0;
  st->max_proc_us = r->proc_max;
  st->frames_total = r->frames_total;
  st->last_round_end_us = r->k > 0 ? r->e_prev : 0;
  return WF_OK;
}

int wf_rounds_reset_stats(wf_rounds *r) {
  if (!r) return fail(WF_E_INVALID_ARG, "rounds is NULL");
  if (r->open) return fail(WF_E_INVALID_ARG, "a round is open");
  r->lat2 = 0;
  r->len_total = r->frames_total = r->proc_total = r->proc_max = 0;
  r->stat_k0 = r->k;
  return WF_OK;
}

int wf_run_rounds(wf_rounds *r, wf_encoder *enc, const void *tracks_dev, int32_t mel_dtype, int64_t track_frames,
                  int32_t pad_to_frames, int32_t n_rounds, void *out_dev, int32_t out_dtype, int64_t out_capacity_tokens,
                  wf_round_record *records, void *hip_stream) {
  if (!r || !enc || !tracks_dev || !out_dev || !records) return fail(WF_E_INVALID_ARG, "a pointer argument is NULL");
  if (n_rounds < 0 || pad_to_frames < 0) return fail(WF_E_INVALID_ARG, "n_rounds or pad_to_frames is negative");
  const int S = r->cfg.n_streams;
  const int64_t need = std::max<int64_t>(r->cfg.max_frames, pad_to_frames);
  if (track_frames <= need) return fail(WF_E_INVALID_ARG, "track_frames = %lld must exceed %lld", (long long)track_frames, (long long)need);
  if ((int64_t)S * track_frames > INT32_MAX) return fail(WF_E_CAPACITY, "tracks hold more than 2^31 frames");
  r->nf.resize(S); r->ff.resize(S); r->act_off.resize(S); r->act_n.resize(S); r->cu.resize(S + 1);
  hipStream_t s = (hipStream_t)hip_stream;
  wf_config ecfg;
  int rc0 = wf_encoder_get_config(enc, &ecfg);
  if (rc0) return rc0;
  for (int k = 0; k < n_rounds; ++k) {
    const auto t0 = std::chrono::steady_clock::now();
    wf_round_record &rec = records[k];
    rec = wf_round_record{};
    int rc = wf_rounds_begin(r, &rec.start_us, r->nf.data(), r->ff.data());
    if (rc) return rc;
    int B = 0;
    for (int i = 0; i < S; ++i) {
      if (r->nf[i] < 1) continue;
      const int32_t n = pad_to_frames > 0 ? pad_to_frames : r->nf[i];
      // circular read: any window of up to `need` frames fits behind the wrapped offset
      r->act_off[B] = (int32_t)((int64_t)i * track_frames + (int64_t)r->ff[i] % (track_frames - need));
      r->act_n[B] = n;
      ++B;
    }
    if (B > 0) {
      rc = wf_encode_batch(enc, tracks_dev, mel_dtype, r->act_off.data(), r->act_n.data(), B, out_dev, out_dtype, out_capacity_tokens,
                           r->cu.data(), hip_stream);
      if (rc) { r->open = false; return rc; }
      hipError_t err = hipStreamSynchronize(s);
      if (err != hipSuccess) { r->open = false; return fail(WF_E_HIP, "round %d: %s", k, hipGetErrorString(err)); }
      rec.tokens = r->cu[B];
      for (int b = 0; b < B; ++b) rec.frames += r->act_n[b] + ecfg.hush_frames;
    }
    const auto t1 = std::chrono::steady_clock::now();
    rec.proc_us = std::max<int64_t>(1, std::chrono::duration_cast<std::chrono::microseconds>(t1 - t0).count());
    rec.n_active = B;
    rc = wf_rounds_end(r, rec.proc_us, &rec.end_us);
    if (rc) return rc;
  }
  return WF_OK;
}

}  // extern "C"
