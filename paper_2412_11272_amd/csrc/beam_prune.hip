// Beam pruning (paper Section "Beam pruning"): the reference-based beam-size state machine.  Host integer
// logic only; the rules are stated with the declarations in include/wf_encoder.h.
#include "host_runtime.h"

#include <new>
#include <unordered_map>

using namespace wf::host;

namespace {
enum Event : int32_t { EV_SKIPPED = 0, EV_ALIGNED, EV_MATCHED, EV_FB_ALIGN, EV_FB_MISMATCH, EV_FB_END, EV_FULL };
}

struct wf_beam_pruner {
  int32_t full = 1, beam = 1, special_from = 0;
  std::vector<int32_t> ref;
  std::unordered_map<int32_t, int32_t> first_pos;   // token -> index of its first occurrence in ref
  std::vector<int32_t> punct;                       // sorted
  int64_t idx = -1;                                 // reference index; -1 until aligned
  bool fallen = false;
  bool filter_reference = true;                     // false: the reference list is matched as handed over

  void set_reference(const int32_t *t, int32_t n) {
    ref.clear();
    for (int32_t i = 0; i < n; ++i)
      if (!filter_reference || !exempt(t[i])) ref.push_back(t[i]);   // filtering: timestamps and punctuation take no part
    first_pos.clear();
    first_pos.reserve(ref.size() * 2 + 1);
    for (size_t i = 0; i < ref.size(); ++i) first_pos.emplace(ref[i], (int32_t)i);   // emplace keeps the first
    beam = 1;
    idx = -1;
    fallen = false;
  }
  bool exempt(int32_t tok) const { return tok >= special_from || std::binary_search(punct.begin(), punct.end(), tok); }
  int32_t fall(int32_t ev) {
    fallen = true;
    beam = full;
    return ev;
  }
  int32_t step(int32_t tok) {
    if (fallen) return EV_FULL;
    if (exempt(tok)) return EV_SKIPPED;
    if (idx < 0) {
      auto it = first_pos.find(tok);
      if (it == first_pos.end()) return fall(EV_FB_ALIGN);
      idx = (int64_t)it->second + 1;
      return EV_ALIGNED;
    }
    if (idx >= (int64_t)ref.size()) return fall(EV_FB_END);
    if (ref[(size_t)idx] == tok) {
      ++idx;
      return EV_MATCHED;
    }
    return fall(EV_FB_MISMATCH);
  }
};

extern "C" {

int wf_beam_pruner_create(int32_t beam_size, const int32_t *ref_tokens, int32_t n_ref, int32_t special_from,
                          const int32_t *punct_ids, int32_t n_punct, int32_t filter_reference, wf_beam_pruner **out) {
  if (!out) return fail(WF_E_INVALID_ARG, "out is NULL");
  *out = nullptr;
  if (beam_size < 1) return fail(WF_E_INVALID_ARG, "beam_size = %d, need >= 1", beam_size);
  if (n_ref < 0 || (n_ref > 0 && !ref_tokens)) return fail(WF_E_INVALID_ARG, "n_ref = %d with ref_tokens %s", n_ref, ref_tokens ? "set" : "NULL");
  if (n_punct < 0 || (n_punct > 0 && !punct_ids)) return fail(WF_E_INVALID_ARG, "n_punct = %d with punct_ids %s", n_punct, punct_ids ? "set" : "NULL");
  wf_beam_pruner *p = new (std::nothrow) wf_beam_pruner();
  if (!p) return fail(WF_E_OOM, "host allocation failed");
  p->full = beam_size;
  p->special_from = special_from;
  p->filter_reference = filter_reference != 0;
  p->punct.assign(punct_ids, punct_ids + n_punct);
  std::sort(p->punct.begin(), p->punct.end());
  p->set_reference(ref_tokens, n_ref);
  *out = p;
  return WF_OK;
}

void wf_beam_pruner_destroy(wf_beam_pruner *p) { delete p; }

int wf_beam_pruner_reset(wf_beam_pruner *p, const int32_t *ref_tokens, int32_t n_ref) {
  if (!p) return fail(WF_E_INVALID_ARG, "pruner is NULL");
  if (n_ref < 0 || (n_ref > 0 && !ref_tokens)) return fail(WF_E_INVALID_ARG, "n_ref = %d with ref_tokens %s", n_ref, ref_tokens ? "set" : "NULL");
  p->set_reference(ref_tokens, n_ref);
  return WF_OK;
}

int wf_beam_pruner_step(wf_beam_pruner *p, int32_t best_token, int32_t *event, int32_t *next_beam) {
  if (!p) return fail(WF_E_INVALID_ARG, "pruner is NULL");
  const int32_t ev = p->step(best_token);
  if (event) *event = ev;
  if (next_beam) *next_beam = p->beam;
  return WF_OK;
}

int wf_beam_prune_session(wf_beam_pruner *p, const int32_t *best_tokens, int32_t n, int32_t *beam_for_step, int32_t *events) {
  if (!p) return fail(WF_E_INVALID_ARG, "pruner is NULL");
  if (n < 0 || (n > 0 && !best_tokens)) return fail(WF_E_INVALID_ARG, "n = %d with best_tokens %s", n, best_tokens ? "set" : "NULL");
  for (int32_t t = 0; t < n; ++t) {
    if (beam_for_step) beam_for_step[t] = p->beam;
    const int32_t ev = p->step(best_tokens[t]);
    if (events) events[t] = ev;
  }
  return WF_OK;
}

}  // extern "C"
