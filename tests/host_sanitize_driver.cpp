// Command interpreter over the host-only entry points of the C ABI (include/wf_encoder.h), meant to be built
// with AddressSanitizer + UndefinedBehaviorSanitizer on the host side and linked statically against the library's
// objects.  tests/test_host_sanitized.py writes commands to stdin (the scenarios of the other host tests), reads
// the results from stdout and compares them with the oracles; any sanitizer report makes the run fail.
// No GPU call is made: only planning, validation, round bookkeeping and the beam-pruning state machine.
//
//   cfgcheck <11 config fields>                                   -> rc
//   plan <11 config fields> B n_frames[B]                         -> rc total_frames total_tokens cu[B+1]
//   beam beam special_from filter np punct[np] nr ref[nr] nt tok[nt]
//                                                                 -> "S" beams[nt] events[nt] (whole session)
//                                                                    "T" beams[nt] events[nt] (one step at a time)
//   rounds S step trim keep max starts[S] n procs[n]              -> per round: s e n[S] f[S]; then the statistics
//   invalid                                                       -> rc of every entry point called with bad arguments
#include <cinttypes>
#include <cstdio>
#include <cstdlib>
#include <iostream>
#include <sstream>
#include <string>
#include <vector>

#include "../include/wf_encoder.h"

namespace {

bool read_cfg(std::istringstream &in, wf_config &c) {
  return static_cast<bool>(in >> c.n_mels >> c.d_model >> c.n_layers >> c.n_heads >> c.d_mlp >> c.hush_frames >> c.max_streams >>
                           c.max_total_frames >> c.max_frames_per_stream >> c.precision >> c.ln_eps);
}

template <typename T>
std::vector<T> read_vec(std::istringstream &in) {
  long n = 0;
  in >> n;
  std::vector<T> v((size_t)(n < 0 ? 0 : n));
  for (auto &x : v) {
    long long t;
    in >> t;
    x = (T)t;
  }
  return v;
}

template <typename T>
void print_vec(const std::vector<T> &v) {
  for (auto x : v) printf(" %lld", (long long)x);
}

}  // namespace

int main() {
  std::string line;
  while (std::getline(std::cin, line)) {
    std::istringstream in(line);
    std::string cmd;
    if (!(in >> cmd)) continue;
    if (cmd == "cfgcheck") {
      wf_config c{};
      if (!read_cfg(in, c)) return 2;
      printf("%d\n", wf_config_check(&c));
    } else if (cmd == "plan") {
      wf_config c{};
      if (!read_cfg(in, c)) return 2;
      std::vector<int32_t> nf = read_vec<int32_t>(in);
      std::vector<int32_t> cu(nf.size() + 1, -1);
      int64_t tf = -1, tt = -1;
      const int rc = wf_plan_batch(&c, nf.data(), (int32_t)nf.size(), cu.data(), &tf, &tt);
      printf("%d %" PRId64 " %" PRId64, rc, tf, tt);
      if (rc == WF_OK) print_vec(cu);
      printf("\n");
    } else if (cmd == "beam") {
      int beam, special_from, filter;
      in >> beam >> special_from >> filter;
      std::vector<int32_t> punct = read_vec<int32_t>(in), ref = read_vec<int32_t>(in), tok = read_vec<int32_t>(in);
      wf_beam_pruner *p = nullptr;
      int rc = wf_beam_pruner_create(beam, ref.empty() ? nullptr : ref.data(), (int32_t)ref.size(), special_from,
                                     punct.empty() ? nullptr : punct.data(), (int32_t)punct.size(), filter, &p);
      if (rc != WF_OK) {
        printf("E %d\n", rc);
        continue;
      }
      std::vector<int32_t> beams(tok.size()), events(tok.size());
      rc = wf_beam_prune_session(p, tok.empty() ? nullptr : tok.data(), (int32_t)tok.size(), beams.data(), events.data());
      printf("S %d", rc);
      print_vec(beams);
      print_vec(events);
      printf("\n");
      rc = wf_beam_pruner_reset(p, ref.empty() ? nullptr : ref.data(), (int32_t)ref.size());
      int32_t run_with = 1;
      for (size_t t = 0; t < tok.size(); ++t) {
        beams[t] = run_with;
        int32_t ev = -1;
        rc |= wf_beam_pruner_step(p, tok[t], &ev, &run_with);
        events[t] = ev;
      }
      printf("T %d", rc);
      print_vec(beams);
      print_vec(events);
      printf("\n");
      wf_beam_pruner_destroy(p);
    } else if (cmd == "rounds") {
      wf_rounds_config c{};
      long long step;
      in >> c.n_streams >> step >> c.trim_frames >> c.keep_frames >> c.max_frames;
      c.step_us = step;
      std::vector<int64_t> starts((size_t)(c.n_streams > 0 ? c.n_streams : 0));
      for (auto &s : starts) {
        long long t;
        in >> t;
        s = t;
      }
      std::vector<int64_t> procs = read_vec<int64_t>(in);
      wf_rounds *r = nullptr;
      int rc = wf_rounds_create(&c, starts.data(), &r);
      if (rc != WF_OK) {
        printf("E %d\n", rc);
        continue;
      }
      std::vector<int32_t> n(starts.size()), f(starts.size());
      for (int64_t proc : procs) {
        int64_t s = -1, e = -1;
        rc = wf_rounds_begin(r, &s, n.data(), f.data());
        rc |= wf_rounds_end(r, proc, &e);
        printf("R %d %" PRId64 " %" PRId64, rc, s, e);
        print_vec(n);
        print_vec(f);
        printf("\n");
      }
      wf_rounds_stats st{};
      rc = wf_rounds_get_stats(r, &st);
      printf("Q %d %" PRId64 " %" PRId64 " %" PRId64 " %" PRId64 " %.17g %.17g\n", rc, (int64_t)st.rounds, (int64_t)st.frames_total,
             (int64_t)st.max_proc_us, (int64_t)st.last_round_end_us, st.mean_proc_us, st.mean_latency_us);
      wf_rounds_destroy(r);
    } else if (cmd == "invalid") {
      // every entry point that can refuse its arguments before touching a GPU
      wf_encoder *enc = nullptr;
      wf_config c{};
      int32_t one = 1;
      int64_t i64 = 0;
      printf("%d", wf_encoder_create(nullptr, nullptr, &enc));
      printf(" %d", wf_encoder_create(&c, nullptr, nullptr));
      printf(" %d", wf_encode_batch(nullptr, nullptr, 0, nullptr, nullptr, 1, nullptr, 0, 0, nullptr, nullptr));
      printf(" %d", wf_plan_batch(nullptr, &one, 1, nullptr, nullptr, nullptr));
      printf(" %d", wf_encoder_set_lanes(nullptr, 1));
      printf(" %d", wf_encoder_get_lanes(nullptr));
      printf(" %d", wf_encoder_set_graphs(nullptr, 1));
      printf(" %d", wf_encoder_graph_stats(nullptr, &i64, &i64, &i64));
      printf(" %d", wf_encoder_set_profiling(nullptr, 1));
      printf(" %d", wf_op_linear(0, nullptr, nullptr, nullptr, nullptr, 1, 128, 64, 0, nullptr));
      printf(" %d", wf_op_layernorm(nullptr, nullptr, nullptr, nullptr, 0, 1, 128, 1e-5f, nullptr));
      printf(" %d", wf_op_ln_linear(nullptr, nullptr, nullptr, 1e-5f, nullptr, nullptr, nullptr, 1, 128, 64, 0, nullptr));
      printf(" %d", wf_gemm_tile_map(256, 256, 256, 256, nullptr, 0));
      printf(" %d", wf_gemm_tile_choice(256, 256, nullptr, nullptr));
      printf(" %d", wf_gelu_host(nullptr, nullptr, 3));
      printf(" %d", wf_op_attention(0, nullptr, nullptr, nullptr, 1, 1, nullptr));
      printf(" %d", wf_op_attention_noalloc(0, nullptr, nullptr, nullptr, 1, 1, nullptr));
      printf(" %d", wf_rounds_create(nullptr, nullptr, nullptr));
      printf(" %d", wf_rounds_begin(nullptr, nullptr, nullptr, nullptr));
      printf(" %d", wf_rounds_end(nullptr, 0, nullptr));
      printf(" %d", wf_beam_pruner_create(0, nullptr, 0, 0, nullptr, 0, 1, nullptr));
      printf(" %d", wf_beam_pruner_step(nullptr, 0, nullptr, nullptr));
      printf(" %d", wf_beam_prune_session(nullptr, nullptr, 0, nullptr, nullptr));
      wf_encoder_destroy(nullptr);
      wf_rounds_destroy(nullptr);
      wf_beam_pruner_destroy(nullptr);
      printf(" | %s\n", wf_last_error()[0] ? "text" : "empty");
    } else {
      fprintf(stderr, "unknown command: %s\n", cmd.c_str());
      return 2;
    }
    fflush(stdout);
  }
  return 0;
}
