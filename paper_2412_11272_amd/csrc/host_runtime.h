// Host-side helpers shared by the encoder, decoder and front-end runtimes: error text, device
// allocations owned by an object, weight upload, per-launch event profiling, the pinned staging ring
// for the small per-call index arrays, and the launch wrappers that attach flop/byte counts.
// Internal to the library; nothing here is part of the public ABI.
#pragma once
#include "../../include/wf_encoder.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <utility>
#include <vector>

#include "kernels.h"

namespace wf {
namespace host {

inline int fail(int code, const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  set_error(code, fmt, ap);
  va_end(ap);
  return code;
}

#define WF_HIP_TRY(expr)                                                                              \
  do {                                                                                                \
    hipError_t e_ = (expr);                                                                           \
    if (e_ != hipSuccess)                                                                             \
      return ::wf::host::fail(e_ == hipErrorOutOfMemory ? WF_E_OOM : WF_E_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

inline int64_t round_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }

// float -> bf16 bits, round to nearest even (NaN kept quiet).
inline uint16_t f32_to_bf16_rne(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

struct ProfRec { int cls; hipEvent_t t0, t1; double flops, bytes; };

// Deep enough that a caller enqueueing short calls back to back only ever blocks on a copy issued many
// calls ago (waking from such a wait costs more than several short calls take on the GPU).
constexpr int kStagingSlots = 32;

// What every runtime object owns on the device and the host.
struct DevCtx {
  int device = 0;
  bool bf16 = true;
  int es = 2;                           // bytes per activation/weight element
  std::vector<void *> allocs;           // every device allocation, for release()
  const char *const *class_names = nullptr;
  int n_classes = 0;
  // pinned staging ring for the small per-call index arrays
  int32_t *stage_host[kStagingSlots] = {};
  hipEvent_t stage_evt[kStagingSlots] = {};
  bool stage_used[kStagingSlots] = {};
  int stage_next = 0;
  // profiling
  bool profiling = false;
  std::vector<ProfRec> prof;
  std::vector<hipEvent_t> evt_pool;
};

inline int dev_alloc(DevCtx *e, void **p, size_t bytes) {
  *p = nullptr;
  if (bytes == 0) bytes = 256;
  hipError_t err = hipMalloc(p, bytes);
  if (err != hipSuccess) {
    (void)hipGetLastError();
    return fail(WF_E_OOM, "hipMalloc(%zu bytes): %s", bytes, hipGetErrorString(err));
  }
  e->allocs.push_back(*p);
  return WF_OK;
}

// Upload n floats as fp32.
inline int upload_f32(DevCtx *e, float **dst, const float *src, size_t n) {
  int rc = dev_alloc(e, (void **)dst, n * 4);
  if (rc) return rc;
  WF_HIP_TRY(hipMemcpy(*dst, src, n * 4, hipMemcpyHostToDevice));
  return WF_OK;
}

// Upload a host fp32 array in the object's weight dtype (bf16 RNE or fp32).
inline int upload_w(DevCtx *e, void **dst, const float *src, size_t n) {
  int rc = dev_alloc(e, dst, n * e->es);
  if (rc) return rc;
  if (e->bf16) {
    std::vector<uint16_t> tmp(n);
    for (size_t i = 0; i < n; ++i) tmp[i] = f32_to_bf16_rne(src[i]);
    WF_HIP_TRY(hipMemcpy(*dst, tmp.data(), n * 2, hipMemcpyHostToDevice));
  } else {
    WF_HIP_TRY(hipMemcpy(*dst, src, n * 4, hipMemcpyHostToDevice));
  }
  return WF_OK;
}
inline int upload_w(DevCtx *e, void **dst, const std::vector<float> &src) { return upload_w(e, dst, src.data(), src.size()); }

// Upload a weight matrix W [n_out, k] (k a multiple of 64) in panel layout [ceil(n_out/256)][k/64][256][64]
// (rows beyond n_out zero): every K step of a GEMM tile then reads one contiguous block.  bf16 objects only.
inline int upload_w_panels(DevCtx *e, void **dst, const float *src, int n_out, int k) {
  const int np = (n_out + 255) / 256, kc = k / 64;
  std::vector<uint16_t> tmp((size_t)np * kc * 16384, 0);
  for (int n = 0; n < n_out; ++n)
    for (int c = 0; c < kc; ++c) {
      uint16_t *d = tmp.data() + (((size_t)(n >> 8) * kc + c) << 14) + ((n & 255) << 6);
      const float *s = src + (size_t)n * k + c * 64;
      for (int j = 0; j < 64; ++j) d[j] = f32_to_bf16_rne(s[j]);
    }
  int rc = dev_alloc(e, dst, tmp.size() * 2);
  if (rc) return rc;
  WF_HIP_TRY(hipMemcpy(*dst, tmp.data(), tmp.size() * 2, hipMemcpyHostToDevice));
  return WF_OK;
}

inline int staging_create(DevCtx *e, size_t ints) {
  for (int i = 0; i < kStagingSlots; ++i) {
    WF_HIP_TRY(hipHostMalloc((void **)&e->stage_host[i], ints * 4, hipHostMallocDefault));
    WF_HIP_TRY(hipEventCreateWithFlags(&e->stage_evt[i], hipEventDisableTiming));
  }
  return WF_OK;
}

// Next staging slot, once its previous copy has left the buffer.
inline int staging_acquire(DevCtx *e, int *slot, int32_t **host) {
  *slot = e->stage_next;
  if (e->stage_used[*slot]) WF_HIP_TRY(hipEventSynchronize(e->stage_evt[*slot]));
  *host = e->stage_host[*slot];
  return WF_OK;
}

inline int staging_submit(DevCtx *e, int slot, void *dev, size_t bytes, hipStream_t s) {
  WF_HIP_TRY(hipMemcpyAsync(dev, e->stage_host[slot], bytes, hipMemcpyHostToDevice, s));
  WF_HIP_TRY(hipEventRecord(e->stage_evt[slot], s));
  e->stage_used[slot] = true;
  e->stage_next = (slot + 1) % kStagingSlots;
  return WF_OK;
}

inline void release(DevCtx *e) {
  (void)hipSetDevice(e->device);
  (void)hipDeviceSynchronize();
  for (auto &r : e->prof) { (void)hipEventDestroy(r.t0); (void)hipEventDestroy(r.t1); }
  for (auto ev : e->evt_pool) (void)hipEventDestroy(ev);
  for (int i = 0; i < kStagingSlots; ++i) {
    if (e->stage_host[i]) (void)hipHostFree(e->stage_host[i]);
    if (e->stage_evt[i]) (void)hipEventDestroy(e->stage_evt[i]);
  }
  for (void *p : e->allocs) (void)hipFree(p);
}

inline hipEvent_t get_event(DevCtx *e) {
  if (!e->evt_pool.empty()) {
    hipEvent_t ev = e->evt_pool.back();
    e->evt_pool.pop_back();
    return ev;
  }
  hipEvent_t ev = nullptr;
  if (hipEventCreate(&ev) != hipSuccess) return nullptr;
  return ev;
}

// Brackets one launch with events when profiling is on.
struct Scope {
  DevCtx *e;
  hipStream_t s;
  ProfRec rec{};
  bool on;
  Scope(DevCtx *ctx, hipStream_t st, int cls, double flops, double bytes) : e(ctx), s(st), on(ctx->profiling) {
    if (!on) return;
    rec.cls = cls; rec.flops = flops; rec.bytes = bytes;
    rec.t0 = get_event(e); rec.t1 = get_event(e);
    if (!rec.t0 || !rec.t1) { on = false; return; }
    (void)hipEventRecord(rec.t0, s);
  }
  ~Scope() {
    if (!on) return;
    (void)hipEventRecord(rec.t1, s);
    e->prof.push_back(rec);
  }
};

inline int collect_stats(DevCtx *e, wf_kernel_stat *stats, int32_t n_stats) {
  if (n_stats < e->n_classes) return fail(WF_E_INVALID_ARG, "n_stats = %d, need %d", n_stats, e->n_classes);
  for (int i = 0; i < e->n_classes; ++i) stats[i] = wf_kernel_stat{e->class_names[i], 0, 0.0, 0.0, 0.0};
  for (auto &r : e->prof) {
    WF_HIP_TRY(hipEventSynchronize(r.t1));
    float ms = 0.0f;
    WF_HIP_TRY(hipEventElapsedTime(&ms, r.t0, r.t1));
    wf_kernel_stat &st = stats[r.cls];
    st.launches += 1; st.total_ms += ms; st.flops += r.flops; st.bytes += r.bytes;
    e->evt_pool.push_back(r.t0);
    e->evt_pool.push_back(r.t1);
  }
  e->prof.clear();
  return WF_OK;
}

// a_rows x a_cols: the part of the activation operand the launch reads (once, algorithmically).
inline int run_gemm(DevCtx *e, hipStream_t s, int cls, const GemmArgs &a, AMode am, Epilogue ep, int k_real, int out_bytes,
                    double a_rows, double a_cols) {
  const double flops = 2.0 * a.M * a.N * k_real;
  double bytes = a_rows * a_cols * e->es + (double)a.N * k_real * e->es + (double)a.M * a.N * out_bytes;
  if (ep == EPI_BIAS_RESID) bytes += (double)a.M * a.N * 4;
  Scope sc(e, s, cls, flops, bytes);
  hipError_t err = e->bf16 ? launch_gemm_bf16(a, am, ep, s) : launch_gemm_f32(a, am, ep, s);
  if (err != hipSuccess) return fail(WF_E_HIP, "%s launch: %s", e->class_names[cls], hipGetErrorString(err));
  return WF_OK;
}

// Plain y = act(A W^T + b): A [M, K] (row stride lda), W [N, K], out [M, ldo].
inline int run_linear(DevCtx *e, hipStream_t s, int cls, const void *A, int lda, const void *W, const float *bias, void *out,
                      int ldo, int M, int N, int K, Epilogue ep) {
  GemmArgs a{};
  a.A = A; a.W = W; a.bias = bias; a.out = out;
  a.M = M; a.N = N; a.K = K; a.lda = lda; a.ldo = ldo;
  const int out_bytes = (ep == EPI_BIAS_RESID || ep == EPI_BIAS_F32) ? 4 : e->es;
  return run_gemm(e, s, cls, a, A_PLAIN, ep, K, out_bytes, M, K);
}

inline int run_ln(DevCtx *e, hipStream_t s, int cls, const float *x, const float *g, const float *b, void *out, int out_bf16,
                  int M, int d, float eps) {
  Scope sc(e, s, cls, 0.0, (double)M * d * (4 + (out_bf16 ? 2 : 4)));
  hipError_t err = launch_layernorm(x, g, b, out, out_bf16, M, d, eps, s);
  if (err != hipSuccess) return fail(WF_E_HIP, "%s launch: %s", e->class_names[cls], hipGetErrorString(err));
  return WF_OK;
}

// Attention work list: one item per (stream, block of q_tile queries), longest streams first so the
// expensive items are scheduled before the cheap ones fill in.  cost[i] orders the streams (NULL: the
// query count).
inline int build_work(const int32_t *cu_q, int B, int q_tile, int32_t *work, const int64_t *cost = nullptr, int stream_base = 0) {
  std::vector<std::pair<int64_t, int>> order(B);
  for (int i = 0; i < B; ++i) order[i] = {cost ? cost[i] : (int64_t)(cu_q[i + 1] - cu_q[i]), i};
  std::stable_sort(order.begin(), order.end(),
                   [](const std::pair<int64_t, int> &a, const std::pair<int64_t, int> &b) { return a.first > b.first; });
  int n = 0, rank = 0;
  for (const auto &o : order) {
    const int Lq = cu_q[o.second + 1] - cu_q[o.second];
    for (int q0 = 0; q0 < Lq; q0 += q_tile) {
      work[2 * n] = o.second + stream_base;     // cu_q points at the first of the B streams; ids stay absolute
      work[2 * n + 1] = q0 | ((rank & 7) << 20); // the stream's rank mod 8 rides along (head -> XCD rotation)
      ++n;
    }
    ++rank;
  }
  return n;
}

// Same work list as build_work (streams by descending query count, ties in input order) without touching the
// heap: `keys` is caller-provided room for B entries.  Each key packs (count, B - 1 - index), so sorting the keys
// in descending order is the stable descending sort by count.
inline int build_work_noalloc(const int32_t *cu_q, int B, int q_tile, int32_t *work, int64_t *keys) {
  for (int i = 0; i < B; ++i) keys[i] = ((int64_t)(cu_q[i + 1] - cu_q[i]) << 32) | (uint32_t)(B - 1 - i);
  std::sort(keys, keys + B, [](int64_t a, int64_t b) { return a > b; });   // introsort: in place
  int n = 0;
  for (int rank = 0; rank < B; ++rank) {
    const int i = B - 1 - (int)(keys[rank] & 0xffffffff);
    const int Lq = cu_q[i + 1] - cu_q[i];
    for (int q0 = 0; q0 < Lq; q0 += q_tile) {
      work[2 * n] = i;
      work[2 * n + 1] = q0 | ((rank & 7) << 20);
      ++n;
    }
  }
  return n;
}

}  // namespace host
}  // namespace wf
