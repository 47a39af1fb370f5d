// Log-mel front end with the hush word appended at the raw-audio level (declared in
// include/wf_encoder.h, which also states the definition).  fp32 throughout: the spectrogram spans
// eight decades.
//
//   frame_map_kernel   packed frame index -> (stream, frame inside the stream); resets the per-stream maxima
//   stft_mel_kernel    per workgroup 32 consecutive packed frames: the windowed, reflect-padded frames of
//                      x (+) h are gathered into LDS; the 400-point DFT is a dense contraction against
//                      cos / -sin tables, run on the fp32 matrix cores (v_mfma_f32_32x32x2_f32): each of
//                      7 waves owns 32 frequency bins and keeps a cosine and a sine accumulator whose
//                      registers line up, so the power is a per-register a*a + b*b; the power tile goes
//                      back to LDS, every thread then does a few mel filters (triangles are narrow: only
//                      the bins under a filter are visited) and writes log10(max(., 1e-10)); the
//                      per-stream maximum is an integer atomicMax on an order-preserving key (first in
//                      LDS per frame, then one global atomic per stream and workgroup), hence
//                      independent of arrival order
//   normalize_kernel   clamp to (stream max - 8), (v + 4) / 4, convert, store packed
#include "../../include/wf_encoder.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "device_utils.h"
#include "kernels.h"

namespace {

constexpr int kHop = 160, kNfft = 400, kBins = 201, kBinsPad = 224, kFramesPerBlock = 32;
constexpr int kRowStride = kNfft + 1;          // LDS row stride of the frame tile (odd: conflict-free column reads)
constexpr double kPi = 3.14159265358979323846;

int ffail(int code, const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  const int rc = wf::set_error(code, fmt, ap);
  va_end(ap);
  return rc;
}

#define FE_HIP_TRY(expr)                                                                       \
  do {                                                                                         \
    hipError_t e_ = (expr);                                                                    \
    if (e_ != hipSuccess) return ffail(e_ == hipErrorOutOfMemory ? WF_E_OOM : WF_E_HIP,        \
                                       "%s: %s", #expr, hipGetErrorString(e_));                \
  } while (0)

struct FeArgs {
  const float *audio;          // caller's samples
  const float *hush;           // [H]
  const float *window;         // [400]
  const float *basis_c;        // [400][224]  cos(2 pi f n / 400), zero for f >= 201
  const float *basis_s;        // [400][224]  -sin(2 pi f n / 400)
  const float *fbank;          // [n_mels][224]
  const int32_t *fb_lo, *fb_hi;// [n_mels] first / one-past-last bin under each filter
  const int64_t *sample_offset;// [B]
  const int32_t *n_samples;    // [B]
  const int32_t *cu_frames;    // [B+1]
  int32_t *frame_stream;       // [F]
  int32_t *frame_t;            // [F]
  float *V;                    // [F][n_mels]  log10 mel before the clamp
  int32_t *smax;               // [B] order-preserving integer key of the stream maximum
  void *out;                   // [F][n_mels]
  int32_t B, F, H, n_mels, out_bf16;
};

__device__ __forceinline__ int32_t float_key(float v) {   // monotone float -> int
  const int32_t b = __float_as_int(v);
  return b >= 0 ? b : b ^ 0x7fffffff;
}
__device__ __forceinline__ float key_float(int32_t k) { return __int_as_float(k >= 0 ? k : k ^ 0x7fffffff); }

__global__ void __launch_bounds__(256) frame_map_kernel(FeArgs p) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r < p.B) p.smax[r] = float_key(-INFINITY);
  if (r >= p.F) return;
  const int i = wf::find_stream(p.cu_frames, p.B, r);
  p.frame_stream[r] = i;
  p.frame_t[r] = r - p.cu_frames[i];
}

typedef float f32x16 __attribute__((ext_vector_type(16)));

__global__ void __launch_bounds__(448) stft_mel_kernel(FeArgs p) {
  extern __shared__ __attribute__((aligned(16))) float lds[];
  float *sFrames = lds;                                   // [32][401] windowed frames; later reused as sPower [32][224]
  __shared__ int sStream[kFramesPerBlock], sT[kFramesPerBlock], sN[kFramesPerBlock], sRowMax[kFramesPerBlock];
  __shared__ long sOff[kFramesPerBlock];
  const int f0 = blockIdx.x * kFramesPerBlock;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, lg = lane >> 5;

  if (tid < kFramesPerBlock) {                             // per-frame metadata, once
    int row = f0 + tid;
    row = row < p.F ? row : p.F - 1;                       // rows past the end are computed but never stored
    const int i = p.frame_stream[row];
    sStream[tid] = i;
    sT[tid] = p.frame_t[row];
    sN[tid] = p.n_samples[i];
    sOff[tid] = p.sample_offset[i];
    sRowMax[tid] = float_key(-INFINITY);
  }
  __syncthreads();

  // ---- gather: sample n of frame (stream i, t) is xp[160 t + n] with xp = reflect-padded x (+) h
  for (int e = tid; e < kFramesPerBlock * kNfft; e += 448) {
    const int fr = e / kNfft, n = e - fr * kNfft;
    const int N = sN[fr], Np = N + p.H;
    int s = kHop * sT[fr] + n - kNfft / 2;
    s = s < 0 ? -s : s;
    s = s >= Np ? 2 * (Np - 1) - s : s;
    const float x = s < N ? p.audio[sOff[fr] + s] : p.hush[s - N];
    sFrames[fr * kRowStride + n] = x * p.window[n];
  }
  __syncthreads();

  // ---- DFT on the fp32 matrix cores: D[frame][bin] += A[frame][k] B[k][bin], two k per instruction.
  // First operand: lane (frame l32, k = lg); second operand: lane (bin l32, k = lg).
  f32x16 acc_c, acc_s;
#pragma unroll
  for (int r = 0; r < 16; ++r) { acc_c[r] = 0.0f; acc_s[r] = 0.0f; }
  const int bin = wave * 32 + l32;
  const float *fa = sFrames + l32 * kRowStride + lg;
  const float *bc = p.basis_c + lg * kBinsPad + bin;
  const float *bs = p.basis_s + lg * kBinsPad + bin;
#pragma unroll 8
  for (int k = 0; k < kNfft; k += 2) {
    const float a = fa[k];
    const float c = bc[k * kBinsPad];
    const float s = bs[k * kBinsPad];
    acc_c = __builtin_amdgcn_mfma_f32_32x32x2f32(a, c, acc_c, 0, 0, 0);
    acc_s = __builtin_amdgcn_mfma_f32_32x32x2f32(a, s, acc_s, 0, 0, 0);
  }
  __syncthreads();                                          // all waves are done reading the frames
  // accumulator register r of lane (l32, lg) is frame 8*(r/4) + 4*lg + r%4, bin (wave*32 + l32)
  float *sPower = lds;                                      // [32][224]
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int fr = 8 * (r >> 2) + 4 * lg + (r & 3);
    sPower[fr * kBinsPad + bin] = acc_c[r] * acc_c[r] + acc_s[r] * acc_s[r];
  }
  __syncthreads();

  // ---- mel filters + log10, one (frame, filter) pair per thread and step; row maxima in LDS
  for (int e = tid; e < kFramesPerBlock * p.n_mels; e += 448) {
    const int fr = e / p.n_mels, j = e - fr * p.n_mels;
    const int row = f0 + fr;
    if (row >= p.F) break;
    float m = 0.0f;
    const float *w = p.fbank + j * kBinsPad;
    for (int f = p.fb_lo[j]; f < p.fb_hi[j]; ++f) m = fmaf(w[f], sPower[fr * kBinsPad + f], m);
    const float v = log10f(fmaxf(m, 1e-10f));
    p.V[(size_t)row * p.n_mels + j] = v;
    atomicMax(&sRowMax[fr], float_key(v));
  }
  __syncthreads();
  // one global atomic per stream present in the block (its frames are consecutive)
  if (tid == 0) {
    const int nrows = min(kFramesPerBlock, p.F - f0);
    int cur = sStream[0], key = sRowMax[0];
    for (int fr = 1; fr < nrows; ++fr) {
      if (sStream[fr] != cur) {
        atomicMax(p.smax + cur, key);
        cur = sStream[fr];
        key = sRowMax[fr];
      } else {
        key = max(key, sRowMax[fr]);
      }
    }
    atomicMax(p.smax + cur, key);
  }
}

template <typename TOUT>
__global__ void __launch_bounds__(256) normalize_kernel(FeArgs p) {
  const long e = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= (long)p.F * p.n_mels) return;
  const int row = (int)(e / p.n_mels);
  const float top = key_float(p.smax[p.frame_stream[row]]);
  const float v = fmaxf(p.V[e], top - 8.0f);
  ((TOUT *)p.out)[e] = (TOUT)((v + 4.0f) * 0.25f);
}

}  // namespace

// Pinned staging slots for the per-call index arrays.  A slot is reused only after its copy has left it; the
// ring is deep enough that a caller who enqueues short calls back to back blocks on work issued many calls
// ago (waking from such a wait costs more than several of these calls take on the GPU).
constexpr int kIdxSlots = 32;

struct wf_frontend {
  wf_frontend_config cfg{};
  int64_t max_frames = 0;
  std::vector<void *> allocs;
  float *hush = nullptr, *window = nullptr, *basis_c = nullptr, *basis_s = nullptr, *fbank = nullptr, *V = nullptr;
  int32_t *fb_lo = nullptr, *fb_hi = nullptr, *frame_stream = nullptr, *frame_t = nullptr, *smax = nullptr;
  unsigned char *idx_dev = nullptr;      // [B] int64 offsets | [B] int32 n_samples | [B+1] int32 cu_frames
  unsigned char *idx_host[kIdxSlots] = {};
  hipEvent_t idx_evt[kIdxSlots] = {};
  bool idx_used[kIdxSlots] = {};
  int idx_next = 0;
  size_t idx_bytes = 0;
};

namespace {

int fe_alloc(wf_frontend *fe, void **p, size_t bytes) {
  *p = nullptr;
  hipError_t err = hipMalloc(p, bytes ? bytes : 256);
  if (err != hipSuccess) {
    (void)hipGetLastError();
    return ffail(WF_E_OOM, "hipMalloc(%zu bytes): %s", bytes, hipGetErrorString(err));
  }
  fe->allocs.push_back(*p);
  return WF_OK;
}

template <typename T>
int fe_upload(wf_frontend *fe, T **dst, const std::vector<T> &src) {
  int rc = fe_alloc(fe, (void **)dst, src.size() * sizeof(T));
  if (rc) return rc;
  FE_HIP_TRY(hipMemcpy(*dst, src.data(), src.size() * sizeof(T), hipMemcpyHostToDevice));
  return WF_OK;
}

double hz_to_mel(double f) { return 2595.0 * std::log10(1.0 + f / 700.0); }
double mel_to_hz(double m) { return 700.0 * (std::pow(10.0, m / 2595.0) - 1.0); }

int fe_create(wf_frontend *fe, const wf_frontend_config *cfg, const float *hush_audio) {
  fe->cfg = *cfg;
  const int n_mels = cfg->n_mels, H = cfg->hush_samples;
  fe->max_frames = cfg->max_total_samples / kHop + cfg->max_streams;
  int rc;
  std::vector<float> hush((size_t)(H > 0 ? H : 1), 0.0f);
  if (H > 0) memcpy(hush.data(), hush_audio, (size_t)H * 4);
  if ((rc = fe_upload(fe, &fe->hush, hush))) return rc;
  std::vector<float> win(kNfft), bc((size_t)kNfft * kBinsPad, 0.0f), bs((size_t)kNfft * kBinsPad, 0.0f);
  for (int n = 0; n < kNfft; ++n) {
    win[n] = (float)(0.5 - 0.5 * std::cos(2.0 * kPi * n / kNfft));
    for (int f = 0; f < kBins; ++f) {
      const int ph = (int)(((long)f * n) % kNfft);            // exact phase reduction before cos/sin
      bc[(size_t)n * kBinsPad + f] = (float)std::cos(2.0 * kPi * ph / kNfft);
      bs[(size_t)n * kBinsPad + f] = (float)(-std::sin(2.0 * kPi * ph / kNfft));
    }
  }
  if ((rc = fe_upload(fe, &fe->window, win))) return rc;
  if ((rc = fe_upload(fe, &fe->basis_c, bc))) return rc;
  if ((rc = fe_upload(fe, &fe->basis_s, bs))) return rc;
  // triangular filters, unit peak, equally spaced on the mel scale over [0, 8000] Hz
  std::vector<double> edges(n_mels + 2);
  const double m_hi = hz_to_mel(8000.0);
  for (int k = 0; k < n_mels + 2; ++k) edges[k] = mel_to_hz(m_hi * k / (n_mels + 1));
  std::vector<float> fb((size_t)n_mels * kBinsPad, 0.0f);
  std::vector<int32_t> lo(n_mels), hi(n_mels);
  for (int k = 0; k < n_mels; ++k) {
    int first = kBins, last = 0;
    for (int f = 0; f < kBins; ++f) {
      const double hz = f * 40.0;
      const double up = (hz - edges[k]) / (edges[k + 1] - edges[k]);
      const double down = (edges[k + 2] - hz) / (edges[k + 2] - edges[k + 1]);
      const double w = std::fmax(0.0, std::fmin(up, down));
      fb[(size_t)k * kBinsPad + f] = (float)w;
      if (w > 0.0) { first = f < first ? f : first; last = f + 1 > last ? f + 1 : last; }
    }
    lo[k] = first < last ? first : 0;
    hi[k] = first < last ? last : 0;
  }
  if ((rc = fe_upload(fe, &fe->fbank, fb))) return rc;
  if ((rc = fe_upload(fe, &fe->fb_lo, lo))) return rc;
  if ((rc = fe_upload(fe, &fe->fb_hi, hi))) return rc;
  if ((rc = fe_alloc(fe, (void **)&fe->V, (size_t)fe->max_frames * n_mels * 4))) return rc;
  if ((rc = fe_alloc(fe, (void **)&fe->frame_stream, (size_t)fe->max_frames * 4))) return rc;
  if ((rc = fe_alloc(fe, (void **)&fe->frame_t, (size_t)fe->max_frames * 4))) return rc;
  if ((rc = fe_alloc(fe, (void **)&fe->smax, (size_t)cfg->max_streams * 4))) return rc;
  fe->idx_bytes = (size_t)cfg->max_streams * 8 + (size_t)cfg->max_streams * 4 + (size_t)(cfg->max_streams + 1) * 4;
  fe->idx_bytes = (fe->idx_bytes + 15) / 16 * 16;
  if ((rc = fe_alloc(fe, (void **)&fe->idx_dev, fe->idx_bytes))) return rc;
  for (int i = 0; i < kIdxSlots; ++i) {
    FE_HIP_TRY(hipHostMalloc((void **)&fe->idx_host[i], fe->idx_bytes, hipHostMallocDefault));
    FE_HIP_TRY(hipEventCreateWithFlags(&fe->idx_evt[i], hipEventDisableTiming));
  }
  FE_HIP_TRY(hipFuncSetAttribute((const void *)stft_mel_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                 kFramesPerBlock * kRowStride * 4));
  FE_HIP_TRY(hipDeviceSynchronize());
  return WF_OK;
}

}  // namespace

extern "C" {

void wf_frontend_destroy(wf_frontend *fe) {
  if (!fe) return;
  (void)hipDeviceSynchronize();
  for (int i = 0; i < kIdxSlots; ++i) {
    if (fe->idx_host[i]) (void)hipHostFree(fe->idx_host[i]);
    if (fe->idx_evt[i]) (void)hipEventDestroy(fe->idx_evt[i]);
  }
  for (void *p : fe->allocs) (void)hipFree(p);
  delete fe;
}

int wf_frontend_create(const wf_frontend_config *cfg, const float *hush_audio, wf_frontend **out) {
  if (!out) return ffail(WF_E_INVALID_ARG, "out is NULL");
  *out = nullptr;
  if (!cfg) return ffail(WF_E_INVALID_ARG, "cfg is NULL");
  if (cfg->n_mels < 1 || cfg->n_mels > 256) return ffail(WF_E_INVALID_ARG, "n_mels = %d, need 1..256", cfg->n_mels);
  if (cfg->hush_samples < 0) return ffail(WF_E_INVALID_ARG, "hush_samples = %d", cfg->hush_samples);
  if (cfg->hush_samples > 0 && !hush_audio) return ffail(WF_E_INVALID_ARG, "hush_audio is NULL but hush_samples = %d", cfg->hush_samples);
  if (cfg->max_streams < 1) return ffail(WF_E_INVALID_ARG, "max_streams = %d", cfg->max_streams);
  if (cfg->max_total_samples < kBins || cfg->max_total_samples > 2000000000LL)
    return ffail(WF_E_INVALID_ARG, "max_total_samples = %lld out of range", (long long)cfg->max_total_samples);
  wf_frontend *fe = new (std::nothrow) wf_frontend();
  if (!fe) return ffail(WF_E_OOM, "host allocation failed");
  int rc = fe_create(fe, cfg, hush_audio);
  if (rc) {
    char keep[512];
    memcpy(keep, wf::error_buffer(), sizeof(keep));
    wf_frontend_destroy(fe);
    memcpy(wf::error_buffer(), keep, sizeof(keep));
    return rc;
  }
  *out = fe;
  return WF_OK;
}

int wf_logmel_batch(wf_frontend *fe, const float *audio_dev, const int64_t *sample_offset, const int32_t *n_samples, int32_t B,
                    void *mel_out_dev, int32_t mel_dtype, int64_t mel_capacity_frames, int32_t *cu_frames_host, void *hip_stream) {
  if (!fe) return ffail(WF_E_INVALID_ARG, "frontend is NULL");
  if (!audio_dev || !sample_offset || !n_samples || !mel_out_dev) return ffail(WF_E_INVALID_ARG, "NULL pointer");
  if (mel_dtype != WF_DTYPE_F32 && mel_dtype != WF_DTYPE_BF16) return ffail(WF_E_INVALID_ARG, "mel_dtype = %d", mel_dtype);
  if (B < 1) return ffail(WF_E_INVALID_ARG, "B = %d, need B >= 1", B);
  if (B > fe->cfg.max_streams) return ffail(WF_E_CAPACITY, "B = %d exceeds max_streams = %d", B, fe->cfg.max_streams);
  const int H = fe->cfg.hush_samples;
  const int slot = fe->idx_next;
  if (fe->idx_used[slot]) FE_HIP_TRY(hipEventSynchronize(fe->idx_evt[slot]));
  unsigned char *hs = fe->idx_host[slot];
  const int S = fe->cfg.max_streams;
  int64_t *h_off = (int64_t *)hs;
  int32_t *h_n = (int32_t *)(hs + (size_t)S * 8);
  int32_t *h_cu = h_n + S;
  int64_t total = 0, frames = 0;
  h_cu[0] = 0;
  for (int i = 0; i < B; ++i) {
    if (n_samples[i] < 0 || sample_offset[i] < 0) return ffail(WF_E_INVALID_ARG, "stream %d: negative length or offset", i);
    const int64_t Np = (int64_t)n_samples[i] + H;
    if (Np < kBins) return ffail(WF_E_INVALID_ARG, "stream %d: %lld samples incl. hush, need >= %d (reflect padding)", i, (long long)Np, kBins);
    total += Np;
    if (total > fe->cfg.max_total_samples)
      return ffail(WF_E_CAPACITY, "total samples incl. hush exceed max_total_samples = %lld (at stream %d)", (long long)fe->cfg.max_total_samples, i);
    frames += Np / kHop;
    h_off[i] = sample_offset[i];
    h_n[i] = n_samples[i];
    h_cu[i + 1] = (int32_t)frames;
  }
  if (frames > mel_capacity_frames)
    return ffail(WF_E_CAPACITY, "batch produces %lld frames but mel_capacity_frames = %lld", (long long)frames, (long long)mel_capacity_frames);
  if (cu_frames_host) memcpy(cu_frames_host, h_cu, (size_t)(B + 1) * 4);
  hipStream_t s = (hipStream_t)hip_stream;
  FE_HIP_TRY(hipMemcpyAsync(fe->idx_dev, hs, fe->idx_bytes, hipMemcpyHostToDevice, s));
  FE_HIP_TRY(hipEventRecord(fe->idx_evt[slot], s));
  fe->idx_used[slot] = true;
  fe->idx_next = (slot + 1) % kIdxSlots;
  if (frames == 0) return WF_OK;

  FeArgs a{};
  a.audio = audio_dev; a.hush = fe->hush; a.window = fe->window; a.basis_c = fe->basis_c; a.basis_s = fe->basis_s;
  a.fbank = fe->fbank; a.fb_lo = fe->fb_lo; a.fb_hi = fe->fb_hi;
  a.sample_offset = (const int64_t *)fe->idx_dev;
  a.n_samples = (const int32_t *)(fe->idx_dev + (size_t)S * 8);
  a.cu_frames = a.n_samples + S;
  a.frame_stream = fe->frame_stream; a.frame_t = fe->frame_t; a.V = fe->V; a.smax = fe->smax; a.out = mel_out_dev;
  a.B = B; a.F = (int32_t)frames; a.H = H; a.n_mels = fe->cfg.n_mels; a.out_bf16 = mel_dtype == WF_DTYPE_BF16;
  const int F = (int)frames;
  const int nmap = F > B ? F : B;
  hipLaunchKernelGGL(frame_map_kernel, dim3((nmap + 255) / 256), dim3(256), 0, s, a);
  hipLaunchKernelGGL(stft_mel_kernel, dim3((F + kFramesPerBlock - 1) / kFramesPerBlock), dim3(448),
                     kFramesPerBlock * kRowStride * 4, s, a);
  const long n = (long)F * a.n_mels;
  if (a.out_bf16) hipLaunchKernelGGL(normalize_kernel<__bf16>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, a);
  else hipLaunchKernelGGL(normalize_kernel<float>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, a);
  hipError_t err = hipGetLastError();
  if (err != hipSuccess) return ffail(WF_E_HIP, "front-end launch: %s", hipGetErrorString(err));
  return WF_OK;
}

}  // extern "C"
