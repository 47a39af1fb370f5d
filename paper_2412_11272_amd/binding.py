"""ctypes binding of libwf_encoder.so: the same entry points as include/wf_encoder.h, argument
marshalling only.  PyTorch appears here solely as the owner of device buffers and streams.

There is no fallback: if the shared library is missing, loading raises."""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libwf_encoder.so")

WF_OK, WF_E_INVALID_ARG, WF_E_CAPACITY, WF_E_OOM, WF_E_HIP = 0, -1, -2, -3, -4
WF_DTYPE_F32, WF_DTYPE_BF16 = 0, 1
WF_PRECISION_BF16, WF_PRECISION_F32 = 0, 1

_fp = C.POINTER(C.c_float)
_ip = C.POINTER(C.c_int32)


class WfConfig(C.Structure):
    _fields_ = [("n_mels", C.c_int32), ("d_model", C.c_int32), ("n_layers", C.c_int32), ("n_heads", C.c_int32),
                ("d_mlp", C.c_int32), ("hush_frames", C.c_int32), ("max_streams", C.c_int32),
                ("max_total_frames", C.c_int32), ("max_frames_per_stream", C.c_int32), ("precision", C.c_int32),
                ("ln_eps", C.c_float)]


_LAYER_FIELDS = ["ln1_g", "ln1_b", "wq", "bq", "wk", "bk", "wv", "bv", "wo", "bo", "ln2_g", "ln2_b", "w1", "b1", "w2", "b2"]


class WfLayerWeights(C.Structure):
    _fields_ = [(n, _fp) for n in _LAYER_FIELDS]


class WfWeights(C.Structure):
    _fields_ = [("conv1_w", _fp), ("conv1_b", _fp), ("conv2_w", _fp), ("conv2_b", _fp), ("hush_mel", _fp),
                ("layers", C.POINTER(WfLayerWeights)), ("lnf_g", _fp), ("lnf_b", _fp)]


class WfKernelStat(C.Structure):
    _fields_ = [("name", C.c_char_p), ("launches", C.c_int64), ("total_ms", C.c_double), ("flops", C.c_double),
                ("bytes", C.c_double)]


class WfFrontendConfig(C.Structure):
    _fields_ = [("n_mels", C.c_int32), ("hush_samples", C.c_int32), ("max_streams", C.c_int32),
                ("max_total_samples", C.c_int64)]


class WfDecoderConfig(C.Structure):
    _fields_ = [("d_model", C.c_int32), ("n_layers", C.c_int32), ("n_heads", C.c_int32), ("d_mlp", C.c_int32),
                ("n_vocab", C.c_int32), ("n_ctx", C.c_int32), ("max_streams", C.c_int32), ("max_enc_tokens", C.c_int32),
                ("max_prompt_tokens", C.c_int32), ("precision", C.c_int32), ("ln_eps", C.c_float)]


_DEC_LAYER_FIELDS = ["ln1_g", "ln1_b", "wq", "bq", "wk", "wv", "bv", "wo", "bo", "lnx_g", "lnx_b", "xwq", "xbq", "xwk", "xwv",
                     "xbv", "xwo", "xbo", "ln2_g", "ln2_b", "w1", "b1", "w2", "b2"]


class WfDecoderLayerWeights(C.Structure):
    _fields_ = [(n, _fp) for n in _DEC_LAYER_FIELDS]


class WfDecoderWeights(C.Structure):
    _fields_ = [("tok_emb", _fp), ("pos_emb", _fp), ("layers", C.POINTER(WfDecoderLayerWeights)), ("lnf_g", _fp), ("lnf_b", _fp)]


class WfRoundsConfig(C.Structure):
    _fields_ = [("n_streams", C.c_int32), ("step_us", C.c_int64), ("trim_frames", C.c_int32), ("keep_frames", C.c_int32),
                ("max_frames", C.c_int32)]


class WfRoundsStats(C.Structure):
    _fields_ = [("rounds", C.c_int64), ("mean_latency_us", C.c_double), ("mean_proc_us", C.c_double),
                ("max_proc_us", C.c_int64), ("frames_total", C.c_int64), ("last_round_end_us", C.c_int64)]


class WfRoundRecord(C.Structure):
    _fields_ = [("start_us", C.c_int64), ("end_us", C.c_int64), ("proc_us", C.c_int64), ("frames", C.c_int64),
                ("tokens", C.c_int64), ("n_active", C.c_int32), ("reserved", C.c_int32)]


class WfError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"wf error {code}: {msg}")
        self.code = code


_lib = None

EXPORTS = ["wf_encoder_create", "wf_encode_batch", "wf_encoder_destroy", "wf_last_error", "wf_plan_batch",
           "wf_config_check", "wf_kernel_class_count", "wf_encoder_set_profiling", "wf_encoder_kernel_stats",
           "wf_op_linear", "wf_op_layernorm", "wf_op_attention",
           "wf_frontend_create", "wf_logmel_batch", "wf_frontend_destroy",
           "wf_decoder_config_check", "wf_decoder_create", "wf_cross_kv", "wf_prefill", "wf_decoder_destroy",
           "wf_decoder_kernel_class_count", "wf_decoder_set_profiling", "wf_decoder_kernel_stats",
           "wf_encoder_get_config", "wf_encoder_set_lanes", "wf_encoder_get_lanes", "wf_rounds_create", "wf_rounds_begin", "wf_rounds_end", "wf_rounds_get_stats", "wf_rounds_reset_stats",
           "wf_rounds_destroy", "wf_run_rounds",
           "wf_beam_pruner_create", "wf_beam_pruner_step", "wf_beam_pruner_reset", "wf_beam_prune_session",
           "wf_beam_pruner_destroy", "wf_op_attention_noalloc",
           "wf_encoder_set_graphs", "wf_encoder_graph_stats", "wf_gemm_tile_map", "wf_gemm_tile_choice", "wf_gelu_host", "wf_device_info", "wf_op_ln_linear"]


def lib() -> C.CDLL:
    """Load the shared library (once).  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} not found: build it with `python -m paper_2412_11272_amd.build`")
    # PyTorch ships its own HIP runtime (soname libamdhip64.so.7).  Import it first so that this
    # library binds to that same runtime: device pointers and streams are only meaningful within one.
    import torch  # noqa: F401
    L = C.CDLL(LIB_PATH)
    L.wf_last_error.restype = C.c_char_p
    L.wf_encoder_create.argtypes = [C.POINTER(WfConfig), C.POINTER(WfWeights), C.POINTER(C.c_void_p)]
    L.wf_encode_batch.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, _ip, _ip, C.c_int32, C.c_void_p, C.c_int32,
                                  C.c_int64, _ip, C.c_void_p]
    L.wf_encoder_destroy.argtypes = [C.c_void_p]
    L.wf_encoder_destroy.restype = None
    L.wf_plan_batch.argtypes = [C.POINTER(WfConfig), _ip, C.c_int32, _ip, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
    L.wf_config_check.argtypes = [C.POINTER(WfConfig)]
    L.wf_encoder_set_profiling.argtypes = [C.c_void_p, C.c_int32]
    L.wf_encoder_kernel_stats.argtypes = [C.c_void_p, C.POINTER(WfKernelStat), C.c_int32]
    L.wf_op_linear.argtypes = [C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32,
                               C.c_int32, C.c_int32, C.c_void_p]
    L.wf_op_layernorm.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32,
                                  C.c_float, C.c_void_p]
    L.wf_op_attention.argtypes = [C.c_int32, C.c_void_p, C.c_void_p, _ip, C.c_int32, C.c_int32, C.c_void_p]
    L.wf_op_attention_noalloc.argtypes = [C.c_int32, C.c_void_p, C.c_void_p, _ip, C.c_int32, C.c_int32, C.c_void_p]
    L.wf_frontend_create.argtypes = [C.POINTER(WfFrontendConfig), C.c_void_p, C.POINTER(C.c_void_p)]
    L.wf_logmel_batch.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_int64), _ip, C.c_int32, C.c_void_p, C.c_int32,
                                  C.c_int64, _ip, C.c_void_p]
    L.wf_frontend_destroy.argtypes = [C.c_void_p]
    L.wf_frontend_destroy.restype = None
    L.wf_decoder_config_check.argtypes = [C.POINTER(WfDecoderConfig)]
    L.wf_decoder_create.argtypes = [C.POINTER(WfDecoderConfig), C.POINTER(WfDecoderWeights), C.POINTER(C.c_void_p)]
    L.wf_cross_kv.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_int64, C.c_void_p]
    L.wf_prefill.argtypes = [C.c_void_p, _ip, _ip, _ip, C.c_int32, C.c_void_p, C.c_int64, C.c_void_p, C.c_int32, C.c_void_p,
                             C.c_void_p, C.c_int64, C.c_void_p]
    L.wf_decoder_destroy.argtypes = [C.c_void_p]
    L.wf_decoder_destroy.restype = None
    L.wf_decoder_set_profiling.argtypes = [C.c_void_p, C.c_int32]
    L.wf_decoder_kernel_stats.argtypes = [C.c_void_p, C.POINTER(WfKernelStat), C.c_int32]
    L.wf_encoder_get_config.argtypes = [C.c_void_p, C.POINTER(WfConfig)]
    L.wf_encoder_set_lanes.argtypes = [C.c_void_p, C.c_int32]
    L.wf_encoder_get_lanes.argtypes = [C.c_void_p]
    L.wf_device_info.argtypes = [_ip, _ip]
    L.wf_op_ln_linear.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32,
                                  C.c_int32, C.c_int32, C.c_int32, C.c_void_p]
    L.wf_gemm_tile_map.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32, _ip, C.c_int32]
    L.wf_gemm_tile_choice.argtypes = [C.c_int32, C.c_int32, _ip, _ip]
    L.wf_gelu_host.argtypes = [C.POINTER(C.c_float), C.POINTER(C.c_float), C.c_int32]
    L.wf_encoder_set_graphs.argtypes = [C.c_void_p, C.c_int32]
    _lp = C.POINTER(C.c_int64)
    L.wf_encoder_graph_stats.argtypes = [C.c_void_p, _lp, _lp, _lp]
    L.wf_rounds_create.argtypes = [C.POINTER(WfRoundsConfig), _lp, C.POINTER(C.c_void_p)]
    L.wf_rounds_begin.argtypes = [C.c_void_p, _lp, _ip, _ip]
    L.wf_rounds_end.argtypes = [C.c_void_p, C.c_int64, _lp]
    L.wf_rounds_get_stats.argtypes = [C.c_void_p, C.POINTER(WfRoundsStats)]
    L.wf_rounds_reset_stats.argtypes = [C.c_void_p]
    L.wf_beam_pruner_create.argtypes = [C.c_int32, _ip, C.c_int32, C.c_int32, _ip, C.c_int32, C.c_int32, C.POINTER(C.c_void_p)]
    L.wf_beam_pruner_step.argtypes = [C.c_void_p, C.c_int32, _ip, _ip]
    L.wf_beam_pruner_reset.argtypes = [C.c_void_p, _ip, C.c_int32]
    L.wf_beam_prune_session.argtypes = [C.c_void_p, _ip, C.c_int32, _ip, _ip]
    L.wf_beam_pruner_destroy.argtypes = [C.c_void_p]
    L.wf_beam_pruner_destroy.restype = None
    L.wf_rounds_destroy.argtypes = [C.c_void_p]
    L.wf_rounds_destroy.restype = None
    L.wf_run_rounds.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_int32, C.c_int32, C.c_void_p,
                                C.c_int32, C.c_int64, C.POINTER(WfRoundRecord), C.c_void_p]
    _lib = L
    return L


def _check(rc: int):
    if rc != WF_OK:
        raise WfError(rc, lib().wf_last_error().decode())


def last_error() -> str:
    return lib().wf_last_error().decode()


def make_config(shape, hush_frames: int, max_streams: int, max_total_frames: int, max_frames_per_stream: int,
                precision: int = WF_PRECISION_BF16, ln_eps: float = 1e-5) -> WfConfig:
    return WfConfig(shape.n_mels, shape.d_model, shape.n_layers, shape.n_heads, shape.d_mlp, hush_frames, max_streams,
                    max_total_frames, max_frames_per_stream, precision, ln_eps)


def config_check(cfg: WfConfig) -> int:
    return lib().wf_config_check(C.byref(cfg))


def plan_batch(cfg: WfConfig, n_frames: Sequence[int]) -> Tuple[np.ndarray, int, int]:
    """Host-only planner: returns (cu_seqlens, total_frames, total_tokens) or raises WfError."""
    B = len(n_frames)
    nf = np.ascontiguousarray(n_frames, dtype=np.int32)
    cu = np.zeros(B + 1, dtype=np.int32)
    tf, tt = C.c_int64(0), C.c_int64(0)
    _check(lib().wf_plan_batch(C.byref(cfg), nf.ctypes.data_as(_ip), B, cu.ctypes.data_as(_ip), C.byref(tf), C.byref(tt)))
    return cu, tf.value, tt.value


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


class Encoder:
    """Owns one wf_encoder.  weights: the dict layout of synth.make_weights (host fp32 arrays)."""

    def __init__(self, cfg: WfConfig, weights: dict, hush: Optional[np.ndarray]):
        self.cfg = cfg
        self._h = C.c_void_p(None)
        keep: List[np.ndarray] = []          # host arrays must outlive the create call only

        def p(a):
            if a is None:
                return None
            a = _f32(a)
            keep.append(a)
            return a.ctypes.data_as(_fp)

        n_layers = len(weights["layers"])
        layers = (WfLayerWeights * max(n_layers, 1))()
        for i, lw in enumerate(weights["layers"]):
            for name in _LAYER_FIELDS:
                setattr(layers[i], name, p(lw.get(name)))
        w = WfWeights(p(weights["conv1_w"]), p(weights["conv1_b"]), p(weights["conv2_w"]), p(weights["conv2_b"]),
                      p(hush) if (hush is not None and len(hush) > 0) else None,
                      layers, p(weights["lnf_g"]), p(weights["lnf_b"]))
        _check(lib().wf_encoder_create(C.byref(cfg), C.byref(w), C.byref(self._h)))

    def encode(self, mel, frame_offset: Sequence[int], n_frames: Sequence[int], out=None, out_dtype=None, stream=None):
        """mel: CUDA tensor [*, n_mels] (float32 or bfloat16).  Returns (out [M, d] CUDA tensor, cu_seqlens ndarray).
        Asynchronous on `stream` (default: torch's current stream)."""
        import torch
        B = len(n_frames)
        cu, _, M = plan_batch(self.cfg, n_frames) if 1 <= B <= self.cfg.max_streams else (np.zeros(B + 1, np.int32), 0, 0)
        if out is None:      # at least one row, so that an invalid batch reaches the library's own checks
            out = torch.empty((max(M, 1), self.cfg.d_model), device=mel.device, dtype=out_dtype or torch.float32)[:M]
        s = stream if stream is not None else torch.cuda.current_stream().cuda_stream
        off = np.ascontiguousarray(frame_offset, dtype=np.int32)
        nf = np.ascontiguousarray(n_frames, dtype=np.int32)
        cu_out = np.zeros(B + 1, dtype=np.int32)
        _check(lib().wf_encode_batch(self._h, C.c_void_p(mel.data_ptr()), _torch_dtype_code(mel.dtype),
                                     off.ctypes.data_as(_ip), nf.ctypes.data_as(_ip), B,
                                     C.c_void_p(out.data_ptr() or out.untyped_storage().data_ptr()), _torch_dtype_code(out.dtype), out.shape[0],
                                     cu_out.ctypes.data_as(_ip), C.c_void_p(s)))
        return out, cu_out

    def set_profiling(self, on: bool):
        _check(lib().wf_encoder_set_profiling(self._h, 1 if on else 0))

    def set_lanes(self, n: int):
        _check(lib().wf_encoder_set_lanes(self._h, int(n)))

    def set_graphs(self, enabled: bool):
        _check(lib().wf_encoder_set_graphs(self._h, 1 if enabled else 0))

    def graph_stats(self) -> dict:
        r, c, d = C.c_int64(0), C.c_int64(0), C.c_int64(0)
        _check(lib().wf_encoder_graph_stats(self._h, C.byref(r), C.byref(c), C.byref(d)))
        return {"replays": r.value, "captures": c.value, "direct_calls": d.value}

    def get_lanes(self) -> int:
        n = lib().wf_encoder_get_lanes(self._h)
        _check(min(n, 0))
        return n

    def kernel_stats(self) -> List[dict]:
        n = lib().wf_kernel_class_count()
        st = (WfKernelStat * n)()
        _check(lib().wf_encoder_kernel_stats(self._h, st, n))
        return [{"name": s.name.decode(), "launches": s.launches, "total_ms": s.total_ms, "flops": s.flops, "bytes": s.bytes}
                for s in st]

    def close(self):
        if self._h:
            lib().wf_encoder_destroy(self._h)
            self._h = C.c_void_p(None)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Frontend:
    """Owns one wf_frontend: raw 16 kHz audio (+ hush word appended at the raw level) -> packed log-mel."""

    def __init__(self, n_mels: int, hush_audio: Optional[np.ndarray], max_streams: int, max_total_samples: int):
        h = None if hush_audio is None or len(hush_audio) == 0 else _f32(hush_audio)
        self.cfg = WfFrontendConfig(n_mels, 0 if h is None else len(h), max_streams, max_total_samples)
        self._h = C.c_void_p(None)
        _check(lib().wf_frontend_create(C.byref(self.cfg), None if h is None else h.ctypes.data_as(C.c_void_p),
                                        C.byref(self._h)))

    def n_frames(self, n_samples: Sequence[int]) -> List[int]:
        return [(int(n) + self.cfg.hush_samples) // 160 for n in n_samples]

    def logmel(self, audio, sample_offset: Sequence[int], n_samples: Sequence[int], out=None, out_dtype=None, stream=None):
        """audio: CUDA float32 tensor of samples.  Returns (mel [sum T', n_mels] CUDA tensor, cu_frames ndarray)."""
        import torch
        B = len(n_samples)
        F = sum(self.n_frames(n_samples))
        if out is None:
            out = torch.empty((max(F, 1), self.cfg.n_mels), device=audio.device, dtype=out_dtype or torch.float32)[:F]
        s = stream if stream is not None else torch.cuda.current_stream().cuda_stream
        off = np.ascontiguousarray(sample_offset, dtype=np.int64)
        ns = np.ascontiguousarray(n_samples, dtype=np.int32)
        cu = np.zeros(B + 1, dtype=np.int32)
        _check(lib().wf_logmel_batch(self._h, C.c_void_p(audio.data_ptr()), off.ctypes.data_as(C.POINTER(C.c_int64)),
                                     ns.ctypes.data_as(_ip), B, C.c_void_p(out.data_ptr() or out.untyped_storage().data_ptr()),
                                     _torch_dtype_code(out.dtype), out.shape[0], cu.ctypes.data_as(_ip), C.c_void_p(s)))
        return out, cu

    def close(self):
        if self._h:
            lib().wf_frontend_destroy(self._h)
            self._h = C.c_void_p(None)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Decoder:
    """Owns one wf_decoder: cross-attention K/V projection of the encoder states and prompt prefill.
    weights: the dict layout of synth.make_decoder_weights (host fp32 arrays)."""

    def __init__(self, shape, weights: dict, max_streams: int, max_enc_tokens: int, max_prompt_tokens: int,
                 precision: int = WF_PRECISION_BF16, ln_eps: float = 1e-5):
        self.cfg = WfDecoderConfig(shape.d_model, shape.n_layers, shape.n_heads, shape.d_mlp, shape.n_vocab, shape.n_ctx,
                                   max_streams, max_enc_tokens, max_prompt_tokens, precision, ln_eps)
        self._h = C.c_void_p(None)
        keep: List[np.ndarray] = []

        def p(a):
            if a is None:
                return None
            a = _f32(a)
            keep.append(a)
            return a.ctypes.data_as(_fp)

        n_layers = len(weights["layers"])
        layers = (WfDecoderLayerWeights * max(n_layers, 1))()
        for i, lw in enumerate(weights["layers"]):
            for name in _DEC_LAYER_FIELDS:
                setattr(layers[i], name, p(lw.get(name)))
        w = WfDecoderWeights(p(weights["tok_emb"]), p(weights["pos_emb"]), layers, p(weights["lnf_g"]), p(weights["lnf_b"]))
        _check(lib().wf_decoder_create(C.byref(self.cfg), C.byref(w), C.byref(self._h)))

    @property
    def act_dtype(self):
        import torch
        return torch.bfloat16 if self.cfg.precision == WF_PRECISION_BF16 else torch.float32

    def cross_kv(self, enc, out=None, stream=None):
        """enc: CUDA [M, d] in the activation dtype.  Returns [n_layers, M, 2 d] (keys | values)."""
        import torch
        M = enc.shape[0]
        if out is None:
            out = torch.empty((self.cfg.n_layers, max(M, 1), 2 * self.cfg.d_model), device=enc.device, dtype=self.act_dtype)
        s = stream if stream is not None else torch.cuda.current_stream().cuda_stream
        _check(lib().wf_cross_kv(self._h, C.c_void_p(enc.data_ptr()), M, C.c_void_p(out.data_ptr()), out.shape[1], C.c_void_p(s)))
        return out

    def prefill(self, prompts: Sequence[Sequence[int]], cu_seqlens: Sequence[int], cross_kv, hidden_dtype=None,
                want_logits: bool = True, want_self_kv: bool = False, hidden=None, logits=None, self_kv=None, stream=None):
        """prompts: per-stream token ids (host).  cross_kv: what cross_kv() returned for the same batch.
        Returns dict(hidden [sum P, d], logits [B, n_vocab] fp32, self_kv [n_layers, sum P, 2 d], cu_prompt)."""
        import torch
        B = len(prompts)
        lens = [len(p) for p in prompts]
        cup = np.zeros(B + 1, dtype=np.int32)
        cup[1:] = np.cumsum(lens)
        Pt = int(cup[-1])
        tok = np.ascontiguousarray(np.concatenate([np.asarray(p, dtype=np.int32) for p in prompts]) if Pt else np.zeros(1, np.int32))
        cus = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
        dev = cross_kv.device
        if hidden is None and hidden_dtype is not None:
            hidden = torch.empty((max(Pt, 1), self.cfg.d_model), device=dev, dtype=hidden_dtype)
        if logits is None and want_logits:
            logits = torch.empty((max(B, 1), self.cfg.n_vocab), device=dev, dtype=torch.float32)
        if self_kv is None and want_self_kv:
            self_kv = torch.empty((self.cfg.n_layers, max(Pt, 1), 2 * self.cfg.d_model), device=dev, dtype=self.act_dtype)
        s = stream if stream is not None else torch.cuda.current_stream().cuda_stream
        _check(lib().wf_prefill(self._h, tok.ctypes.data_as(_ip), cup.ctypes.data_as(_ip), cus.ctypes.data_as(_ip), B,
                                C.c_void_p(cross_kv.data_ptr()), cross_kv.shape[1],
                                C.c_void_p(hidden.data_ptr()) if hidden is not None else None,
                                _torch_dtype_code(hidden.dtype) if hidden is not None else 0,
                                C.c_void_p(logits.data_ptr()) if logits is not None else None,
                                C.c_void_p(self_kv.data_ptr()) if self_kv is not None else None,
                                self_kv.shape[1] if self_kv is not None else 0, C.c_void_p(s)))
        return {"hidden": hidden[:Pt] if hidden is not None else None, "logits": logits[:B] if logits is not None else None,
                "self_kv": self_kv, "cu_prompt": cup}

    def set_profiling(self, on: bool):
        _check(lib().wf_decoder_set_profiling(self._h, 1 if on else 0))

    def kernel_stats(self) -> List[dict]:
        n = lib().wf_decoder_kernel_class_count()
        st = (WfKernelStat * n)()
        _check(lib().wf_decoder_kernel_stats(self._h, st, n))
        return [{"name": s.name.decode(), "launches": s.launches, "total_ms": s.total_ms, "flops": s.flops, "bytes": s.bytes}
                for s in st]

    def close(self):
        if self._h:
            lib().wf_decoder_destroy(self._h)
            self._h = C.c_void_p(None)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Rounds:
    """Owns one wf_rounds: snapshot / trimming / latency bookkeeping of processing rounds (host only),
    and run(): the driver that pushes every round's ragged batch through an Encoder."""

    def __init__(self, start_us: Sequence[int], step_us: int, trim_frames: int = 1500, keep_frames: int = 100,
                 max_frames: int = 3000):
        st = np.ascontiguousarray(start_us, dtype=np.int64)
        self.cfg = WfRoundsConfig(len(st), step_us, trim_frames, keep_frames, max_frames)
        self._h = C.c_void_p(None)
        _check(lib().wf_rounds_create(C.byref(self.cfg), st.ctypes.data_as(C.POINTER(C.c_int64)), C.byref(self._h)))

    def begin(self):
        S = self.cfg.n_streams
        n, f, s = np.zeros(S, np.int32), np.zeros(S, np.int32), C.c_int64(0)
        _check(lib().wf_rounds_begin(self._h, C.byref(s), n.ctypes.data_as(_ip), f.ctypes.data_as(_ip)))
        return s.value, n, f

    def end(self, proc_us: int) -> int:
        e = C.c_int64(0)
        _check(lib().wf_rounds_end(self._h, int(proc_us), C.byref(e)))
        return e.value

    def stats(self) -> dict:
        st = WfRoundsStats()
        _check(lib().wf_rounds_get_stats(self._h, C.byref(st)))
        return {k: getattr(st, k) for k, _ in WfRoundsStats._fields_}

    def reset_stats(self):
        _check(lib().wf_rounds_reset_stats(self._h))

    def run(self, enc: "Encoder", tracks, n_rounds: int, out, pad_to_frames: int = 0, stream=None) -> List[dict]:
        """tracks: CUDA [n_streams, track_frames, n_mels]; out: CUDA [capacity, d_model].  Returns per-round records."""
        import torch
        rec = (WfRoundRecord * max(n_rounds, 1))()
        s = stream if stream is not None else torch.cuda.current_stream().cuda_stream
        _check(lib().wf_run_rounds(self._h, enc._h, C.c_void_p(tracks.data_ptr()), _torch_dtype_code(tracks.dtype), tracks.shape[1],
                                   pad_to_frames, n_rounds, C.c_void_p(out.data_ptr()), _torch_dtype_code(out.dtype), out.shape[0],
                                   rec, C.c_void_p(s)))
        return [{k: getattr(rec[i], k) for k, _ in WfRoundRecord._fields_ if k != "reserved"} for i in range(n_rounds)]

    def close(self):
        if self._h:
            lib().wf_rounds_destroy(self._h)
            self._h = C.c_void_p(None)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class BeamPruner:
    """Owns one wf_beam_pruner: the reference-based beam-size state machine (host only)."""

    def __init__(self, beam_size: int, reference: Sequence[int], special_from: int, punctuation: Sequence[int] = (),
                 filter_reference: bool = True):
        ref = np.ascontiguousarray(reference, dtype=np.int32)
        pun = np.ascontiguousarray(list(punctuation), dtype=np.int32)
        self._h = C.c_void_p(None)
        _check(lib().wf_beam_pruner_create(beam_size, ref.ctypes.data_as(_ip) if len(ref) else None, len(ref), special_from,
                                           pun.ctypes.data_as(_ip) if len(pun) else None, len(pun),
                                           1 if filter_reference else 0, C.byref(self._h)))

    def step(self, best_token: int) -> Tuple[int, int]:
        ev, nb = C.c_int32(0), C.c_int32(0)
        _check(lib().wf_beam_pruner_step(self._h, int(best_token), C.byref(ev), C.byref(nb)))
        return ev.value, nb.value

    def reset(self, reference: Sequence[int]):
        ref = np.ascontiguousarray(reference, dtype=np.int32)
        _check(lib().wf_beam_pruner_reset(self._h, ref.ctypes.data_as(_ip) if len(ref) else None, len(ref)))

    def session(self, best_tokens: Sequence[int]) -> Tuple[np.ndarray, np.ndarray]:
        """Returns (beam size each step ran with, event of each step)."""
        tok = np.ascontiguousarray(best_tokens, dtype=np.int32)
        beams, events = np.zeros(len(tok), np.int32), np.zeros(len(tok), np.int32)
        _check(lib().wf_beam_prune_session(self._h, tok.ctypes.data_as(_ip) if len(tok) else None, len(tok),
                                           beams.ctypes.data_as(_ip), events.ctypes.data_as(_ip)))
        return beams, events

    def close(self):
        if self._h:
            lib().wf_beam_pruner_destroy(self._h)
            self._h = C.c_void_p(None)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def _torch_dtype_code(dt) -> int:
    import torch
    if dt == torch.float32:
        return WF_DTYPE_F32
    if dt == torch.bfloat16:
        return WF_DTYPE_BF16
    raise TypeError(f"unsupported dtype {dt}")


def pack_mels(mels: Sequence[np.ndarray]):
    """Concatenate per-stream host buffers into one [sum T_i, n_mels] array + (frame_offset, n_frames)."""
    n_frames = [int(m.shape[0]) for m in mels]
    offs = np.concatenate([[0], np.cumsum(n_frames)[:-1]]).astype(np.int32)
    return np.concatenate(mels, axis=0).astype(np.float32), offs, np.asarray(n_frames, np.int32)


def encoder_for_workload(wl, weights, hush, precision: int = WF_PRECISION_BF16, slack_streams: int = 0) -> Encoder:
    """Capacity sized exactly for one workload."""
    per = [(m if wl.pad_to_frames is None else max(m, wl.pad_to_frames)) + wl.hush_frames for m in wl.n_frames]
    cfg = make_config(wl.shape, wl.hush_frames, len(per) + slack_streams, sum(per), max(per), precision)
    return Encoder(cfg, weights, hush)


# ---- operator-level entry points ---------------------------------------------------------------
def op_linear(precision: int, a, w, bias, out, epilogue: int, stream=None):
    import torch
    M, K = a.shape
    N = w.shape[0]
    s = stream if stream is not None else torch.cuda.current_stream().cuda_stream
    _check(lib().wf_op_linear(precision, C.c_void_p(a.data_ptr()), C.c_void_p(w.data_ptr()), C.c_void_p(bias.data_ptr()),
                              C.c_void_p(out.data_ptr()), M, N, K, epilogue, C.c_void_p(s)))
    return out


def op_layernorm(x, g, b, out, eps: float = 1e-5, stream=None):
    import torch
    M, d = x.shape
    s = stream if stream is not None else torch.cuda.current_stream().cuda_stream
    _check(lib().wf_op_layernorm(C.c_void_p(x.data_ptr()), C.c_void_p(g.data_ptr()), C.c_void_p(b.data_ptr()),
                                 C.c_void_p(out.data_ptr()), _torch_dtype_code(out.dtype), M, d, eps, C.c_void_p(s)))
    return out


def op_attention(precision: int, qkv, out, cu_seqlens: Sequence[int], n_heads: int, stream=None):
    import torch
    cu = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
    s = stream if stream is not None else torch.cuda.current_stream().cuda_stream
    _check(lib().wf_op_attention(precision, C.c_void_p(qkv.data_ptr()), C.c_void_p(out.data_ptr()), cu.ctypes.data_as(_ip),
                                 len(cu) - 1, n_heads, C.c_void_p(s)))
    return out


def op_attention_noalloc(precision: int, qkv, out, cu_seqlens: Sequence[int], n_heads: int, stream=None):
    """wf_op_attention_noalloc: same result as op_attention, no device allocation, asynchronous on the stream."""
    import torch
    cu = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
    s = stream if stream is not None else torch.cuda.current_stream().cuda_stream
    _check(lib().wf_op_attention_noalloc(precision, C.c_void_p(qkv.data_ptr()), C.c_void_p(out.data_ptr()), cu.ctypes.data_as(_ip),
                                         len(cu) - 1, n_heads, C.c_void_p(s)))
    return out


def gemm_tile_map(M: int, N: int, tile_m: int = 256, tile_n: int = 256) -> np.ndarray:
    """[n_units, 3] (first row, first column, width) of the GEMM's work units in workgroup order (host only)."""
    cap = 2 * ((M + tile_m - 1) // tile_m) * (N // tile_n) + 8
    units = np.zeros((cap, 3), dtype=np.int32)
    n = lib().wf_gemm_tile_map(M, N, tile_m, tile_n, units.ctypes.data_as(_ip), cap)
    _check(min(n, 0))
    return units[:n]


def gemm_tile_choice(M: int, N: int) -> tuple:
    """(tile rows, tile columns) the bf16 MFMA GEMM picks for an M x N product; (0, 0) = small-batch kernel (host only)."""
    tm, tn = C.c_int32(0), C.c_int32(0)
    _check(lib().wf_gemm_tile_choice(M, N, C.byref(tm), C.byref(tn)))
    return tm.value, tn.value


def gelu_host(z: np.ndarray) -> np.ndarray:
    """The bf16 kernels' GELU evaluated on the host by the library's own code (host only)."""
    z = np.ascontiguousarray(z, dtype=np.float32)
    out = np.empty_like(z)
    fp = C.POINTER(C.c_float)
    _check(lib().wf_gelu_host(z.ctypes.data_as(fp), out.ctypes.data_as(fp), z.size))
    return out


def device_info() -> dict:
    """Compute units and maximum shader clock (kHz) of the current device, as the HIP runtime reports them."""
    cu, khz = C.c_int32(0), C.c_int32(0)
    _check(lib().wf_device_info(C.byref(cu), C.byref(khz)))
    return {"compute_units": cu.value, "clock_khz": khz.value}


def op_ln_linear(x, g, b, w, bias, out, epilogue: int, eps: float = 1e-5, stream=None):
    """out = epilogue(LayerNorm(x) w^T + bias) on the small-batch kernel (x fp32 [M, K], w bf16 [N, K], out bf16 [M, N])."""
    import torch
    M, K = x.shape
    N = w.shape[0]
    s = stream if stream is not None else torch.cuda.current_stream().cuda_stream
    _check(lib().wf_op_ln_linear(C.c_void_p(x.data_ptr()), C.c_void_p(g.data_ptr()), C.c_void_p(b.data_ptr()), eps,
                                 C.c_void_p(w.data_ptr()), C.c_void_p(bias.data_ptr()), C.c_void_p(out.data_ptr()), M, N, K, epilogue,
                                 C.c_void_p(s)))
    return out
