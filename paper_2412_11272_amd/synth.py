"""Seeded synthetic inputs: encoder shapes, weights, log-mel buffers, hush segment, buffer lengths.

This module draws random numbers and nothing else.  It holds none of the encoder's
arithmetic, so it can feed both the HIP path and the CPU oracle used by the tests
without making either depend on the other.

The inputs stand in for the paper's workloads (Section "Methodology": streaming
buffers of a few to ~15 s and short-form clips of 5-25 s; Section "Hush word":
1 s of audio is a (100, 80) log-mel matrix and the hush word is 0.5 s long).  No
dataset item, trained weight or trained hush word is reproduced: every value below is
drawn from a seeded NumPy generator.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

BASE_SEED = 241211272
FRAMES_PER_SECOND = 100      # Section "Hush word", target-level paragraph: 1 s -> (100, 80)
HUSH_FRAMES = 50             # 0.5 s hush word (Section "Hush word", length paragraph)
WEIGHT_STD = 0.02
MEL_MEAN, MEL_STD = -0.3, 0.4
PAD_VALUE = -1.0             # clip floor, used as "silence" in the padded 30 s window


@dataclass(frozen=True)
class Shape:
    """Encoder architecture."""
    n_mels: int
    d_model: int
    n_layers: int
    n_heads: int
    d_mlp: int

    @property
    def d_head(self) -> int:
        return self.d_model // self.n_heads


SHAPES: Dict[str, Shape] = {
    "tiny": Shape(80, 384, 4, 6, 1536),
    "base": Shape(80, 512, 6, 8, 2048),
    "small": Shape(80, 768, 12, 12, 3072),
    "medium": Shape(80, 1024, 24, 16, 4096),
    "large-v3": Shape(128, 1280, 32, 20, 5120),
    # not one of the five benchmark shapes: a two-layer, two-head shape for fast unit tests
    "unit": Shape(16, 128, 2, 2, 256),
    # stem only (no transformer block): lets a test drive the two convolutions at a batch size that takes
    # their large-tile kernels while the oracle still finishes in seconds
    "stem": Shape(128, 256, 0, 4, 1024),
}


@dataclass
class Workload:
    """One batch of streams: the shape, the per-stream payload lengths and the seeds."""
    name: str
    shape: Shape
    n_frames: List[int]                  # T_i, payload mel frames per stream (hush excluded)
    hush_frames: int = HUSH_FRAMES
    seed_index: int = 0                  # c in BASE_SEED + 10 c (+0 weights, +1 mel, +2 hush, +3 lengths)
    pad_to_frames: Optional[int] = None  # padded-window baseline: pad each stream with PAD_VALUE
    q_scale: float = 1.0                 # >1 scales Wq, bq and Wk: sharp softmax (stress case for online softmax)
    note: str = ""
    extra: dict = field(default_factory=dict)

    @property
    def seeds(self):
        b = BASE_SEED + 10 * self.seed_index
        return {"weights": b, "mel": b + 1, "hush": b + 2, "lengths": b + 3}


def _clipped_normal(rng: np.random.Generator, shape) -> np.ndarray:
    x = rng.normal(MEL_MEAN, MEL_STD, size=shape)
    return np.clip(x, -1.0, 1.0).astype(np.float32)


def make_weights(shape: Shape, seed: int, q_scale: float = 1.0) -> dict:
    """All matrices, conv kernels and their biases ~ N(0, 0.02); LayerNorm gain 1, shift 0; no K bias.

    Layout: linear weights are [out, in]; conv kernels are [out_channels, in_channels, 3].
    """
    rng = np.random.default_rng(seed)
    d, f, m = shape.d_model, shape.d_mlp, shape.n_mels

    def n(*s):
        return rng.normal(0.0, WEIGHT_STD, size=s).astype(np.float32)

    w = {
        "conv1_w": n(d, m, 3), "conv1_b": n(d),
        "conv2_w": n(d, d, 3), "conv2_b": n(d),
        "layers": [],
        "lnf_g": np.ones(d, np.float32), "lnf_b": np.zeros(d, np.float32),
    }
    for _ in range(shape.n_layers):
        layer = {
            "ln1_g": np.ones(d, np.float32), "ln1_b": np.zeros(d, np.float32),
            "wq": n(d, d), "bq": n(d),
            "wk": n(d, d), "bk": None,
            "wv": n(d, d), "bv": n(d),
            "wo": n(d, d), "bo": n(d),
            "ln2_g": np.ones(d, np.float32), "ln2_b": np.zeros(d, np.float32),
            "w1": n(f, d), "b1": n(f),
            "w2": n(d, f), "b2": n(d),
        }
        if q_scale != 1.0:
            layer["wq"] = (layer["wq"] * np.float32(q_scale)).astype(np.float32)
            layer["bq"] = (layer["bq"] * np.float32(q_scale)).astype(np.float32)
            layer["wk"] = (layer["wk"] * np.float32(q_scale)).astype(np.float32)
        w["layers"].append(layer)
    return w


def randomize_affine(weights: dict, seed: int) -> dict:
    """Replace the LayerNorm gains/shifts (1/0 in the benchmark recipe) and the absent K bias by
    random values, so tests also exercise those code paths."""
    rng = np.random.default_rng(seed)
    d = weights["lnf_g"].shape[0]

    def g():
        return (1.0 + 0.2 * rng.standard_normal(d)).astype(np.float32)

    def b():
        return (0.1 * rng.standard_normal(d)).astype(np.float32)

    weights["lnf_g"], weights["lnf_b"] = g(), b()
    for layer in weights["layers"]:
        layer["ln1_g"], layer["ln1_b"] = g(), b()
        layer["ln2_g"], layer["ln2_b"] = g(), b()
        layer["bk"] = b()
    return weights


def make_hush(shape: Shape, seed: int, hush_frames: int = HUSH_FRAMES) -> np.ndarray:
    """The fixed appended segment, [hush_frames, n_mels], same for every stream of a model."""
    rng = np.random.default_rng(seed)
    return _clipped_normal(rng, (hush_frames, shape.n_mels))


def make_mels(shape: Shape, n_frames: List[int], seed: int,
              pad_to_frames: Optional[int] = None) -> List[np.ndarray]:
    """Per-stream log-mel buffers, time-major [T_i, n_mels].  With pad_to_frames the seeded frames
    are followed by constant PAD_VALUE frames up to that length (the padded-window baseline)."""
    rng = np.random.default_rng(seed)
    out = []
    for t in n_frames:
        x = _clipped_normal(rng, (t, shape.n_mels))
        if pad_to_frames is not None and pad_to_frames > t:
            pad = np.full((pad_to_frames - t, shape.n_mels), PAD_VALUE, np.float32)
            x = np.concatenate([x, pad], axis=0)
        out.append(x)
    return out


SAMPLE_RATE = 16000           # Section "Hush word", target level: raw audio is sampled at 16 kHz
HUSH_SAMPLES = 8000           # Section "Key Implementation Details": the hush word is a 1-d tensor of shape (8000,)
SAMPLES_PER_FRAME = SAMPLE_RATE // FRAMES_PER_SECOND


def make_audio(n_samples: int, seed: int) -> np.ndarray:
    """Seeded synthetic raw audio in [-1, 1]: a few tones with slow amplitude envelopes over white noise.
    Stands in for the speech recordings of the paper's datasets (none of which is reproduced)."""
    rng = np.random.default_rng(seed)
    t = np.arange(n_samples, dtype=np.float64) / SAMPLE_RATE
    x = 0.02 * rng.standard_normal(n_samples)
    for _ in range(4):
        f = rng.uniform(80.0, 3800.0)
        a = rng.uniform(0.05, 0.25)
        env = 0.5 * (1.0 + np.sin(2 * np.pi * rng.uniform(0.3, 3.0) * t + rng.uniform(0, 2 * np.pi)))
        x += a * env * np.sin(2 * np.pi * f * t + rng.uniform(0, 2 * np.pi))
    return np.clip(x, -1.0, 1.0).astype(np.float32)


def make_audios(n_frames: List[int], seed: int) -> List[np.ndarray]:
    """One raw-audio buffer per stream, n_frames[i] * 160 samples each."""
    return [make_audio(t * SAMPLES_PER_FRAME, seed + 1000 + i) for i, t in enumerate(n_frames)]


def make_hush_audio(seed: int, n_samples: int = HUSH_SAMPLES) -> np.ndarray:
    """The fixed appended raw-audio segment (synthetic: the trained hush words are not available)."""
    return make_audio(n_samples, seed + 500)


# ---- decoder side (cross-attention K/V projection and prompt prefill) -----------------------------

@dataclass(frozen=True)
class DecoderShape:
    """Decoder architecture that goes with an encoder Shape of the same d_model."""
    d_model: int
    n_layers: int
    n_heads: int
    d_mlp: int
    n_vocab: int
    n_ctx: int          # rows of the learned position table


DEC_SHAPES: Dict[str, DecoderShape] = {
    "tiny": DecoderShape(384, 4, 6, 1536, 51865, 448),
    "base": DecoderShape(512, 6, 8, 2048, 51865, 448),
    "small": DecoderShape(768, 12, 12, 3072, 51865, 448),
    "medium": DecoderShape(1024, 24, 16, 4096, 51865, 448),
    "large-v3": DecoderShape(1280, 32, 20, 5120, 51866, 448),
    "unit": DecoderShape(128, 2, 2, 256, 1000, 160),
}
PROMPT_TOKENS = 100          # Section "CPU/GPU pipelining", categorization of workloads: ~100 prompt tokens


def make_decoder_weights(shape: DecoderShape, seed: int, q_scale: float = 1.0, affine_random: bool = False) -> dict:
    """Matrices, embeddings and biases ~ N(0, 0.02); LayerNorm gain 1 / shift 0 unless affine_random.
    Linear weights are [out, in].  Self-attention: wq bq wk wv bv wo bo; cross-attention: xwq xbq xwk
    xwv xbv xwo xbo (key projections carry no bias)."""
    rng = np.random.default_rng(seed)
    d, f = shape.d_model, shape.d_mlp

    def n(*s):
        return rng.normal(0.0, WEIGHT_STD, size=s).astype(np.float32)

    def gain():
        return (1.0 + 0.2 * rng.standard_normal(d)).astype(np.float32) if affine_random else np.ones(d, np.float32)

    def shift():
        return (0.1 * rng.standard_normal(d)).astype(np.float32) if affine_random else np.zeros(d, np.float32)

    w = {"tok_emb": n(shape.n_vocab, d), "pos_emb": n(shape.n_ctx, d), "layers": []}
    qs = np.float32(q_scale)
    for _ in range(shape.n_layers):
        w["layers"].append({
            "ln1_g": gain(), "ln1_b": shift(),
            "wq": n(d, d) * qs, "bq": n(d) * qs, "wk": n(d, d) * qs, "wv": n(d, d), "bv": n(d), "wo": n(d, d), "bo": n(d),
            "lnx_g": gain(), "lnx_b": shift(),
            "xwq": n(d, d) * qs, "xbq": n(d) * qs, "xwk": n(d, d) * qs, "xwv": n(d, d), "xbv": n(d), "xwo": n(d, d), "xbo": n(d),
            "ln2_g": gain(), "ln2_b": shift(),
            "w1": n(f, d), "b1": n(f), "w2": n(d, f), "b2": n(d),
        })
    w["lnf_g"], w["lnf_b"] = gain(), shift()
    return w


def make_prompts(lengths: List[int], n_vocab: int, seed: int) -> List[np.ndarray]:
    """Uniformly drawn token ids, one int32 array per stream."""
    rng = np.random.default_rng(seed)
    return [rng.integers(0, n_vocab, size=int(p), dtype=np.int64).astype(np.int32) for p in lengths]


def make_enc_states(n_tokens: int, d_model: int, seed: int) -> np.ndarray:
    """Stand-in encoder states for decoder-only tests: unit normal, like rows after a LayerNorm."""
    rng = np.random.default_rng(seed)
    return rng.standard_normal((n_tokens, d_model)).astype(np.float32)


# ---- beam pruning: synthetic decoding sessions ------------------------------------------------------

BEAM_SIZE = 5                 # Section "CPU/GPU pipelining", categorization of workloads: 5 hypotheses per round
SESSION_TOKENS = 150          # same passage: a decoding session averages 150 rounds
TEXT_VOCAB = 50257            # ids below this are ordinary text tokens; timestamps / special tokens lie above
PUNCT_IDS = (11, 13, 30, 0)   # a handful of ids standing in for punctuation tokens


def make_beam_sessions(n_sessions: int, seed: int, n_tokens: int = SESSION_TOKENS, trim_max: int = 40, new_max: int = 25,
                       p_substitute: float = 0.004, p_punct: float = 0.08, p_timestamp: float = 0.06):
    """(reference, best_tokens) pairs shaped like consecutive processing rounds over a sliding buffer: the new
    transcript starts somewhere inside the previous one (front trimmed), repeats it with rare substitutions,
    inconsistent punctuation and timestamp tokens, and continues with tokens for the newly arrived audio."""
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n_sessions):
        ref_text = rng.integers(1000, TEXT_VOCAB, size=n_tokens)
        ref = []
        for t in ref_text:
            ref.append(int(t))
            if rng.random() < p_punct:
                ref.append(int(rng.choice(PUNCT_IDS)))
        a = int(rng.integers(0, trim_max + 1))
        cur = [TEXT_VOCAB + 1 + int(rng.integers(0, 1500))]          # leading timestamp
        for t in ref_text[a:]:
            cur.append(int(t) if rng.random() >= p_substitute else int(rng.integers(1000, TEXT_VOCAB)))
            if rng.random() < p_punct:
                cur.append(int(rng.choice(PUNCT_IDS)))
            if rng.random() < p_timestamp:
                cur.append(TEXT_VOCAB + 1 + int(rng.integers(0, 1500)))
        cur += [int(t) for t in rng.integers(1000, TEXT_VOCAB, size=int(rng.integers(0, new_max + 1)))]
        out.append((np.asarray(ref, np.int32), np.asarray(cur, np.int32)))
    return out


def draw_lengths_uniform(n: int, lo_s: float, hi_s: float, seed: int) -> List[int]:
    u = np.random.default_rng(seed).random(n)
    return [int(round(FRAMES_PER_SECOND * (lo_s + (hi_s - lo_s) * x))) for x in u]


def draw_lengths_loguniform(n: int, lo_s: float, hi_s: float, seed: int) -> List[int]:
    u = np.random.default_rng(seed).random(n)
    return [int(round(FRAMES_PER_SECOND * lo_s * (hi_s / lo_s) ** x)) for x in u]


def workload(name: str) -> Workload:
    """The benchmark configurations (and a few unit-sized ones).

    cfg1            tiny, 1 stream of 1.0 s
    cfg2-2s/4s/8s   base, 1 stream of 2 / 4 / 8 s
    cfg3            small, 16 streams, lengths uniform in [1, 10] s
    cfg4a           medium, 8 streams as padded 30 s windows (600 seeded frames + 2400 pad, no hush)
    cfg4b           medium, 8 streams of 6 s + hush
    cfg5            large-v3 shape, 64 streams, lengths log-uniform in [1, 30] s
    """
    S = SHAPES
    if name == "cfg1":
        return Workload(name, S["tiny"], [100], seed_index=1)
    if name in ("cfg2-2s", "cfg2-4s", "cfg2-8s"):
        t = {"cfg2-2s": 200, "cfg2-4s": 400, "cfg2-8s": 800}[name]
        return Workload(name, S["base"], [t], seed_index=2)
    if name == "cfg3":
        wl = Workload(name, S["small"], [], seed_index=3)
        wl.n_frames = draw_lengths_uniform(16, 1.0, 10.0, wl.seeds["lengths"])
        return wl
    if name == "cfg4a":
        return Workload(name, S["medium"], [600] * 8, hush_frames=0, seed_index=4, pad_to_frames=3000)
    if name == "cfg4b":
        return Workload(name, S["medium"], [600] * 8, seed_index=4)
    if name == "cfg5":
        wl = Workload(name, S["large-v3"], [], seed_index=5)
        wl.n_frames = draw_lengths_loguniform(64, 1.0, 30.0, wl.seeds["lengths"])
        return wl
    # unit-sized workloads: odd lengths, a 1-frame stream, several tiles and a ragged tail
    if name == "unit":
        return Workload(name, S["unit"], [37, 1, 150, 64, 263], hush_frames=5, seed_index=7)
    if name == "unit-sharp":
        return Workload(name, S["unit"], [37, 1, 150, 64, 263], hush_frames=5, seed_index=7, q_scale=8.0)
    if name == "tiny-ragged":
        return Workload(name, S["tiny"], [100, 333, 41, 1, 702, 256], seed_index=8)
    if name == "tiny-sharp":
        return Workload(name, S["tiny"], [100, 333, 41, 1, 702, 256], seed_index=8, q_scale=8.0)
    if name == "stem-wide":
        # 36 long streams (odd and even lengths, one short, one single frame): ~53 k tokens
        return Workload(name, S["stem"], [2901 + 7 * (i % 5) for i in range(34)] + [77, 1], seed_index=9)
    raise KeyError(name)


WORKLOAD_NAMES = ["cfg1", "cfg2-2s", "cfg2-4s", "cfg2-8s", "cfg3", "cfg4a", "cfg4b", "cfg5"]


def materialize(wl: Workload, affine_random: bool = False):
    """Return (weights, hush, mels) for a workload.  mels[i] has wl.n_frames[i] rows, or
    pad_to_frames rows for the padded-window baseline."""
    weights = make_weights(wl.shape, wl.seeds["weights"], wl.q_scale)
    if affine_random:
        randomize_affine(weights, wl.seeds["weights"] + 5)
    hush = make_hush(wl.shape, wl.seeds["hush"], wl.hush_frames)
    mels = make_mels(wl.shape, wl.n_frames, wl.seeds["mel"], wl.pad_to_frames)
    return weights, hush, mels
