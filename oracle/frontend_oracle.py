"""CPU oracle for the log-mel front end with the hush word appended at the raw-audio level.
TEST INFRASTRUCTURE ONLY (same rules as encoder_oracle.py: never imported by the product path).

What it follows:
  * Raw audio is a one-dimensional array sampled at 16 kHz; one second of it becomes a (100, 80)
    log-mel matrix (paper Section "Hush word", hush word target level) -- hence a hop of 160 samples.
  * The hush word is a fixed raw-audio vector of 8000 samples = 0.5 s (Section "Key Implementation
    Details", hush word training) placed at the END of the audio, x (+) h, before the spectrogram
    is computed (Section "Hush word", position and target level).
  * The paper fixes nothing else about the front end.  The readings used here (listed in the design
    notes): periodic Hann window of 400 samples (25 ms), frames centred on multiples of 160 samples
    with reflect padding of 200 samples, 400-point DFT (201 bins), power spectrum, n_mels unit-peak
    triangular filters equally spaced on the mel scale m(f) = 2595 log10(1 + f/700) between 0 and
    8000 Hz, log10 with a floor of 1e-10, values clamped to within 8 decades of the stream's
    maximum, then (v + 4) / 4.

The result has a plain definition, so the oracle is that definition: the DFT is the explicit sum
against cos/sin tables (a matrix product), in fp64.
"""
from __future__ import annotations

import math
from typing import Optional, Sequence, Tuple

import numpy as np

SAMPLE_RATE = 16000
HOP = 160
N_FFT = 400
N_BINS = N_FFT // 2 + 1
LOG_FLOOR = 1e-10
DYNAMIC_RANGE_DECADES = 8.0


def n_frames(n_samples: int) -> int:
    """Frames of a signal of n_samples: one per hop, floor(n / 160).  16000 samples -> 100 frames."""
    return n_samples // HOP


def hann_window() -> np.ndarray:
    n = np.arange(N_FFT, dtype=np.float64)
    return 0.5 - 0.5 * np.cos(2.0 * math.pi * n / N_FFT)


def hz_to_mel(f):
    return 2595.0 * np.log10(1.0 + np.asarray(f, dtype=np.float64) / 700.0)


def mel_to_hz(m):
    return 700.0 * (10.0 ** (np.asarray(m, dtype=np.float64) / 2595.0) - 1.0)


def mel_filterbank(n_mels: int) -> np.ndarray:
    """[n_mels, 201]: filter k rises linearly (in Hz) from centre k-1 to centre k and falls to centre
    k+1, peak 1; the n_mels + 2 edge/centre frequencies are equally spaced in mel on [0, 8000] Hz."""
    edges = mel_to_hz(np.linspace(hz_to_mel(0.0), hz_to_mel(SAMPLE_RATE / 2.0), n_mels + 2))
    freqs = np.arange(N_BINS, dtype=np.float64) * SAMPLE_RATE / N_FFT
    fb = np.zeros((n_mels, N_BINS), dtype=np.float64)
    for k in range(n_mels):
        lo, ce, hi = edges[k], edges[k + 1], edges[k + 2]
        up = (freqs - lo) / (ce - lo)
        down = (hi - freqs) / (hi - ce)
        fb[k] = np.maximum(0.0, np.minimum(up, down))
    return fb


def reflect_pad(x: np.ndarray, pad: int) -> np.ndarray:
    """x[-k] = x[k], x[N-1+k] = x[N-1-k] for k = 1..pad (the end samples are not repeated)."""
    n = len(x)
    assert n > pad, "signal shorter than the padding"
    left = x[1:pad + 1][::-1]
    right = x[n - pad - 1:n - 1][::-1]
    return np.concatenate([left, x, right])


def power_spectrogram(x: np.ndarray) -> np.ndarray:
    """[T, 201] with P[t, f] = |sum_n w[n] xp[160 t + n] exp(-2 pi i f n / 400)|^2, xp the reflect-padded
    signal, T = floor(N / 160)."""
    x = np.asarray(x, dtype=np.float64)
    T = n_frames(len(x))
    xp = reflect_pad(x, N_FFT // 2)
    w = hann_window()
    frames = np.stack([xp[HOP * t:HOP * t + N_FFT] * w for t in range(T)]) if T > 0 else np.zeros((0, N_FFT))
    n = np.arange(N_FFT, dtype=np.float64)
    f = np.arange(N_BINS, dtype=np.float64)
    ang = 2.0 * math.pi * np.outer(n, f) / N_FFT                 # [400, 201]
    re = frames @ np.cos(ang)
    im = -(frames @ np.sin(ang))
    return re * re + im * im


def log_mel(x: np.ndarray, hush: Optional[np.ndarray], n_mels: int) -> np.ndarray:
    """Log-mel matrix [T', n_mels] of x (+) h."""
    x = np.asarray(x, dtype=np.float64)
    if hush is not None and len(hush) > 0:
        x = np.concatenate([x, np.asarray(hush, dtype=np.float64)])      # appended at the raw-audio level
    mel = power_spectrogram(x) @ mel_filterbank(n_mels).T
    v = np.log10(np.maximum(mel, LOG_FLOOR))
    v = np.maximum(v, v.max() - DYNAMIC_RANGE_DECADES)
    return (v + 4.0) / 4.0


def log_mel_batch(audios: Sequence[np.ndarray], hush: Optional[np.ndarray], n_mels: int) -> Tuple[np.ndarray, np.ndarray]:
    """Every stream on its own, stacked without padding.  Returns (mel [sum T', n_mels], cu_frames [B+1])."""
    outs = [log_mel(a, hush, n_mels) for a in audios]
    cu = np.zeros(len(outs) + 1, dtype=np.int64)
    cu[1:] = np.cumsum([o.shape[0] for o in outs])
    return (np.concatenate(outs, axis=0) if outs else np.zeros((0, n_mels))), cu
