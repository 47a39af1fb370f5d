"""CPU oracle for the ragged Whisper-style audio encoder.  TEST INFRASTRUCTURE ONLY.

This file is the plain definition of what the encoder computes, written out step by step with
NumPy in fp64 (fp32 on request).  It exists so the HIP path can be checked against something that
is obviously correct; it is slow on purpose and is never part of the product path.  Only the tests,
the smoke check and the benchmark's CPU-baseline leg may import it.  It shares no code with the
HIP path and imports nothing from it.

What it follows:
  * The encoder is the dense, always-on-GPU stage of a processing round (paper Section
    "Operations", workload mapping; Section "CPU/GPU pipelining", categorization of workloads):
    30 s of audio is 1500 tokens that pass through a stack of transformer blocks (Section "Why
    SSP is challenging").
  * Instead of padding to 30 s, one fixed short segment h is appended to each input x: the
    encoder sees x (+) h (Section "Hush word", hush word position).  One hush word per model
    (Section "Operations", offline development).  Here h lives at the log-mel level, 1 s of
    audio being a (100, 80) matrix (Section "Hush word", target level).
  * Inputs of different lengths are not padded to a common length (Section "Hush word", offline
    training details; Section "Applicability"): every stream is encoded at its own length.
  * The paper does not spell out the blocks' internals; the layer-by-layer definition (two
    width-3 Conv1d + GELU, the second with stride 2; sinusoidal positions; pre-LN blocks with
    multi-head bidirectional attention and a GELU MLP; final LayerNorm) is the standard
    Whisper-style encoder the benchmark spec names, with the readings listed in the design notes.

Every result here has a plain definition and the method reaches it exactly (ragged packing,
conv-as-GEMM, online softmax and fusion are exact re-arrangements), so the oracle is that
definition.  Library primitives used as steps: matrix product (@), exp, erf, sin, cos, sqrt.

Pins: tests/test_oracle_*.py (brute-force sums on tiny inputs, closed forms, invariants, and a
composition of PyTorch-CPU library routines).
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence, Tuple

import numpy as np
from scipy.special import erf as _erf

LN_EPS = 1e-5


def stem_length(n_frames: int) -> int:
    """Tokens produced from n_frames mel frames: width-3, pad-1 convs, the second with stride 2,
    give floor((n + 2 - 3)/2) + 1 = floor((n + 1)/2).  30 s = 3000 frames -> 1500 tokens and
    0.5 s = 50 frames -> 25 tokens, as in the paper (Sections "Why SSP is challenging" and "Our key
    ideas")."""
    return (n_frames + 1) // 2


def gelu(z: np.ndarray) -> np.ndarray:
    """Exact GELU: z * Phi(z) = z/2 * (1 + erf(z / sqrt 2))."""
    return 0.5 * z * (1.0 + _erf(z / math.sqrt(2.0)))


def conv1d_k3(x: np.ndarray, w: np.ndarray, b: np.ndarray, stride: int) -> np.ndarray:
    """Width-3 convolution over time with one zero frame of padding on each side.

    x [T, C_in] time-major, w [C_out, C_in, 3], b [C_out]  ->  [T_out, C_out] with
    out[t, c] = b[c] + sum_k sum_m w[c, m, k] * x[stride*t + k - 1, m],  rows outside [0, T) being 0,
    for t in [0, T_out), T_out = floor((T + 2 - 3)/stride) + 1.
    """
    T, c_in = x.shape
    t_out = (T + 2 - 3) // stride + 1
    xp = np.zeros((T + 2, c_in), dtype=x.dtype)
    xp[1:T + 1] = x
    out = np.broadcast_to(b, (t_out, w.shape[0])).astype(x.dtype).copy()
    for k in range(3):
        rows = xp[k:k + stride * (t_out - 1) + 1:stride]      # rows stride*t + k of the padded input
        out += rows @ np.ascontiguousarray(w[:, :, k]).T       # tap k as a [C_in, C_out] matrix product
    return out


def sinusoid_table(n_pos: int, d: int, dtype=np.float64) -> np.ndarray:
    """Sinusoidal positions P [n_pos, d]: P[j, c] = sin(j w_c), P[j, d/2 + c] = cos(j w_c) with
    w_c = 10000^(-c / (d/2 - 1)), c in [0, d/2): geometric from 1 down to 1/10000."""
    half = d // 2
    c = np.arange(half, dtype=np.float64)
    omega = np.exp(-math.log(10000.0) * c / (half - 1))
    ang = np.arange(n_pos, dtype=np.float64)[:, None] * omega[None, :]
    return np.concatenate([np.sin(ang), np.cos(ang)], axis=1).astype(dtype)


def layer_norm(x: np.ndarray, g: np.ndarray, b: np.ndarray, eps: float = LN_EPS) -> np.ndarray:
    """Row-wise LayerNorm with the biased variance: (x - mean) / sqrt(var + eps) * g + b."""
    mu = x.mean(axis=1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * g + b


def linear(x: np.ndarray, w: np.ndarray, b: Optional[np.ndarray]) -> np.ndarray:
    """y = x w^T (+ b), w stored [out, in]."""
    y = x @ w.T
    if b is not None:
        y = y + b
    return y


def attention_weights(q: np.ndarray, k: np.ndarray) -> np.ndarray:
    """Softmax over all keys of one stream, one head: A[r, :] = softmax(q_r . k / sqrt(d_head)).
    Bidirectional: no mask inside a stream."""
    s = (q @ k.T) / math.sqrt(q.shape[1])
    s = s - s.max(axis=1, keepdims=True)
    e = np.exp(s)
    return e / e.sum(axis=1, keepdims=True)


def multi_head_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, n_heads: int) -> np.ndarray:
    """Head eta owns columns [eta*d_head, (eta+1)*d_head) of q, k, v and of the result."""
    L, d = q.shape
    dh = d // n_heads
    o = np.empty_like(q)
    for eta in range(n_heads):
        c = slice(eta * dh, (eta + 1) * dh)
        o[:, c] = attention_weights(q[:, c], k[:, c]) @ v[:, c]
    return o


def encoder_block(x: np.ndarray, lw: dict, n_heads: int) -> np.ndarray:
    """One pre-LN transformer block on one stream's tokens x [L, d]."""
    u = layer_norm(x, lw["ln1_g"], lw["ln1_b"])
    q = linear(u, lw["wq"], lw["bq"])
    k = linear(u, lw["wk"], lw.get("bk"))
    v = linear(u, lw["wv"], lw["bv"])
    x = x + linear(multi_head_attention(q, k, v, n_heads), lw["wo"], lw["bo"])
    u = layer_norm(x, lw["ln2_g"], lw["ln2_b"])
    x = x + linear(gelu(linear(u, lw["w1"], lw["b1"])), lw["w2"], lw["b2"])
    return x


def stem(frames: np.ndarray, w: dict) -> np.ndarray:
    """Conv stem + positions on one stream's frames [T', n_mels] -> [floor((T'+1)/2), d]."""
    g = gelu(conv1d_k3(frames, w["conv1_w"], w["conv1_b"], stride=1))
    y = gelu(conv1d_k3(g, w["conv2_w"], w["conv2_b"], stride=2))
    return y + sinusoid_table(y.shape[0], y.shape[1], dtype=y.dtype)


def _cast(tree, dtype):
    if tree is None:
        return None
    if isinstance(tree, dict):
        return {k: _cast(v, dtype) for k, v in tree.items()}
    if isinstance(tree, (list, tuple)):
        return [_cast(v, dtype) for v in tree]
    return np.asarray(tree, dtype=dtype)


def encode_stream(weights: dict, n_heads: int, mel: np.ndarray, hush: Optional[np.ndarray],
                  dtype=np.float64, _cast_weights: bool = True) -> np.ndarray:
    """Encoder states [L, d] for one stream: x (+) h, then stem, blocks, final LayerNorm."""
    w = _cast(weights, dtype) if _cast_weights else weights
    frames = np.asarray(mel, dtype=dtype)
    if hush is not None and len(hush) > 0:
        frames = np.concatenate([frames, np.asarray(hush, dtype=dtype)], axis=0)   # append, not prepend
    x = stem(frames, w)
    for lw in w["layers"]:
        x = encoder_block(x, lw, n_heads)
    return layer_norm(x, w["lnf_g"], w["lnf_b"])


def encode_batch(weights: dict, n_heads: int, mels: Sequence[np.ndarray], hush: Optional[np.ndarray],
                 dtype=np.float64) -> Tuple[np.ndarray, np.ndarray]:
    """Every stream on its own, results stacked stream-major without padding.

    Returns (out [M, d], cu_seqlens [B+1]) with stream i at rows [cu_seqlens[i], cu_seqlens[i+1])."""
    w = _cast(weights, dtype)
    outs: List[np.ndarray] = [encode_stream(w, n_heads, m, hush, dtype, _cast_weights=False) for m in mels]
    cu = np.zeros(len(mels) + 1, dtype=np.int64)
    cu[1:] = np.cumsum([o.shape[0] for o in outs])
    d = w["lnf_g"].shape[0]
    packed = np.concatenate(outs, axis=0) if outs else np.zeros((0, d), dtype=dtype)
    return packed, cu
