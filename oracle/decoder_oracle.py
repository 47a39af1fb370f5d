"""CPU oracle for the decoder-side consumers of the encoder states.  TEST INFRASTRUCTURE ONLY.

Plain NumPy fp64 definition of the two dense steps that follow the encoder in a processing round
(paper Section "Operations", workload mapping: prompt prefilling is always mapped to the GPU;
Section "CPU/GPU pipelining", categorization of workloads, item (2): about 100 prompt tokens go
through the decoder in one parallel pass):

  * cross_kv: every decoder layer projects the encoder states of a stream once into the keys and
    values its cross-attention reads for the rest of the round;
  * prefill: the prompt tokens of a stream run through the decoder stack in one pass (causal
    self-attention among the prompt tokens, cross-attention over that stream's encoder states),
    giving the hidden states, the per-layer self-attention keys/values (what token-by-token
    decoding continues from) and the logits of the last prompt position.

The paper does not spell out the decoder's internals; the definition below is the standard
pre-LN encoder-decoder transformer that goes with the Whisper-style encoder of
encoder_oracle.py, with these readings: token embedding plus a learned position table; per
block: LayerNorm -> causal self-attention -> residual, LayerNorm -> cross-attention -> residual,
LayerNorm -> GELU MLP -> residual; final LayerNorm; logits against the token embedding matrix
(tied); key projections carry no bias; softmax scale 1/sqrt(head size).

Slow on purpose; only the tests, the smoke check and the benchmark's CPU-baseline leg import it.
Shares no code with the HIP path.  Pins: tests/test_decoder_oracle_pins.py (PyTorch's own
TransformerDecoderLayer, brute-force sums, causality, set-invariance over encoder tokens,
degenerate lengths).
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from .encoder_oracle import _cast, gelu, layer_norm, linear


def masked_attention_weights(q: np.ndarray, k: np.ndarray, causal: bool) -> np.ndarray:
    """A[r, :] = softmax over the allowed keys of q_r . k / sqrt(d_head); with causal=True query r
    (position r of the same sequence as the keys) sees keys 0..r only."""
    s = (q @ k.T) / math.sqrt(q.shape[1])
    if causal:
        r = np.arange(q.shape[0])[:, None]
        c = np.arange(k.shape[0])[None, :]
        s = np.where(c <= r, s, -np.inf)
    s = s - s.max(axis=1, keepdims=True)
    e = np.exp(s)
    return e / e.sum(axis=1, keepdims=True)


def multi_head(q: np.ndarray, k: np.ndarray, v: np.ndarray, n_heads: int, causal: bool) -> np.ndarray:
    """Head eta owns columns [eta*d_head, (eta+1)*d_head) of q, k, v and of the result."""
    d = q.shape[1]
    dh = d // n_heads
    o = np.empty((q.shape[0], d), dtype=q.dtype)
    for eta in range(n_heads):
        c = slice(eta * dh, (eta + 1) * dh)
        o[:, c] = masked_attention_weights(q[:, c], k[:, c], causal) @ v[:, c]
    return o


def cross_kv(lw: dict, enc: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Keys and values one decoder layer's cross-attention reads: K = enc Wk^T, V = enc Wv^T + bv."""
    return linear(enc, lw["xwk"], None), linear(enc, lw["xwv"], lw["xbv"])


def decoder_block(x: np.ndarray, enc: np.ndarray, lw: dict, n_heads: int):
    """One pre-LN decoder block on one stream: x [P, d] prompt states, enc [L, d] encoder states.
    Returns (x_out, self_k, self_v)."""
    u = layer_norm(x, lw["ln1_g"], lw["ln1_b"])
    q = linear(u, lw["wq"], lw["bq"])
    k = linear(u, lw["wk"], None)
    v = linear(u, lw["wv"], lw["bv"])
    x = x + linear(multi_head(q, k, v, n_heads, causal=True), lw["wo"], lw["bo"])
    u = layer_norm(x, lw["lnx_g"], lw["lnx_b"])
    xq = linear(u, lw["xwq"], lw["xbq"])
    xk, xv = cross_kv(lw, enc)
    x = x + linear(multi_head(xq, xk, xv, n_heads, causal=False), lw["xwo"], lw["xbo"])
    u = layer_norm(x, lw["ln2_g"], lw["ln2_b"])
    x = x + linear(gelu(linear(u, lw["w1"], lw["b1"])), lw["w2"], lw["b2"])
    return x, k, v


def prefill_stream(weights: dict, n_heads: int, tokens: Sequence[int], enc: np.ndarray, dtype=np.float64,
                   _cast_weights: bool = True) -> Dict[str, object]:
    """Prompt prefill for one stream.

    tokens: P >= 1 token ids; enc [L, d] that stream's encoder states.
    Returns hidden [P, d] (after the final LayerNorm), logits [n_vocab] of the last position,
    self_k / self_v: per-layer [P, d]."""
    w = _cast(weights, dtype) if _cast_weights else weights
    tok = np.asarray(tokens, dtype=np.int64)
    enc = np.asarray(enc, dtype=dtype)
    x = w["tok_emb"][tok] + w["pos_emb"][:len(tok)]
    ks: List[np.ndarray] = []
    vs: List[np.ndarray] = []
    for lw in w["layers"]:
        x, k, v = decoder_block(x, enc, lw, n_heads)
        ks.append(k)
        vs.append(v)
    hidden = layer_norm(x, w["lnf_g"], w["lnf_b"])
    logits = hidden[-1] @ w["tok_emb"].T
    return {"hidden": hidden, "logits": logits, "self_k": ks, "self_v": vs}


def prefill_batch(weights: dict, n_heads: int, prompts: Sequence[Sequence[int]], enc_packed: np.ndarray,
                  cu_seqlens: Sequence[int], dtype=np.float64):
    """Every stream on its own.  Returns (hidden [sum P, d] stream-major, logits [B, n_vocab], cu_prompt [B+1])."""
    w = _cast(weights, dtype)
    hs, lg = [], []
    for i, p in enumerate(prompts):
        r = prefill_stream(w, n_heads, p, enc_packed[cu_seqlens[i]:cu_seqlens[i + 1]], dtype, _cast_weights=False)
        hs.append(r["hidden"])
        lg.append(r["logits"])
    cu = np.zeros(len(prompts) + 1, dtype=np.int64)
    cu[1:] = np.cumsum([len(p) for p in prompts])
    return np.concatenate(hs, axis=0), np.stack(lg, axis=0), cu


def cross_kv_batch(weights: dict, enc_packed: np.ndarray, dtype=np.float64) -> np.ndarray:
    """[n_layers, M, 2 d]: keys in the first d columns, values in the last d (token-wise, so the packed
    batch is projected as it stands)."""
    w = _cast(weights, dtype)
    enc = np.asarray(enc_packed, dtype=dtype)
    out = []
    for lw in w["layers"]:
        k, v = cross_kv(lw, enc)
        out.append(np.concatenate([k, v], axis=1))
    return np.stack(out, axis=0)
