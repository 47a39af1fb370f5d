"""Pins for oracle/decoder_oracle.py against things other than itself: PyTorch's own
TransformerDecoderLayer, explicit scalar sums on tiny inputs, and the invariants the definition fixes
(causality, set-invariance over encoder tokens, degenerate lengths, bias-free keys)."""
import math

import numpy as np
import pytest
import torch

from oracle import decoder_oracle as D
from paper_2412_11272_amd import synth

UNIT = synth.DEC_SHAPES["unit"]


def _weights(seed=11, q_scale=1.0, shape=UNIT):
    return synth.make_decoder_weights(shape, seed, q_scale=q_scale, affine_random=True)


def _w64(w):
    return D._cast(w, np.float64)


def test_block_matches_torch_decoder_layer():
    """norm_first TransformerDecoderLayer with exact GELU is the same block (keys given a zero bias)."""
    w = _weights(q_scale=6.0)
    lw = _w64(w)["layers"][0]
    d, f, h = UNIT.d_model, UNIT.d_mlp, UNIT.n_heads
    rng = np.random.default_rng(5)
    x = rng.standard_normal((13, d))
    enc = rng.standard_normal((29, d))
    layer = torch.nn.TransformerDecoderLayer(d, h, f, dropout=0.0, activation=torch.nn.functional.gelu, batch_first=True,
                                             norm_first=True, dtype=torch.float64)
    T = lambda a: torch.from_numpy(np.ascontiguousarray(a))
    z = np.zeros(d)
    with torch.no_grad():
        layer.self_attn.in_proj_weight.copy_(T(np.concatenate([lw["wq"], lw["wk"], lw["wv"]])))
        layer.self_attn.in_proj_bias.copy_(T(np.concatenate([lw["bq"], z, lw["bv"]])))
        layer.self_attn.out_proj.weight.copy_(T(lw["wo"])); layer.self_attn.out_proj.bias.copy_(T(lw["bo"]))
        layer.multihead_attn.in_proj_weight.copy_(T(np.concatenate([lw["xwq"], lw["xwk"], lw["xwv"]])))
        layer.multihead_attn.in_proj_bias.copy_(T(np.concatenate([lw["xbq"], z, lw["xbv"]])))
        layer.multihead_attn.out_proj.weight.copy_(T(lw["xwo"])); layer.multihead_attn.out_proj.bias.copy_(T(lw["xbo"]))
        layer.linear1.weight.copy_(T(lw["w1"])); layer.linear1.bias.copy_(T(lw["b1"]))
        layer.linear2.weight.copy_(T(lw["w2"])); layer.linear2.bias.copy_(T(lw["b2"]))
        layer.norm1.weight.copy_(T(lw["ln1_g"])); layer.norm1.bias.copy_(T(lw["ln1_b"]))
        layer.norm2.weight.copy_(T(lw["lnx_g"])); layer.norm2.bias.copy_(T(lw["lnx_b"]))
        layer.norm3.weight.copy_(T(lw["ln2_g"])); layer.norm3.bias.copy_(T(lw["ln2_b"]))
        mask = torch.triu(torch.full((13, 13), float("-inf"), dtype=torch.float64), diagonal=1)
        ref = layer(T(x)[None], T(enc)[None], tgt_mask=mask)[0].numpy()
    got, _, _ = D.decoder_block(x, enc, lw, h)
    assert np.abs(got - ref).max() < 1e-11


def _brute_prefill(w, n_heads, tokens, enc):
    """The whole prefill as scalar sums over Python lists (one layer or more), no matrix products."""
    d = len(w["lnf_g"])
    dh = d // n_heads
    P, L = len(tokens), len(enc)

    def ln(rows, g, b):
        out = []
        for r in rows:
            mu = sum(r) / d
            var = sum((v - mu) ** 2 for v in r) / d
            out.append([(r[c] - mu) / math.sqrt(var + 1e-5) * g[c] + b[c] for c in range(d)])
        return out

    def lin(rows, W, b):
        return [[sum(r[i] * W[o][i] for i in range(len(r))) + (b[o] if b is not None else 0.0) for o in range(len(W))] for r in rows]

    def attend(q, k, v, causal):
        out = [[0.0] * d for _ in q]
        for eta in range(n_heads):
            lo = eta * dh
            for r in range(len(q)):
                keys = range(r + 1) if causal else range(len(k))
                s = [sum(q[r][lo + c] * k[j][lo + c] for c in range(dh)) / math.sqrt(dh) for j in keys]
                m = max(s)
                e = [math.exp(t - m) for t in s]
                z = sum(e)
                for c in range(dh):
                    out[r][lo + c] = sum(e[n] / z * v[j][lo + c] for n, j in enumerate(keys))
        return out

    def gelu(z):
        return 0.5 * z * (1.0 + math.erf(z / math.sqrt(2.0)))

    x = [[float(w["tok_emb"][tokens[t]][c] + w["pos_emb"][t][c]) for c in range(d)] for t in range(P)]
    encl = [[float(v) for v in r] for r in enc]
    for lw in w["layers"]:
        u = ln(x, lw["ln1_g"], lw["ln1_b"])
        o = attend(lin(u, lw["wq"], lw["bq"]), lin(u, lw["wk"], None), lin(u, lw["wv"], lw["bv"]), True)
        a = lin(o, lw["wo"], lw["bo"])
        x = [[x[t][c] + a[t][c] for c in range(d)] for t in range(P)]
        u = ln(x, lw["lnx_g"], lw["lnx_b"])
        o = attend(lin(u, lw["xwq"], lw["xbq"]), lin(encl, lw["xwk"], None), lin(encl, lw["xwv"], lw["xbv"]), False)
        a = lin(o, lw["xwo"], lw["xbo"])
        x = [[x[t][c] + a[t][c] for c in range(d)] for t in range(P)]
        u = ln(x, lw["ln2_g"], lw["ln2_b"])
        m = [[gelu(v) for v in r] for r in lin(u, lw["w1"], lw["b1"])]
        a = lin(m, lw["w2"], lw["b2"])
        x = [[x[t][c] + a[t][c] for c in range(d)] for t in range(P)]
    hid = ln(x, w["lnf_g"], w["lnf_b"])
    logits = [sum(hid[-1][c] * w["tok_emb"][j][c] for c in range(d)) for j in range(len(w["tok_emb"]))]
    return np.array(hid), np.array(logits)


def test_prefill_matches_scalar_sums():
    shape = synth.DecoderShape(8, 2, 2, 12, 9, 6)
    w = _w64(synth.make_decoder_weights(shape, 3, q_scale=20.0, affine_random=True))
    for lw in w["layers"]:            # make the block contributions comparable to the embeddings
        for k in ("wv", "wo", "xwv", "xwo", "w1", "w2"):
            lw[k] = lw[k] * 20.0
    w["tok_emb"] = w["tok_emb"] * 30.0
    w["pos_emb"] = w["pos_emb"] * 30.0
    rng = np.random.default_rng(9)
    enc = rng.standard_normal((4, 8))
    tokens = [7, 0, 3, 3, 8]
    r = D.prefill_stream(w, 2, tokens, enc)
    hid, logits = _brute_prefill(w, 2, tokens, enc)
    assert np.abs(r["hidden"] - hid).max() < 1e-11
    assert np.abs(r["logits"] - logits).max() < 1e-10
    assert len(r["self_k"]) == 2 and r["self_k"][0].shape == (5, 8)


def test_causality_and_full_dependence_on_encoder():
    w = _weights(q_scale=6.0)
    rng = np.random.default_rng(1)
    enc = rng.standard_normal((17, UNIT.d_model))
    tok = list(rng.integers(0, UNIT.n_vocab, size=12))
    a = D.prefill_stream(w, UNIT.n_heads, tok, enc)["hidden"]
    tok2 = list(tok)
    tok2[7] = (tok2[7] + 1) % UNIT.n_vocab
    b = D.prefill_stream(w, UNIT.n_heads, tok2, enc)["hidden"]
    assert np.array_equal(a[:7], b[:7])                       # earlier positions never see a later token
    assert all(np.abs(a[t] - b[t]).max() > 1e-6 for t in range(7, 12))
    enc2 = enc.copy()
    enc2[16] += 0.5                                           # any encoder token reaches every prompt position
    c = D.prefill_stream(w, UNIT.n_heads, tok, enc2)["hidden"]
    assert all(np.abs(a[t] - c[t]).max() > 1e-7 for t in range(12))


def test_encoder_tokens_are_a_set_for_cross_attention():
    w = _weights(q_scale=6.0)
    rng = np.random.default_rng(2)
    enc = rng.standard_normal((23, UNIT.d_model))
    tok = list(rng.integers(0, UNIT.n_vocab, size=9))
    a = D.prefill_stream(w, UNIT.n_heads, tok, enc)
    b = D.prefill_stream(w, UNIT.n_heads, tok, enc[rng.permutation(23)])
    assert np.abs(a["hidden"] - b["hidden"]).max() < 1e-12
    assert np.abs(a["logits"] - b["logits"]).max() < 1e-12


def test_single_key_and_single_query_cases():
    w = _w64(_weights(q_scale=6.0))
    lw = dict(w["layers"][0])
    rng = np.random.default_rng(3)
    x = rng.standard_normal((6, UNIT.d_model))
    enc1 = rng.standard_normal((1, UNIT.d_model))
    base, _, _ = D.decoder_block(x, enc1, lw, UNIT.n_heads)
    lw2 = dict(lw)
    lw2["xwq"] = lw["xwq"] * -3.0                              # one encoder token: its weight is 1 whatever the query
    alt, _, _ = D.decoder_block(x, enc1, lw2, UNIT.n_heads)
    assert np.abs(base - alt).max() < 1e-12
    x1 = x[:1]
    enc = rng.standard_normal((5, UNIT.d_model))
    base1, k1, v1 = D.decoder_block(x1, enc, lw, UNIT.n_heads)
    lw3 = dict(lw)
    lw3["wq"] = lw["wq"] * 2.0                                 # one prompt token: it attends to itself only
    alt1, _, _ = D.decoder_block(x1, enc, lw3, UNIT.n_heads)
    assert np.abs(base1 - alt1).max() < 1e-12
    # and the first row of a longer prompt equals the one-token result (causal mask)
    full, _, _ = D.decoder_block(x, enc, lw, UNIT.n_heads)
    assert np.abs(full[0] - base1[0]).max() < 1e-12


def test_uniform_weights_give_the_mean_of_visible_values():
    rng = np.random.default_rng(4)
    q = np.zeros((5, 8)); k = rng.standard_normal((5, 8)); v = rng.standard_normal((5, 8))
    o = D.multi_head(q, k, v, 2, causal=True)
    for r in range(5):
        assert np.allclose(o[r], v[:r + 1].mean(axis=0), atol=1e-13)
    o = D.multi_head(q[:2], k, v, 2, causal=False)
    assert np.allclose(o, np.tile(v.mean(axis=0), (2, 1)), atol=1e-13)


def test_cross_kv_is_tokenwise_and_keys_have_no_bias():
    w = _weights()
    rng = np.random.default_rng(6)
    enc = rng.standard_normal((11, UNIT.d_model))
    kv = D.cross_kv_batch(w, enc)
    assert kv.shape == (UNIT.n_layers, 11, 2 * UNIT.d_model)
    one = D.cross_kv_batch(w, enc[4:5])
    assert np.abs(kv[:, 4:5] - one).max() < 1e-13
    zero = D.cross_kv_batch(w, np.zeros((2, UNIT.d_model)))
    for l in range(UNIT.n_layers):
        assert np.all(zero[l][:, :UNIT.d_model] == 0.0)
        assert np.allclose(zero[l][:, UNIT.d_model:], w["layers"][l]["xbv"])
    # explicit sum for one element: K[l=1, token 3, feature 5] and V[...]
    lw = w["layers"][1]
    kk = sum(float(enc[3, i]) * float(lw["xwk"][5, i]) for i in range(UNIT.d_model))
    vv = sum(float(enc[3, i]) * float(lw["xwv"][5, i]) for i in range(UNIT.d_model)) + float(lw["xbv"][5])
    assert abs(kv[1, 3, 5] - kk) < 1e-12 and abs(kv[1, 3, UNIT.d_model + 5] - vv) < 1e-12


def test_batch_is_per_stream():
    w = _weights()
    rng = np.random.default_rng(7)
    lens_enc, lens_p = [5, 1, 12], [4, 9, 1]
    enc = rng.standard_normal((sum(lens_enc), UNIT.d_model))
    cu = np.concatenate([[0], np.cumsum(lens_enc)])
    prompts = synth.make_prompts(lens_p, UNIT.n_vocab, 8)
    hid, logits, cup = D.prefill_batch(w, UNIT.n_heads, prompts, enc, cu)
    assert list(cup) == [0, 4, 13, 14] and logits.shape == (3, UNIT.n_vocab)
    for i in range(3):
        r = D.prefill_stream(w, UNIT.n_heads, prompts[i], enc[cu[i]:cu[i + 1]])
        assert np.array_equal(hid[cup[i]:cup[i + 1]], r["hidden"])
        assert np.array_equal(logits[i], r["logits"])
