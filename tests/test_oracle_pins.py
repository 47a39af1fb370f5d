"""Pins for the CPU oracle: each test fixes a part of oracle/encoder_oracle.py to something other
than itself -- explicit sums on tiny inputs, closed forms, invariants, the shape facts the paper
prints (tests/golden/shape_facts.txt), or PyTorch-CPU library routines."""
import math
import os

import numpy as np
import pytest
import torch

from oracle import encoder_oracle as O
from paper_2412_11272_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
RNG = np.random.default_rng(12345)


# ------------------------------------------------------------------ stem length
def test_stem_length_matches_paper_shape_facts():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "shape_facts.txt")) if l.strip() and not l.startswith("#")]
    assert len(rows) >= 4
    for seconds, frames, tokens in rows:
        assert int(round(float(seconds) * synth.FRAMES_PER_SECOND)) == int(frames)
        assert O.stem_length(int(frames)) == int(tokens)


@pytest.mark.parametrize("frames,tokens", [(150, 75), (250, 125), (450, 225), (850, 425), (650, 325),
                                           (3000, 1500), (3050, 1525), (1, 1), (2, 1), (3, 2)])
def test_stem_length_closed_form_and_actual_conv_output(frames, tokens):
    assert O.stem_length(frames) == tokens
    x = RNG.standard_normal((frames, 2))
    w = RNG.standard_normal((3, 2, 3))
    assert O.conv1d_k3(x, w, np.zeros(3), 2).shape == (tokens, 3)
    assert O.conv1d_k3(x, w, np.zeros(3), 1).shape == (frames, 3)


# ------------------------------------------------------------------ convolution
def _conv_brute(x, w, b, stride):
    T, cin = x.shape
    cout = w.shape[0]
    t_out = (T - 1) // stride + 1
    out = [[0.0] * cout for _ in range(t_out)]
    for t in range(t_out):
        for c in range(cout):
            acc = float(b[c])
            for k in range(3):
                src = stride * t + k - 1
                if 0 <= src < T:
                    for m in range(cin):
                        acc += float(w[c, m, k]) * float(x[src, m])
            out[t][c] = acc
    return np.array(out)


@pytest.mark.parametrize("T", [1, 2, 3, 4, 6, 7])
@pytest.mark.parametrize("stride", [1, 2])
def test_conv_brute_force_tiny(T, stride):
    x = RNG.standard_normal((T, 3))
    w = RNG.standard_normal((2, 3, 3))
    b = RNG.standard_normal(2)
    np.testing.assert_allclose(O.conv1d_k3(x, w, b, stride), _conv_brute(x, w, b, stride), rtol=0, atol=1e-13)


def test_conv_all_ones_kernel_is_moving_sum():
    T = 9
    x = RNG.standard_normal((T, 4))
    w = np.ones((1, 4, 3))
    y = O.conv1d_k3(x, w, np.zeros(1), 1)[:, 0]
    rs = x.sum(axis=1)
    assert y[0] == pytest.approx(rs[0] + rs[1])
    assert y[T - 1] == pytest.approx(rs[T - 2] + rs[T - 1])
    for t in range(1, T - 1):
        assert y[t] == pytest.approx(rs[t - 1] + rs[t] + rs[t + 1])
    y2 = O.conv1d_k3(x, w, np.zeros(1), 2)[:, 0]
    np.testing.assert_allclose(y2, y[::2], atol=1e-13)


def test_conv_tap_order_is_not_reversed():
    # a kernel that only has the k=0 tap copies the PREVIOUS frame (t-1), k=2 the NEXT one
    x = RNG.standard_normal((5, 1))
    w = np.zeros((1, 1, 3)); w[0, 0, 0] = 1.0
    y = O.conv1d_k3(x, w, np.zeros(1), 1)[:, 0]
    np.testing.assert_allclose(y, np.concatenate([[0.0], x[:-1, 0]]))
    w = np.zeros((1, 1, 3)); w[0, 0, 2] = 1.0
    y = O.conv1d_k3(x, w, np.zeros(1), 1)[:, 0]
    np.testing.assert_allclose(y, np.concatenate([x[1:, 0], [0.0]]))


@pytest.mark.parametrize("T,stride", [(11, 1), (11, 2), (12, 2), (1, 2)])
def test_conv_matches_torch_conv1d(T, stride):
    x = RNG.standard_normal((T, 5)); w = RNG.standard_normal((7, 5, 3)); b = RNG.standard_normal(7)
    ref = torch.nn.functional.conv1d(torch.from_numpy(x.T[None]), torch.from_numpy(w), torch.from_numpy(b),
                                     stride=stride, padding=1)[0].T.numpy()
    np.testing.assert_allclose(O.conv1d_k3(x, w, b, stride), ref, atol=1e-12)


# ------------------------------------------------------------------ GELU
def test_gelu_closed_forms():
    z = np.array([0.0, 1.0, -1.0, 6.0, 8.0, -8.0, 0.3, -0.3])
    g = O.gelu(z)
    assert g[0] == 0.0
    assert g[1] == pytest.approx(0.5 * (1 + math.erf(1 / math.sqrt(2))), abs=1e-15)
    assert g[1] == pytest.approx(0.8413447460685429, abs=1e-12)   # Phi(1)
    np.testing.assert_allclose(O.gelu(z) - O.gelu(-z), z, atol=1e-15)   # z Phi(z) - (-z) Phi(-z) = z
    assert g[3] == pytest.approx(6.0, abs=1e-8) and g[4] == pytest.approx(8.0, abs=1e-14)
    assert abs(g[5]) < 1e-14
    # not the tanh approximation: they differ by > 1e-4 near |z| ~ 2.5
    zt = 2.5
    tanh_form = 0.5 * zt * (1 + math.tanh(math.sqrt(2 / math.pi) * (zt + 0.044715 * zt ** 3)))
    assert abs(O.gelu(np.array([zt]))[0] - tanh_form) > 1e-4
    ref = torch.nn.functional.gelu(torch.from_numpy(z)).numpy()
    np.testing.assert_allclose(g, ref, atol=1e-14)


# ------------------------------------------------------------------ positions
def test_sinusoid_table_properties():
    d = 12
    P = O.sinusoid_table(40, d)
    half = d // 2
    assert np.all(P[0, :half] == 0.0) and np.all(P[0, half:] == 1.0)
    np.testing.assert_allclose(P[:, :half] ** 2 + P[:, half:] ** 2, 1.0, atol=1e-14)
    np.testing.assert_allclose(P[:, 0], np.sin(np.arange(40)), atol=1e-14)          # first frequency is 1
    np.testing.assert_allclose(P[:, half - 1], np.sin(np.arange(40) / 10000.0), atol=1e-12)   # last is 1/10000
    np.testing.assert_allclose(P[:, half], np.cos(np.arange(40)), atol=1e-14)
    # geometric progression of frequencies, explicit loop
    for j in (1, 7, 39):
        for c in range(half):
            w = 10000.0 ** (-c / (half - 1))
            assert P[j, c] == pytest.approx(math.sin(j * w), abs=1e-12)
            assert P[j, half + c] == pytest.approx(math.cos(j * w), abs=1e-12)


# ------------------------------------------------------------------ LayerNorm
def test_layer_norm_properties_and_torch():
    x = RNG.standard_normal((6, 16)) * 3 + 1.5
    g = RNG.standard_normal(16); b = RNG.standard_normal(16)
    y = O.layer_norm(x, np.ones(16), np.zeros(16))
    np.testing.assert_allclose(y.mean(axis=1), 0, atol=1e-14)
    var = x.var(axis=1)                                   # biased
    np.testing.assert_allclose(y.var(axis=1), var / (var + 1e-5), rtol=1e-12)
    const = np.full((2, 16), 3.25)
    np.testing.assert_allclose(O.layer_norm(const, g, b), np.broadcast_to(b, (2, 16)), atol=1e-12)
    ref = torch.nn.functional.layer_norm(torch.from_numpy(x), (16,), torch.from_numpy(g), torch.from_numpy(b), 1e-5)
    np.testing.assert_allclose(O.layer_norm(x, g, b), ref.numpy(), atol=1e-13)
    # explicit sums for one row
    r = x[2]; mu = sum(r) / 16; v = sum((t - mu) ** 2 for t in r) / 16
    np.testing.assert_allclose(O.layer_norm(x, g, b)[2], [(t - mu) / math.sqrt(v + 1e-5) * g[i] + b[i] for i, t in enumerate(r)],
                               atol=1e-13)


# ------------------------------------------------------------------ attention
def test_attention_rows_sum_to_one_and_brute_force():
    L, dh = 7, 4
    q = RNG.standard_normal((L, dh)) * 3; k = RNG.standard_normal((L, dh)) * 3
    A = O.attention_weights(q, k)
    np.testing.assert_allclose(A.sum(axis=1), 1.0, atol=1e-14)
    assert np.all(A > 0)
    for r in range(L):
        logits = [sum(q[r, c] * k[s, c] for c in range(dh)) / math.sqrt(dh) for s in range(L)]
        z = sum(math.exp(t) for t in logits)
        for s in range(L):
            assert A[r, s] == pytest.approx(math.exp(logits[s]) / z, rel=1e-12)


def test_attention_special_cases():
    d, h = 8, 2
    v = RNG.standard_normal((1, d))
    o = O.multi_head_attention(RNG.standard_normal((1, d)), RNG.standard_normal((1, d)), v, h)
    np.testing.assert_allclose(o, v, atol=1e-15)                        # one token attends to itself only
    L = 6
    v = RNG.standard_normal((L, d)); k = RNG.standard_normal((L, d))
    o = O.multi_head_attention(np.zeros((L, d)), k, v, h)               # q = 0: uniform weights
    np.testing.assert_allclose(o, np.broadcast_to(v.mean(axis=0), (L, d)), atol=1e-14)
    q = RNG.standard_normal((L, d))
    bk = RNG.standard_normal(d)
    np.testing.assert_allclose(O.multi_head_attention(q, k + bk, v, h), O.multi_head_attention(q, k, v, h), atol=1e-12)
    # large logits do not overflow
    o = O.multi_head_attention(q * 400, k * 400, v, h)
    assert np.all(np.isfinite(o))


def test_attention_heads_are_column_slices_and_matches_torch_sdpa():
    L, d, h = 9, 12, 3
    q, k, v = (RNG.standard_normal((L, d)) for _ in range(3))
    o = O.multi_head_attention(q, k, v, h)
    tq, tk, tv = (torch.from_numpy(a).reshape(L, h, d // h).permute(1, 0, 2) for a in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv).permute(1, 0, 2).reshape(L, d).numpy()
    np.testing.assert_allclose(o, ref, atol=1e-12)


def test_block_permutation_equivariance():
    wl = synth.workload("unit")
    w, _, _ = synth.materialize(wl, affine_random=True)
    w = O._cast(w, np.float64)
    x = RNG.standard_normal((11, wl.shape.d_model))
    perm = RNG.permutation(11)
    y = O.encoder_block(x, w["layers"][0], wl.shape.n_heads)
    yp = O.encoder_block(x[perm], w["layers"][0], wl.shape.n_heads)
    np.testing.assert_allclose(yp, y[perm], atol=1e-12)


# ------------------------------------------------------------------ whole block, brute force
def _block_brute(x, lw):
    """Single-head pre-LN block as explicit sums (pure Python floats)."""
    L, d = len(x), len(x[0])

    def ln(rows, g, b):
        out = []
        for r in rows:
            mu = sum(r) / d
            var = sum((t - mu) ** 2 for t in r) / d
            out.append([(r[c] - mu) / math.sqrt(var + 1e-5) * g[c] + b[c] for c in range(d)])
        return out

    def lin(rows, w, b):
        n_out = len(w)
        return [[sum(r[i] * w[o][i] for i in range(len(r))) + (b[o] if b is not None else 0.0)
                 for o in range(n_out)] for r in rows]

    def gelu(t):
        return 0.5 * t * (1 + math.erf(t / math.sqrt(2)))

    u = ln(x, lw["ln1_g"], lw["ln1_b"])
    q, k, v = lin(u, lw["wq"], lw["bq"]), lin(u, lw["wk"], lw["bk"]), lin(u, lw["wv"], lw["bv"])
    o = []
    for r in range(L):
        logit = [sum(q[r][c] * k[s][c] for c in range(d)) / math.sqrt(d) for s in range(L)]
        mx = max(logit)
        e = [math.exp(t - mx) for t in logit]
        z = sum(e)
        o.append([sum(e[s] / z * v[s][c] for s in range(L)) for c in range(d)])
    a = lin(o, lw["wo"], lw["bo"])
    x1 = [[x[r][c] + a[r][c] for c in range(d)] for r in range(L)]
    u = ln(x1, lw["ln2_g"], lw["ln2_b"])
    hdn = [[gelu(t) for t in row] for row in lin(u, lw["w1"], lw["b1"])]
    m = lin(hdn, lw["w2"], lw["b2"])
    return [[x1[r][c] + m[r][c] for c in range(d)] for r in range(L)]


@pytest.mark.parametrize("L,d", [(5, 8), (1, 4), (3, 6)])
def test_single_head_block_brute_force(L, d):
    f = 2 * d + 1
    r = np.random.default_rng(100 + L)
    lw = {"ln1_g": r.standard_normal(d), "ln1_b": r.standard_normal(d),
          "wq": r.standard_normal((d, d)), "bq": r.standard_normal(d),
          "wk": r.standard_normal((d, d)), "bk": r.standard_normal(d),
          "wv": r.standard_normal((d, d)), "bv": r.standard_normal(d),
          "wo": r.standard_normal((d, d)), "bo": r.standard_normal(d),
          "ln2_g": r.standard_normal(d), "ln2_b": r.standard_normal(d),
          "w1": r.standard_normal((f, d)), "b1": r.standard_normal(f),
          "w2": r.standard_normal((d, f)), "b2": r.standard_normal(d)}
    x = r.standard_normal((L, d))
    ref = np.array(_block_brute(x.tolist(), {k: v.tolist() for k, v in lw.items()}))
    np.testing.assert_allclose(O.encoder_block(x, lw, 1), ref, atol=1e-11)


def test_single_layer_single_head_encoder_brute_force():
    """Whole path (hush append, stem, positions, one block, final LN) against explicit sums."""
    d, m, T, H = 6, 3, 4, 3
    r = np.random.default_rng(77)
    lw = {"ln1_g": r.standard_normal(d), "ln1_b": r.standard_normal(d),
          "wq": r.standard_normal((d, d)), "bq": r.standard_normal(d),
          "wk": r.standard_normal((d, d)), "bk": None,
          "wv": r.standard_normal((d, d)), "bv": r.standard_normal(d),
          "wo": r.standard_normal((d, d)), "bo": r.standard_normal(d),
          "ln2_g": r.standard_normal(d), "ln2_b": r.standard_normal(d),
          "w1": r.standard_normal((2 * d, d)), "b1": r.standard_normal(2 * d),
          "w2": r.standard_normal((d, 2 * d)), "b2": r.standard_normal(d)}
    w = {"conv1_w": r.standard_normal((d, m, 3)), "conv1_b": r.standard_normal(d),
         "conv2_w": r.standard_normal((d, d, 3)), "conv2_b": r.standard_normal(d),
         "layers": [lw], "lnf_g": r.standard_normal(d), "lnf_b": r.standard_normal(d)}
    mel = r.standard_normal((T, m)); hush = r.standard_normal((H, m))
    out = O.encode_stream(w, 1, mel, hush)
    # explicit reference
    X = np.concatenate([mel, hush])                 # x (+) h: hush AFTER the payload
    g = _conv_brute(X, w["conv1_w"], w["conv1_b"], 1)
    g = np.vectorize(lambda t: 0.5 * t * (1 + math.erf(t / math.sqrt(2))))(g)
    y = _conv_brute(g, w["conv2_w"], w["conv2_b"], 2)
    y = np.vectorize(lambda t: 0.5 * t * (1 + math.erf(t / math.sqrt(2))))(y)
    L = (T + H + 1) // 2
    assert y.shape == (L, d)
    half = d // 2
    for j in range(L):
        for c in range(half):
            om = 10000.0 ** (-c / (half - 1))
            y[j, c] += math.sin(j * om)
            y[j, half + c] += math.cos(j * om)
    lwl = {k: (v.tolist() if v is not None else None) for k, v in lw.items()}
    xb = np.array(_block_brute(y.tolist(), lwl))
    mu = xb.mean(axis=1, keepdims=True); var = ((xb - mu) ** 2).mean(axis=1, keepdims=True)
    ref = (xb - mu) / np.sqrt(var + 1e-5) * w["lnf_g"] + w["lnf_b"]
    np.testing.assert_allclose(out, ref, atol=1e-11)


# ------------------------------------------------------------------ whole-encoder invariants
def _unit(affine=True, name="unit"):
    wl = synth.workload(name)
    w, hush, mels = synth.materialize(wl, affine_random=affine)
    return wl, w, hush, mels


def test_identity_blocks_reduce_to_ln_of_stem():
    wl, w, hush, mels = _unit()
    for lw in w["layers"]:
        for k in ("wo", "bo", "w2", "b2"):
            lw[k] = np.zeros_like(lw[k])
    out, cu = O.encode_batch(w, wl.shape.n_heads, mels, hush)
    w64 = O._cast(w, np.float64)
    for i, mel in enumerate(mels):
        frames = np.concatenate([mel, hush]).astype(np.float64)
        ref = O.layer_norm(O.stem(frames, w64), w64["lnf_g"], w64["lnf_b"])
        np.testing.assert_allclose(out[cu[i]:cu[i + 1]], ref, atol=1e-13)


def test_ragged_equals_per_stream_and_reordering():
    wl, w, hush, mels = _unit()
    out, cu = O.encode_batch(w, wl.shape.n_heads, mels, hush)
    lens = [O.stem_length(len(m) + len(hush)) for m in mels]
    assert cu.tolist() == np.concatenate([[0], np.cumsum(lens)]).tolist()
    for i, mel in enumerate(mels):
        alone = O.encode_stream(w, wl.shape.n_heads, mel, hush)
        assert np.array_equal(out[cu[i]:cu[i + 1]], alone)
    order = [3, 0, 4, 2, 1]
    out2, cu2 = O.encode_batch(w, wl.shape.n_heads, [mels[i] for i in order], hush)
    for pos, i in enumerate(order):
        assert np.array_equal(out2[cu2[pos]:cu2[pos + 1]], out[cu[i]:cu[i + 1]])


def test_hush_semantics():
    wl, w, hush, mels = _unit()
    h = wl.shape.n_heads
    out, cu = O.encode_batch(w, h, mels, hush)
    # library-appended hush == caller-appended hush with the append turned off
    pre = [np.concatenate([m, hush]) for m in mels]
    out_pre, cu_pre = O.encode_batch(w, h, pre, None)
    assert np.array_equal(cu, cu_pre) and np.array_equal(out, out_pre)
    # appended at the END, not the beginning
    front = O.encode_stream(w, h, np.concatenate([hush, mels[0]]), None)
    assert np.abs(front - out[cu[0]:cu[1]]).max() > 1e-3
    # a different hush changes every token of a stream (bidirectional attention)
    hush2 = hush.copy(); hush2[-1, 0] += 0.5
    out2, _ = O.encode_batch(w, h, mels, hush2)
    assert np.all(np.abs(out2 - out).max(axis=1) > 0)
    # ... and changing one stream's payload changes no other stream
    mels3 = [m.copy() for m in mels]; mels3[2][0, 0] += 0.5
    out3, _ = O.encode_batch(w, h, mels3, hush)
    for i in range(len(mels)):
        same = np.array_equal(out3[cu[i]:cu[i + 1]], out[cu[i]:cu[i + 1]])
        assert same == (i != 2)


def test_final_output_rows_are_normalised_with_unit_gain():
    wl, w, hush, mels = _unit(affine=False)
    out, _ = O.encode_batch(w, wl.shape.n_heads, mels, hush)
    np.testing.assert_allclose(out.mean(axis=1), 0, atol=1e-12)
    v = out.var(axis=1)
    assert np.all(v < 1.0) and np.all(v > 0.9)


def test_k_bias_invariance_whole_encoder():
    wl, w, hush, mels = _unit(affine=True)
    out, _ = O.encode_batch(w, wl.shape.n_heads, mels, hush)
    for lw in w["layers"]:
        lw["bk"] = None
    out2, _ = O.encode_batch(w, wl.shape.n_heads, mels, hush)
    np.testing.assert_allclose(out, out2, atol=1e-10)


def test_fp32_mode_close_to_fp64():
    wl, w, hush, mels = _unit()
    o64, _ = O.encode_batch(w, wl.shape.n_heads, mels, hush)
    o32, _ = O.encode_batch(w, wl.shape.n_heads, mels, hush, dtype=np.float32)
    assert o32.dtype == np.float32
    assert np.abs(o32 - o64).max() / np.abs(o64).max() < 2e-5


# ------------------------------------------------------------------ library composition
def _torch_encoder(w, n_heads, mel, hush):
    t = lambda a: torch.from_numpy(np.asarray(a, np.float64))
    F = torch.nn.functional
    x = torch.cat([t(mel), t(hush)], 0).T[None]                       # [1, n_mels, T']
    x = F.gelu(F.conv1d(x, t(w["conv1_w"]), t(w["conv1_b"]), padding=1))
    x = F.gelu(F.conv1d(x, t(w["conv2_w"]), t(w["conv2_b"]), stride=2, padding=1))
    x = x[0].T                                                         # [L, d]
    L, d = x.shape
    half = d // 2
    inc = math.log(10000.0) / (half - 1)
    ang = torch.arange(L, dtype=torch.float64)[:, None] * torch.exp(-inc * torch.arange(half, dtype=torch.float64))[None]
    x = x + torch.cat([ang.sin(), ang.cos()], 1)
    for lw in w["layers"]:
        u = F.layer_norm(x, (d,), t(lw["ln1_g"]), t(lw["ln1_b"]), 1e-5)
        q = F.linear(u, t(lw["wq"]), t(lw["bq"]))
        k = F.linear(u, t(lw["wk"]), None if lw["bk"] is None else t(lw["bk"]))
        v = F.linear(u, t(lw["wv"]), t(lw["bv"]))
        sh = lambda a: a.reshape(L, n_heads, d // n_heads).permute(1, 0, 2)
        o = F.scaled_dot_product_attention(sh(q), sh(k), sh(v)).permute(1, 0, 2).reshape(L, d)
        x = x + F.linear(o, t(lw["wo"]), t(lw["bo"]))
        u = F.layer_norm(x, (d,), t(lw["ln2_g"]), t(lw["ln2_b"]), 1e-5)
        x = x + F.linear(F.gelu(F.linear(u, t(lw["w1"]), t(lw["b1"]))), t(lw["w2"]), t(lw["b2"]))
    return F.layer_norm(x, (d,), t(w["lnf_g"]), t(w["lnf_b"]), 1e-5).numpy()


@pytest.mark.parametrize("name,affine", [("unit", True), ("unit-sharp", True), ("cfg1", False)])
def test_whole_encoder_matches_torch_library_composition(name, affine):
    wl, w, hush, mels = _unit(affine=affine, name=name)
    out, cu = O.encode_batch(w, wl.shape.n_heads, mels, hush)
    for i, mel in enumerate(mels):
        ref = _torch_encoder(w, wl.shape.n_heads, mel, hush)
        assert ref.shape == (cu[i + 1] - cu[i], wl.shape.d_model)
        np.testing.assert_allclose(out[cu[i]:cu[i + 1]], ref, atol=1e-9)


def test_sharp_workload_has_peaked_softmax():
    """The stress workload must really have logits far from uniform, else it pins nothing."""
    wl, w, hush, mels = _unit(name="unit-sharp")
    w64 = O._cast(w, np.float64)
    x = O.stem(np.concatenate([mels[4], hush]).astype(np.float64), w64)
    lw = w64["layers"][0]
    u = O.layer_norm(x, lw["ln1_g"], lw["ln1_b"])
    q = O.linear(u, lw["wq"], lw["bq"])[:, :64]; k = O.linear(u, lw["wk"], None)[:, :64]
    A = O.attention_weights(q, k)
    assert A.max(axis=1).mean() > 5.0 / A.shape[1]
