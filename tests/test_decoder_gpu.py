"""GPU parity of the decoder-side steps (cross-attention K/V projection, prompt prefill) against
oracle/decoder_oracle.py, through the C ABI.  Same bars as the encoder: max|err| / max|ref| <= 2e-2 on
the bf16 MFMA path, <= 1e-4 on the fp32 debug path."""
import numpy as np
import pytest

from oracle import decoder_oracle as D
from oracle import encoder_oracle as O
from paper_2412_11272_amd import binding as wf
from paper_2412_11272_amd import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu

PREC = [pytest.param(wf.WF_PRECISION_F32, id="f32"), pytest.param(wf.WF_PRECISION_BF16, id="bf16")]


def _tol(precision):
    return H.F32_TOL if precision == wf.WF_PRECISION_F32 else H.BF16_TOL


def _case(shape_name, enc_lens, prompt_lens, seed, q_scale=1.0):
    shape = synth.DEC_SHAPES[shape_name]
    w = synth.make_decoder_weights(shape, seed, q_scale=q_scale, affine_random=True)
    enc = synth.make_enc_states(sum(enc_lens), shape.d_model, seed + 1)
    prompts = synth.make_prompts(prompt_lens, shape.n_vocab, seed + 2)
    cu = np.concatenate([[0], np.cumsum(enc_lens)]).astype(np.int32)
    return shape, w, enc, prompts, cu


def _gpu(shape, w, enc, prompts, cu, precision, want_self_kv=True):
    import torch
    dec = wf.Decoder(shape, w, len(prompts), int(cu[-1]), sum(len(p) for p in prompts), precision)
    try:
        e = torch.from_numpy(enc).cuda().to(dec.act_dtype)
        kv = dec.cross_kv(e)
        r = dec.prefill(prompts, cu, kv, hidden_dtype=torch.float32, want_self_kv=want_self_kv)
        torch.cuda.synchronize()
        return (kv.float().cpu().numpy(), r["hidden"].cpu().numpy(), r["logits"].cpu().numpy(),
                r["self_kv"].float().cpu().numpy() if want_self_kv else None, r["cu_prompt"])
    finally:
        dec.close()


@pytest.mark.parametrize("precision", PREC)
def test_cross_kv_matches_oracle(precision):
    shape, w, enc, prompts, cu = _case("unit", [37, 1, 150, 64, 263], [1] * 5, 21)
    kv, _, _, _, _ = _gpu(shape, w, enc, prompts, cu, precision, want_self_kv=False)
    ref = D.cross_kv_batch(w, enc)
    assert kv.shape == ref.shape
    err = H.rel_err(kv, ref)
    print(f"\ncross_kv rel err {err:.3e}", flush=True)
    assert err <= _tol(precision)


@pytest.mark.parametrize("sharp", [False, True], ids=["plain", "sharp"])
@pytest.mark.parametrize("precision", PREC)
def test_prefill_matches_oracle_unit(precision, sharp):
    # "sharp" scales the query and key projections so the softmax is peaked (stress for the running-max
    # softmax and the causal mask).  At x8 the oracle itself, with only its activations and weights rounded to
    # bf16 at the points where the GPU path stores them, is 2.1e-2 away from its fp64 result on this 128-wide
    # model (0.7e-2 at x6; tests/test_bf16_storage_rounding.py computes both), so the bf16 case runs at x6 and the
    # fp32 case, whose bar is about indexing, at x8.
    q_scale = 1.0 if not sharp else (8.0 if precision == wf.WF_PRECISION_F32 else 6.0)
    # prompts: one token, a ragged tail, exactly one key tile, more than one query tile (130 > 128)
    shape, w, enc, prompts, cu = _case("unit", [37, 1, 150, 64, 263], [5, 1, 130, 64, 100], 23, q_scale)
    kv, hidden, logits, self_kv, cup = _gpu(shape, w, enc, prompts, cu, precision)
    ref_h, ref_l, ref_cup = D.prefill_batch(w, shape.n_heads, prompts, enc, cu)
    assert cup.tolist() == ref_cup.tolist()
    eh, el = H.rel_err(hidden, ref_h), H.rel_err(logits, ref_l)
    print(f"\nprefill unit q_scale={q_scale}: hidden {eh:.3e} logits {el:.3e}", flush=True)
    assert eh <= _tol(precision) and el <= _tol(precision)
    # per-layer self-attention keys/values of one stream
    i = 2
    r = D.prefill_stream(w, shape.n_heads, prompts[i], enc[cu[i]:cu[i + 1]])
    for l in range(shape.n_layers):
        ref_kv = np.concatenate([r["self_k"][l], r["self_v"][l]], axis=1)
        assert H.rel_err(self_kv[l, cup[i]:cup[i + 1]], ref_kv) <= _tol(precision)


@pytest.mark.parametrize("precision", PREC)
def test_prefill_matches_oracle_tiny_full_context(precision):
    """Real vocabulary size (not a multiple of the GEMM tile) and a prompt that fills the context:
    448 tokens = 4 query tiles x 7 key tiles of the causal kernel."""
    # query/key scale: x4 on the fp32 path; x3 on the bf16 path (at x4 bf16 storage rounding of the activations
    # alone, simulated on the oracle, already gives 2.1e-2 on this model; 0.75e-2 at x3: tests/test_bf16_storage_rounding.py)
    q_scale = 4.0 if precision == wf.WF_PRECISION_F32 else 3.0
    shape, w, enc, prompts, cu = _case("tiny", [75, 700, 20], [448, 100, 1], 29, q_scale=q_scale)
    _, hidden, logits, _, cup = _gpu(shape, w, enc, prompts, cu, precision, want_self_kv=False)
    ref_h, ref_l, _ = D.prefill_batch(w, shape.n_heads, prompts, enc, cu)
    eh, el = H.rel_err(hidden, ref_h), H.rel_err(logits, ref_l)
    print(f"\nprefill tiny: hidden {eh:.3e} logits {el:.3e}", flush=True)
    assert logits.shape == (3, shape.n_vocab)
    assert eh <= _tol(precision) and el <= _tol(precision)
    if precision == wf.WF_PRECISION_F32:          # the decision the logits feed: same best token
        assert np.array_equal(logits.argmax(axis=1), ref_l.argmax(axis=1))


def test_causality_and_stream_isolation_on_gpu():
    """Changing one prompt token changes nothing before it and nothing in other streams (bit-exact)."""
    import torch
    shape, w, enc, prompts, cu = _case("unit", [40, 90], [150, 33], 31, q_scale=6.0)
    dec = wf.Decoder(shape, w, 2, int(cu[-1]), 183, wf.WF_PRECISION_BF16)
    try:
        kv = dec.cross_kv(torch.from_numpy(enc).cuda().bfloat16())
        a = dec.prefill(prompts, cu, kv, hidden_dtype=torch.float32)["hidden"].clone()
        p2 = [prompts[0].copy(), prompts[1]]
        p2[0][140] = (p2[0][140] + 1) % shape.n_vocab
        b = dec.prefill(p2, cu, kv, hidden_dtype=torch.float32)["hidden"].clone()
        torch.cuda.synchronize()
        assert torch.equal(a[:140], b[:140])
        assert torch.equal(a[150:], b[150:])
        assert not torch.equal(a[140:150], b[140:150])
    finally:
        dec.close()


def test_encoder_to_prefill_end_to_end():
    """mel -> encoder -> cross K/V -> prefill, all on the GPU in bf16, against the fp64 oracle chain."""
    import torch
    wl, w, hush, mels = H.inputs("unit")
    ref_enc, cu = H.oracle_batch("unit")
    shape = synth.DEC_SHAPES["unit"]
    dw = synth.make_decoder_weights(shape, 41, q_scale=4.0, affine_random=True)
    prompts = synth.make_prompts([100, 3, 64, 17, 129], shape.n_vocab, 43)
    ref_h, ref_l, _ = D.prefill_batch(dw, shape.n_heads, prompts, ref_enc, cu)
    enc = wf.encoder_for_workload(wl, w, hush, wf.WF_PRECISION_BF16)
    dec = wf.Decoder(shape, dw, len(prompts), int(cu[-1]), sum(len(p) for p in prompts), wf.WF_PRECISION_BF16)
    try:
        flat, offs, nf = wf.pack_mels(mels)
        states, cu_gpu = enc.encode(torch.from_numpy(flat).cuda(), offs, nf, out_dtype=torch.bfloat16)
        assert cu_gpu.tolist() == cu.tolist()
        kv = dec.cross_kv(states)
        r = dec.prefill(prompts, cu_gpu, kv, hidden_dtype=torch.float32)
        torch.cuda.synchronize()
        eh, el = H.rel_err(r["hidden"].cpu().numpy(), ref_h), H.rel_err(r["logits"].cpu().numpy(), ref_l)
        print(f"\nend to end: hidden {eh:.3e} logits {el:.3e}", flush=True)
        assert eh <= H.BF16_TOL and el <= H.BF16_TOL
    finally:
        enc.close()
        dec.close()


def test_decoder_argument_errors_are_reported_before_any_launch():
    import torch
    shape, w, enc, prompts, cu = _case("unit", [10, 20], [4, 6], 37)
    dec = wf.Decoder(shape, w, 2, 30, 10, wf.WF_PRECISION_BF16)
    try:
        e = torch.from_numpy(enc).cuda().bfloat16()
        kv = dec.cross_kv(e)
        with pytest.raises(wf.WfError) as ei:                      # id outside the vocabulary
            dec.prefill([np.array([1, 2, 3, shape.n_vocab], np.int32), prompts[1]], cu, kv)
        assert ei.value.code == wf.WF_E_INVALID_ARG
        with pytest.raises(wf.WfError) as ei:                      # more prompt tokens than the capacity
            dec.prefill([prompts[0], np.zeros(7, np.int32)], cu, kv)
        assert ei.value.code == wf.WF_E_CAPACITY
        with pytest.raises(wf.WfError) as ei:                      # too many streams
            dec.prefill([prompts[0][:2], prompts[0][:2], prompts[1]], [0, 10, 20, 30], kv)
        assert ei.value.code == wf.WF_E_CAPACITY
        with pytest.raises(wf.WfError) as ei:                      # an empty prompt
            dec.prefill([prompts[0], np.zeros(0, np.int32)], cu, kv)
        assert ei.value.code == wf.WF_E_INVALID_ARG
        with pytest.raises(wf.WfError) as ei:                      # a stream without encoder tokens
            dec.prefill(prompts, [0, 30, 30], kv)
        assert ei.value.code == wf.WF_E_INVALID_ARG
        small = torch.empty((shape.n_layers, 5, 2 * shape.d_model), device="cuda", dtype=torch.bfloat16)
        with pytest.raises(wf.WfError) as ei:                      # K/V buffer smaller than the batch
            dec.cross_kv(e, out=small)
        assert ei.value.code == wf.WF_E_CAPACITY
        r = dec.prefill(prompts, cu, kv, hidden_dtype=torch.float32)   # and the object still works
        torch.cuda.synchronize()
        assert torch.isfinite(r["hidden"]).all() and torch.isfinite(r["logits"]).all()
    finally:
        dec.close()


@pytest.mark.timeout(900)
def test_full_size_cross_kv_every_row_and_prefill_on_a_spread_of_streams(capsys):
    """large-v3 decoder shape on cfg 5's 64 encoder lengths with 100 prompt tokens per stream (the launch
    configuration bench.py times).  The cross-attention keys/values are compared row by row over the whole
    batch on four layers; the prefill is compared on 20 streams spread over the length distribution (every
    fourth of the length order, the longest, and the first, middle and last stream of the packed batch)."""
    import torch
    wl = synth.workload("cfg5")
    shape = synth.DEC_SHAPES["large-v3"]
    enc_lens = [O.stem_length(t + wl.hush_frames) for t in wl.n_frames]
    B = len(enc_lens)
    cu = np.concatenate([[0], np.cumsum(enc_lens)]).astype(np.int32)
    w = synth.make_decoder_weights(shape, wl.seeds["weights"] + 6)
    enc = synth.make_enc_states(int(cu[-1]), shape.d_model, wl.seeds["weights"] + 8)
    prompts = synth.make_prompts([synth.PROMPT_TOKENS] * B, shape.n_vocab, wl.seeds["weights"] + 7)
    dec = wf.Decoder(shape, w, B, int(cu[-1]), synth.PROMPT_TOKENS * B, wf.WF_PRECISION_BF16)
    layers = sorted({0, shape.n_layers // 3, 2 * shape.n_layers // 3, shape.n_layers - 1})
    try:
        e = torch.from_numpy(enc).cuda().bfloat16()
        kv = dec.cross_kv(e)
        r = dec.prefill(prompts, cu, kv, hidden_dtype=torch.bfloat16)
        hidden, logits = r["hidden"].float().cpu().numpy(), r["logits"].cpu().numpy()
        r2 = dec.prefill(prompts, cu, kv, hidden_dtype=torch.bfloat16)
        torch.cuda.synchronize()
        assert torch.equal(r["logits"], r2["logits"])             # deterministic run to run
        kv_host = {l: kv[l].float().cpu().numpy() for l in layers}
    finally:
        dec.close()
    assert np.all(np.isfinite(hidden)) and np.all(np.isfinite(logits))
    w64 = D._cast(w, np.float64)
    enc64 = enc.astype(np.float64)
    for l in layers:                                              # every row of the batch, keys | values
        k, v = D.cross_kv(w64["layers"][l], enc64)
        err = H.rel_err(kv_host[l], np.concatenate([k, v], axis=1))
        with capsys.disabled():
            print(f"[cross_kv large-v3] layer {l}: {cu[-1]} rows, rel err {err:.3e}", flush=True)
        assert err <= H.BF16_TOL
    order = [int(i) for i in np.argsort(enc_lens)]
    picks = sorted(set(order[::4] + [order[-1], 0, B // 2 - 1, B // 2, B - 1]))
    assert len(picks) >= 16
    P = synth.PROMPT_TOKENS
    worst = 0.0
    for i in picks:
        ref = D.prefill_stream(w64, shape.n_heads, prompts[i], enc[cu[i]:cu[i + 1]], _cast_weights=False)
        eh = H.rel_err(hidden[i * P:(i + 1) * P], ref["hidden"])
        el = H.rel_err(logits[i], ref["logits"])
        worst = max(worst, eh, el)
        with capsys.disabled():
            print(f"[prefill large-v3] stream {i}: {enc_lens[i]} encoder tokens, hidden {eh:.3e} logits {el:.3e}", flush=True)
        assert eh <= H.BF16_TOL and el <= H.BF16_TOL
