"""The round driver on the GPU: every round's ragged batch goes through the encoder; the bookkeeping it
reports must be what the oracle gives for the same measured processing times, and the states of the last
round must be bit-identical to a direct wf_encode_batch call on the same buffers."""
import numpy as np
import pytest

from oracle import encoder_oracle as O
from oracle import rounds_oracle as R
from paper_2412_11272_amd import binding as wf
from paper_2412_11272_amd import synth
from tests import helpers as H

pytestmark = pytest.mark.gpu

STARTS = [0, 300_000, 1_100_000, 2_500_000]
STEP, TRIM, KEEP, MAXF, TRACK = 200_000, 300, 50, 400, 1000


def _setup(hush_frames):
    import torch
    shape = synth.SHAPES["tiny"]
    w = synth.make_weights(shape, 77)
    hush = synth.make_hush(shape, 78, hush_frames) if hush_frames else None
    cfg = wf.make_config(shape, hush_frames, len(STARTS), len(STARTS) * (MAXF + hush_frames), MAXF + hush_frames)
    enc = wf.Encoder(cfg, w, hush)
    rng = np.random.default_rng(79)
    tracks = np.clip(rng.normal(-0.3, 0.4, size=(len(STARTS), TRACK, shape.n_mels)), -1, 1).astype(np.float32)
    return shape, w, hush, enc, torch.from_numpy(tracks).cuda(), tracks


def test_rounds_driver_matches_oracle_bookkeeping_and_direct_encode():
    import torch
    H_FR = 50
    shape, w, hush, enc, tracks, tracks_h = _setup(H_FR)
    sim = wf.Rounds(STARTS, STEP, TRIM, KEEP, MAXF)
    out = torch.zeros((len(STARTS) * (MAXF + H_FR + 1) // 2 + 4, shape.d_model), device="cuda", dtype=torch.float32)
    try:
        K = 25
        rec = sim.run(enc, tracks, K, out)
        st = sim.stats()
        ref, ref_st = R.run(STARTS, STEP, TRIM, KEEP, MAXF, [r["proc_us"] for r in rec])
        for k in range(K):
            n = ref[k]["n_frames"]
            act = [x for x in n if x >= 1]
            assert rec[k]["start_us"] == ref[k]["start_us"] and rec[k]["end_us"] == ref[k]["end_us"]
            assert rec[k]["n_active"] == len(act)
            assert rec[k]["frames"] == sum(x + H_FR for x in act)
            assert rec[k]["tokens"] == sum(O.stem_length(x + H_FR) for x in act)
        assert st["rounds"] == K and st["frames_total"] == ref_st["frames_total"]
        assert abs(st["mean_latency_us"] - ref_st["mean_latency_us"]) <= 1e-9 * ref_st["mean_latency_us"]
        assert max(max(r["n_frames"]) for r in ref) >= TRIM          # the run reached the trimming regime
        # last round again, directly
        n, ff = ref[-1]["n_frames"], ref[-1]["first_frame"]
        offs = [i * TRACK + ff[i] % (TRACK - MAXF) for i in range(len(n)) if n[i] >= 1]
        lens = [x for x in n if x >= 1]
        direct, cu = enc.encode(tracks.reshape(-1, shape.n_mels), offs, lens, out_dtype=torch.float32)
        torch.cuda.synchronize()
        M = int(cu[-1])
        assert M == rec[-1]["tokens"]
        assert torch.equal(out[:M], direct)
        # and that batch is right: one stream against the oracle
        i = 0
        mel = tracks_h.reshape(-1, shape.n_mels)[offs[i]:offs[i] + lens[i]]
        ref_states = O.encode_stream(w, shape.n_heads, mel, hush)
        assert H.rel_err(direct[cu[i]:cu[i + 1]].cpu().numpy(), ref_states) <= H.BF16_TOL
    finally:
        sim.close()
        enc.close()


def test_rounds_driver_padded_window_baseline():
    import torch
    shape, w, hush, enc, tracks, _ = _setup(0)
    sim = wf.Rounds(STARTS, STEP, TRIM, KEEP, MAXF)
    out = torch.zeros((len(STARTS) * MAXF // 2, shape.d_model), device="cuda", dtype=torch.bfloat16)
    try:
        rec = sim.run(enc, tracks, 8, out, pad_to_frames=MAXF)
        for r in rec:
            assert r["frames"] == r["n_active"] * MAXF and r["tokens"] == r["n_active"] * MAXF // 2
        assert rec[-1]["n_active"] == len(STARTS) - 1 or rec[-1]["n_active"] == len(STARTS)
        assert torch.isfinite(out[:rec[-1]["tokens"]].float()).all()
    finally:
        sim.close()
        enc.close()


def test_rounds_driver_rejects_short_tracks():
    import torch
    shape, w, hush, enc, tracks, _ = _setup(50)
    sim = wf.Rounds(STARTS, STEP, TRIM, KEEP, MAXF)
    out = torch.zeros((1000, shape.d_model), device="cuda", dtype=torch.float32)
    try:
        with pytest.raises(wf.WfError) as ei:
            sim.run(enc, tracks[:, :MAXF].contiguous(), 2, out)
        assert ei.value.code == wf.WF_E_INVALID_ARG
    finally:
        sim.close()
        enc.close()
