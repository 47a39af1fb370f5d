"""GPU parity of the log-mel front end (hush word appended at the raw-audio level) against its oracle, and of
the chain audio -> log-mel -> encoder against the chained oracles."""
import numpy as np
import pytest

from oracle import encoder_oracle as O
from oracle import frontend_oracle as F
from paper_2412_11272_amd import binding as wf
from paper_2412_11272_amd import synth

pytestmark = pytest.mark.gpu

# fp32 DFT on the matrix cores against fp64: the normalised log-mel lives in about [-1, 1.5];
# an amplitude error of 1e-7 of the loudest bin on a bin 8 decades down is 4e-4 in log10, 1e-4 after the /4
LOGMEL_ATOL = 1e-4


def _run(n_mels, lens, hush, out_dtype=None, seed=3):
    import torch
    audios = [synth.make_audio(n, seed + i) for i, n in enumerate(lens)]
    fe = wf.Frontend(n_mels, hush, len(lens), sum(lens) + len(lens) * (0 if hush is None else len(hush)))
    try:
        flat = np.concatenate(audios)
        offs = np.concatenate([[0], np.cumsum(lens)[:-1]])
        out, cu = fe.logmel(torch.from_numpy(flat).cuda(), offs, lens, out_dtype=out_dtype)
        torch.cuda.synchronize()
        got = out.float().cpu().numpy()
    finally:
        fe.close()
    ref, cu_ref = F.log_mel_batch(audios, hush, n_mels)
    assert cu.tolist() == cu_ref.tolist()
    return got, ref, cu


@pytest.mark.parametrize("n_mels", [80, 128])
@pytest.mark.parametrize("lens", [[16000], [1600, 48000, 161, 5000, 32001], [201, 320, 159999]])
def test_logmel_parity_with_hush(n_mels, lens):
    hush = synth.make_hush_audio(77)
    got, ref, cu = _run(n_mels, lens, hush)
    assert got.shape == ref.shape and np.all(np.isfinite(got))
    err = np.abs(got - ref).max()
    print(f"\n[logmel n_mels={n_mels} lens={lens}] max abs err {err:.2e}")
    assert err <= LOGMEL_ATOL


def test_logmel_without_hush_short_and_bf16():
    import torch
    got, ref, _ = _run(80, [201, 4000, 1234], None)
    assert np.abs(got - ref).max() <= LOGMEL_ATOL
    got, ref, _ = _run(80, [8000, 3210], synth.make_hush_audio(5), out_dtype=torch.bfloat16)
    assert np.abs(got - ref).max() <= 8e-3            # one bf16 rounding of values up to ~1.5


def test_logmel_errors():
    import torch
    hush = synth.make_hush_audio(1)
    fe = wf.Frontend(80, hush, 2, 40000)
    try:
        a = torch.zeros(40000, device="cuda")
        with pytest.raises(wf.WfError) as e:
            fe.logmel(a, [0, 0, 0], [100, 100, 100])
        assert e.value.code == wf.WF_E_CAPACITY
        with pytest.raises(wf.WfError) as e:
            fe.logmel(a, [0], [40000])
        assert e.value.code == wf.WF_E_CAPACITY
        with pytest.raises(wf.WfError) as e:
            fe.logmel(a, [0], [-1])
        assert e.value.code == wf.WF_E_INVALID_ARG
        with pytest.raises(wf.WfError) as e:
            fe.logmel(a, [0], [1000], out=torch.empty((10, 80), device="cuda"))
        assert e.value.code == wf.WF_E_CAPACITY
    finally:
        fe.close()
    fe0 = wf.Frontend(80, None, 1, 1000)
    try:
        with pytest.raises(wf.WfError) as e:
            fe0.logmel(torch.zeros(1000, device="cuda"), [0], [200])     # shorter than the reflect padding
        assert e.value.code == wf.WF_E_INVALID_ARG
    finally:
        fe0.close()


def test_audio_to_encoder_states_end_to_end():
    """Raw audio + raw-level hush word -> log-mel -> encoder (no mel-level append) against the chained oracles."""
    import torch
    shape = synth.SHAPES["tiny"]
    weights = synth.make_weights(shape, 4242)
    hush = synth.make_hush_audio(6)
    lens = [16000, 4800, 26000]
    audios = [synth.make_audio(n, 50 + i) for i, n in enumerate(lens)]
    mel_ref, cu_f = F.log_mel_batch(audios, hush, shape.n_mels)
    ref, cu_t = O.encode_batch(weights, shape.n_heads, [mel_ref[cu_f[i]:cu_f[i + 1]] for i in range(3)], None)
    fe = wf.Frontend(shape.n_mels, hush, 3, sum(lens) + 3 * len(hush))
    frames = fe.n_frames(lens)
    cfg = wf.make_config(shape, 0, 3, sum(frames), max(frames), wf.WF_PRECISION_BF16)
    enc = wf.Encoder(cfg, weights, None)
    try:
        mel, cu = fe.logmel(torch.from_numpy(np.concatenate(audios)).cuda(), np.concatenate([[0], np.cumsum(lens)[:-1]]), lens)
        assert cu.tolist() == cu_f.tolist() == [0, 150, 230, 442]       # 1 s + 0.5 s hush = 150 frames, as in the paper
        out, cu2 = enc.encode(mel, cu[:-1], frames)
        torch.cuda.synchronize()
        assert cu2.tolist() == cu_t.tolist()
        err = np.abs(out.cpu().numpy() - ref).max() / np.abs(ref).max()
        print(f"\n[audio -> states] rel err {err:.3e}")
        assert err <= 2e-2
    finally:
        enc.close()
        fe.close()
