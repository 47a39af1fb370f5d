"""Pins for the front-end oracle (log-mel with the hush word appended at the raw-audio level)."""
import math

import numpy as np
import pytest
import torch

from oracle import frontend_oracle as F
from paper_2412_11272_amd import synth

RNG = np.random.default_rng(321)


def test_shape_facts_of_the_paper():
    # 1 s of 16 kHz audio -> (100, 80); the 8000-sample hush word -> 50 frames = 25 tokens after the stride-2 stem
    assert F.n_frames(16000) == 100 and F.n_frames(8000) == 50 and F.n_frames(30 * 16000) == 3000
    x = synth.make_audio(16000, 1)
    assert F.log_mel(x, None, 80).shape == (100, 80)
    h = synth.make_hush_audio(2)
    assert h.shape == (8000,)
    assert F.log_mel(x, h, 80).shape == (150, 80)
    assert F.log_mel(x, h, 128).shape == (150, 128)


def test_power_spectrum_brute_force_single_frame():
    x = RNG.standard_normal(800)
    P = F.power_spectrogram(x)
    xp = np.concatenate([x[1:201][::-1], x, x[-201:-1][::-1]])
    t = 2
    for f in (0, 1, 7, 100, 200):
        re = im = 0.0
        for n in range(400):
            w = 0.5 - 0.5 * math.cos(2 * math.pi * n / 400)
            v = w * xp[160 * t + n]
            re += v * math.cos(2 * math.pi * f * n / 400)
            im -= v * math.sin(2 * math.pi * f * n / 400)
        assert P[t, f] == pytest.approx(re * re + im * im, rel=1e-10)


def test_pure_tone_closed_form():
    # a cosine on bin k: |X[k]| = N/4, |X[k +- 1]| = N/8 (Hann leakage), everything else 0, for interior frames
    k = 37
    n = np.arange(16000)
    x = np.cos(2 * math.pi * k * n / 400 + 0.3)
    P = F.power_spectrogram(x)
    for t in (5, 40, 90):
        assert P[t, k] == pytest.approx(100.0 ** 2, rel=1e-9)
        assert P[t, k - 1] == pytest.approx(50.0 ** 2, rel=1e-9)
        assert P[t, k + 1] == pytest.approx(50.0 ** 2, rel=1e-9)
        rest = np.delete(P[t], [k - 1, k, k + 1])
        assert rest.max() < 1e-12


def test_parseval_per_frame():
    x = RNG.standard_normal(1600)
    P = F.power_spectrogram(x)
    xp = F.reflect_pad(x, 200)
    w = F.hann_window()
    c = np.full(201, 2.0); c[0] = c[200] = 1.0
    for t in range(P.shape[0]):
        fr = xp[160 * t:160 * t + 400] * w
        assert (P[t] * c).sum() == pytest.approx(400 * (fr ** 2).sum(), rel=1e-10)


def test_reflect_padding_and_frame_centres():
    x = np.arange(1000, dtype=np.float64)
    xp = F.reflect_pad(x, 200)
    assert len(xp) == 1400 and xp[200] == 0 and xp[199] == 1 and xp[0] == 200 and xp[-1] == 799 and xp[1199] == 999
    # an impulse at sample 160 t sits at the window centre (where the Hann window is 1) of frame t only
    imp = np.zeros(1600); imp[480] = 1.0
    P = F.power_spectrogram(imp)
    np.testing.assert_allclose(P[3], 1.0, atol=1e-12)          # |w[200] * 1|^2 on every bin
    assert P[0].max() < 1e-12 and P[6].max() < 1e-12           # frames whose window does not reach it


def test_matches_torch_stft():
    x = synth.make_audio(4000, 5).astype(np.float64)
    S = torch.stft(torch.from_numpy(x), 400, 160, window=torch.hann_window(400, dtype=torch.float64), center=True,
                   pad_mode="reflect", return_complex=True)
    P = (S.abs() ** 2).numpy().T
    np.testing.assert_allclose(F.power_spectrogram(x), P[:F.n_frames(4000)], rtol=1e-9, atol=1e-12)


@pytest.mark.parametrize("n_mels", [80, 128])
def test_mel_filterbank_properties(n_mels):
    fb = F.mel_filterbank(n_mels)
    assert fb.shape == (n_mels, 201) and fb.min() >= 0 and fb.max() <= 1
    assert float(F.hz_to_mel(1000.0)) == pytest.approx(1000.0, abs=0.05)       # the mel scale's anchor
    np.testing.assert_allclose(F.mel_to_hz(F.hz_to_mel([0, 440, 8000])), [0, 440, 8000], atol=1e-9)
    edges = F.mel_to_hz(np.linspace(F.hz_to_mel(0), F.hz_to_mel(8000), n_mels + 2))
    assert np.all(np.diff(edges) > 0) and edges[0] == pytest.approx(0) and edges[-1] == pytest.approx(8000)
    freqs = np.arange(201) * 40.0
    # unit-peak triangles: between the first and the last centre the filters sum to exactly 1
    inside = (freqs >= edges[1]) & (freqs <= edges[n_mels])
    np.testing.assert_allclose(fb[:, inside].sum(axis=0), 1.0, atol=1e-12)
    # filter k is zero outside (edges[k], edges[k+2])
    for k in (0, n_mels // 2, n_mels - 1):
        out = (freqs <= edges[k]) | (freqs >= edges[k + 2])
        assert fb[k, out].max(initial=0.0) == 0.0


def test_log_compression_clamp_and_gain_invariance():
    x = synth.make_audio(8000, 9).astype(np.float64)
    m = F.log_mel(x, None, 80)
    assert m.max() - m.min() <= 2.0 + 1e-12                     # 8 decades / 4
    m10 = F.log_mel(10.0 * x, None, 80)                         # power x100 -> log10 +2 -> output +0.5
    np.testing.assert_allclose(m10, m + 0.5, atol=1e-9)
    z = F.log_mel(np.zeros(1600), None, 80)                     # silence: floor 1e-10 -> (-10 + 4)/4
    np.testing.assert_allclose(z, -1.5, atol=1e-12)


def test_hush_is_appended_at_the_end_at_raw_level():
    x = synth.make_audio(3200, 11).astype(np.float64)
    h = synth.make_hush_audio(12).astype(np.float64)
    P = F.power_spectrogram(np.concatenate([x, h]))
    Px = F.power_spectrogram(x)
    # frames whose window ends before the join are those of x alone; the next ones differ (no reflection there any more)
    last_clean = (3200 - 200) // 160 - 1
    np.testing.assert_allclose(P[:last_clean + 1], Px[:last_clean + 1], rtol=1e-12, atol=1e-15)
    assert np.abs(P[19] - Px[19]).max() > 1e-6
    assert F.log_mel(x, h, 80).shape[0] == 20 + 50
    # prepending instead of appending gives something else
    assert np.abs(F.log_mel(np.concatenate([h, x]), None, 80) - F.log_mel(x, h, 80)).max() > 1e-2
    # batch = every stream alone
    out, cu = F.log_mel_batch([x, x[:1600]], h, 80)
    assert cu.tolist() == [0, 70, 130]
    assert np.array_equal(out[70:], F.log_mel(x[:1600], h, 80))
