"""CPU-only checks of the C-ABI library: it loads, exports what the header declares, and its
host-side validation and ragged-batch planner behave as documented.  No compute call is made."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2412_11272_amd import binding as wf
from paper_2412_11272_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _cfg(**kw):
    base = dict(n_mels=80, d_model=384, n_layers=4, n_heads=6, d_mlp=1536, hush_frames=50, max_streams=4,
                max_total_frames=4000, max_frames_per_stream=3050, precision=0, ln_eps=1e-5)
    base.update(kw)
    return wf.WfConfig(**base)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "wf_encoder.h")).read()
    declared = set(re.findall(r"\b(wf_[a-z_0-9]+)\s*\(", header))
    assert {"wf_encoder_create", "wf_encode_batch", "wf_encoder_destroy"} <= declared
    L = wf.lib()
    for name in declared:
        assert hasattr(L, name), f"{name} declared in the header but not exported"
    assert declared == set(wf.EXPORTS)


def test_config_struct_layout_matches_header():
    assert C.sizeof(wf.WfConfig) == 11 * 4
    assert C.sizeof(wf.WfLayerWeights) == 16 * C.sizeof(C.c_void_p)
    assert C.sizeof(wf.WfWeights) == 8 * C.sizeof(C.c_void_p)


def test_config_check():
    assert wf.config_check(_cfg()) == wf.WF_OK
    for bad in (dict(n_heads=5), dict(d_model=100, n_heads=1), dict(n_mels=81), dict(d_mlp=100), dict(n_layers=-1),
                dict(hush_frames=-1), dict(max_streams=0), dict(max_frames_per_stream=50), dict(precision=7),
                dict(max_total_frames=100)):
        assert wf.config_check(_cfg(**bad)) == wf.WF_E_INVALID_ARG, bad
        assert wf.last_error() != ""
    for shape in synth.SHAPES.values():
        cfg = wf.make_config(shape, 50, 64, 200000, 3050)
        assert wf.config_check(cfg) == wf.WF_OK
    # 32-bit operand offsets: (frames / 2 + 256) * d_mlp * 2 bytes must stay under 4 GiB (large-v3: ~838 k frames)
    big = synth.SHAPES["large-v3"]
    assert wf.config_check(wf.make_config(big, 50, 64, 830000, 3050)) == wf.WF_OK
    assert wf.config_check(wf.make_config(big, 50, 64, 840000, 3050)) == wf.WF_E_INVALID_ARG
    assert "4 GiB" in wf.last_error()


def test_plan_batch_prefix_sums_and_paper_shape_facts():
    cfg = _cfg(max_streams=8, max_total_frames=20000)
    cu, tf, tt = wf.plan_batch(cfg, [100, 3000, 1, 2, 1450])
    lens = [(t + 50 + 1) // 2 for t in (100, 3000, 1, 2, 1450)]
    assert lens == [75, 1525, 26, 26, 750]        # 1 s + hush -> 75; 30 s + hush -> 1525; 15 s incl. hush -> 750
    assert cu.tolist() == [0] + np.cumsum(lens).tolist()
    assert tf == sum(t + 50 for t in (100, 3000, 1, 2, 1450)) and tt == sum(lens)
    cfg0 = _cfg(hush_frames=0, max_frames_per_stream=3000)
    cu, tf, tt = wf.plan_batch(cfg0, [3000, 50])
    assert cu.tolist() == [0, 1500, 1525]          # 30 s -> 1500 tokens, 0.5 s -> 25 tokens


def test_plan_batch_errors():
    cfg = _cfg()
    with pytest.raises(wf.WfError) as e:
        wf.plan_batch(cfg, [100, 0])
    assert e.value.code == wf.WF_E_INVALID_ARG
    with pytest.raises(wf.WfError) as e:
        wf.plan_batch(cfg, [])
    assert e.value.code == wf.WF_E_INVALID_ARG
    with pytest.raises(wf.WfError) as e:
        wf.plan_batch(cfg, [10] * 5)
    assert e.value.code == wf.WF_E_CAPACITY
    with pytest.raises(wf.WfError) as e:
        wf.plan_batch(cfg, [3001])
    assert e.value.code == wf.WF_E_CAPACITY and "max_frames_per_stream" in str(e.value)
    with pytest.raises(wf.WfError) as e:
        wf.plan_batch(cfg, [2000, 2000])
    assert e.value.code == wf.WF_E_CAPACITY and "max_total_frames" in str(e.value)
    assert wf.lib().wf_plan_batch(None, None, 1, None, None, None) == wf.WF_E_INVALID_ARG


def test_null_arguments_are_rejected_without_a_gpu():
    L = wf.lib()
    assert L.wf_encoder_create(None, None, None) == wf.WF_E_INVALID_ARG
    h = C.c_void_p(None)
    cfg = _cfg()
    assert L.wf_encoder_create(C.byref(cfg), None, C.byref(h)) == wf.WF_E_INVALID_ARG and not h
    assert L.wf_encode_batch(None, None, 0, None, None, 1, None, 0, 0, None, None) == wf.WF_E_INVALID_ARG
    L.wf_encoder_destroy(None)                      # NULL-safe
    assert L.wf_kernel_class_count() >= 8
    assert L.wf_encoder_set_lanes(None, 2) == wf.WF_E_INVALID_ARG
    assert L.wf_encoder_get_lanes(None) == wf.WF_E_INVALID_ARG
    assert "NULL" in wf.last_error()


def test_workload_recipes():
    wl = synth.workload("cfg5")
    assert len(wl.n_frames) == 64 and min(wl.n_frames) >= 100 and max(wl.n_frames) <= 3000
    assert synth.workload("cfg5").n_frames == wl.n_frames            # seeded
    wl3 = synth.workload("cfg3")
    assert len(wl3.n_frames) == 16 and min(wl3.n_frames) >= 100 and max(wl3.n_frames) <= 1000
    w, hush, mels = synth.materialize(synth.workload("cfg1"))
    assert hush.shape == (50, 80) and mels[0].shape == (100, 80)
    assert mels[0].min() >= -1 and mels[0].max() <= 1 and abs(mels[0].mean() + 0.3) < 0.05
    assert abs(w["layers"][0]["wq"].std() - 0.02) < 1e-3 and w["layers"][0]["bk"] is None
    w4, h4, m4 = synth.materialize(synth.workload("cfg4a"))
    assert m4[0].shape == (3000, 80) and np.all(m4[0][600:] == -1.0) and len(h4) == 0


@pytest.mark.parametrize("M,N,tm,tn", [(31694, 3840, 256, 256), (31694, 5120, 256, 256), (31694, 1280, 256, 256), (15847, 3840, 256, 256),
                                       (12000, 4096, 256, 256), (6400, 1280, 128, 128), (75, 384, 128, 128), (1, 128, 128, 128),
                                       (65536, 2560, 256, 256), (257, 256, 256, 256), (63408, 1280, 256, 256),
                                       (31694, 3840, 320, 256), (31694, 5120, 320, 256), (31694, 1280, 320, 256), (12000, 5120, 320, 256),
                                       (321, 256, 320, 256)])
def test_gemm_work_units_cover_every_tile_exactly_once(M, N, tm, tn):
    """The workgroup -> tile decoding the GEMM kernel runs (XCD striping, column groups, half-width units for the
    last partial round), enumerated on the host: every column block of every tile row exactly once."""
    units = wf.gemm_tile_map(M, N, tm, tn)
    tiles_m = (M + tm - 1) // tm
    cover = np.zeros((tiles_m, N // (tn // 2)), dtype=np.int32)       # in half-tile columns
    for m0, n0, w in units:
        assert m0 % tm == 0 and 0 <= m0 < tiles_m * tm and n0 % (tn // 2) == 0 and w in (tn, tn // 2) and n0 + w <= N
        if w == tn:
            assert n0 % tn == 0
        cover[m0 // tm, n0 // (tn // 2):(n0 + w) // (tn // 2)] += 1
    assert cover.min() == 1 and cover.max() == 1
    full = int((units[:, 2] == tn).sum())
    assert full % 256 == 0 or len(units) == full                     # halves only after whole rounds of the chip


def test_gemm_tile_choice_follows_the_last_round_of_the_chip():
    """Small batches -> small-batch kernel; in-between -> 128 x 128; large -> 320 or 256 rows, whichever needs fewer
    (weighted) rounds of 256 workgroups.  The headline configuration's four projections all take 320 rows."""
    assert wf.gemm_tile_choice(75, 384) == (0, 0) and wf.gemm_tile_choice(1024, 5120) == (0, 0)
    assert wf.gemm_tile_choice(6400, 1280) == (128, 128) and wf.gemm_tile_choice(2600, 3072) == (128, 128)
    assert wf.gemm_tile_choice(2600, 4096) == (256, 256)          # 176 tiles of 256 x 256: from 160 on the large tile
    for n in (3840, 1280, 5120):
        assert wf.gemm_tile_choice(31694, n) == (320, 256)
    # 12000 x 1280: 235 tiles of 256 rows fill one round; 190 tiles of 320 rows would also take one, each 1.18 x as long
    assert wf.gemm_tile_choice(12000, 1280) == (256, 256)
    assert wf.gemm_tile_choice(12000, 5120) == (320, 256)
    with pytest.raises(wf.WfError):
        wf.gemm_tile_choice(100, 100)


def test_kernel_gelu_stays_close_to_the_erf_form():
    """The polynomial GELU of the bf16 epilogues, run on the host by the library's own code, against the oracle's erf
    form: absolute error <= 1.5e-4 for |z| <= 4 and <= 6e-5 |z| beyond (Phi saturates at 0.99994 past the clamp),
    relative error <= 5e-4 wherever |GELU| > 0.05 (a quarter of the half-ulp of the bf16 value it is rounded to),
    exact zero at zero, and GELU(z) - GELU(-z) = z."""
    from oracle import encoder_oracle as O
    z = np.concatenate([np.linspace(-12, 12, 200001), [0.0, 1e-30, -1e-30, 50.0, -50.0]]).astype(np.float32)
    got = wf.gelu_host(z).astype(np.float64)
    ref = O.gelu(z.astype(np.float64))
    err = np.abs(got - ref)
    assert err[np.abs(z) <= 4].max() <= 1.5e-4
    far = np.abs(z) > 4
    assert (err[far] / np.abs(z[far])).max() <= 6e-5
    big = np.abs(ref) > 0.05
    assert (err[big] / np.abs(ref[big])).max() <= 5e-4
    assert wf.gelu_host(np.zeros(1))[0] == 0.0
    zz = np.linspace(0, 10, 1001).astype(np.float32)
    np.testing.assert_allclose(wf.gelu_host(zz) - wf.gelu_host(-zz), zz, rtol=0, atol=4e-6)

