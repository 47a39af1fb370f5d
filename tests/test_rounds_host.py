"""The library's processing-round bookkeeping (host code behind the C ABI, no GPU call) against
oracle/rounds_oracle.py: integers bit-exact, the mean latency to double rounding."""
import numpy as np
import pytest

from oracle import rounds_oracle as R
from paper_2412_11272_amd import binding as wf


def _compare(starts, step, trim, keep, mx, procs):
    ref, ref_st = R.run(starts, step, trim, keep, mx, procs)
    sim = wf.Rounds(starts, step, trim, keep, mx)
    try:
        for k, p in enumerate(procs):
            s, n, f = sim.begin()
            e = sim.end(p)
            assert s == ref[k]["start_us"] and e == ref[k]["end_us"], k
            assert n.tolist() == ref[k]["n_frames"], k
            assert f.tolist() == ref[k]["first_frame"], k
        st = sim.stats()
    finally:
        sim.close()
    assert st["rounds"] == ref_st["rounds"] and st["frames_total"] == ref_st["frames_total"]
    assert st["max_proc_us"] == ref_st["max_proc_us"] and st["last_round_end_us"] == ref_st["last_round_end_us"]
    assert st["mean_proc_us"] == ref_st["mean_proc_us"]
    assert abs(st["mean_latency_us"] - ref_st["mean_latency_us"]) <= 1e-12 * max(1.0, ref_st["mean_latency_us"])


@pytest.mark.parametrize("seed", range(8))
def test_library_matches_oracle_on_random_scenarios(seed):
    rng = np.random.default_rng(100 + seed)
    S = int(rng.integers(1, 65))
    starts = [int(x) for x in rng.integers(0, 30_000_000, size=S)]
    step = int(rng.choice([10_000, 250_000, 500_000, 1_000_000, 2_000_000]))
    trim = int(rng.choice([300, 1000, 1500, 3000]))
    keep = int(rng.choice([0, 100, 400]))
    procs = [int(x) for x in rng.integers(5_000, 1_500_000, size=300)]
    _compare(starts, step, trim, keep, 3000, procs)


def test_library_matches_oracle_on_the_pinned_cases():
    _compare([0], 1_000_000, 1500, 100, 3000, [100_000] * 32)              # the hand-worked sawtooth
    _compare([0], 10_000, 1500, 100, 3000, [400_000] * 9)                  # best effort
    _compare([0], 40_000_000, 3000, 0, 3000, [1000, 1000])                 # window cap
    _compare([0, 2_500_000], 1_000_000, 1500, 100, 3000, [100_000] * 6)    # late stream


def test_argument_errors():
    with pytest.raises(wf.WfError):
        wf.Rounds([0], 0)
    with pytest.raises(wf.WfError):
        wf.Rounds([0], 1000, trim_frames=4000, max_frames=3000)
    with pytest.raises(wf.WfError):
        wf.Rounds([-5], 1000)
    sim = wf.Rounds([0], 1000)
    try:
        with pytest.raises(wf.WfError):
            sim.end(10)                      # no round open
        sim.begin()
        with pytest.raises(wf.WfError):
            sim.begin()                      # already open
        sim.end(10)
    finally:
        sim.close()
