"""Pins for oracle/rounds_oracle.py: closed forms that the paper's definitions fix (Section "Operations":
a word's latency = wait until the next round + two rounds; Section "Key Implementation Details": step
length and best-effort mode), exact buffer sequences worked by hand, and conservation of frames."""
import numpy as np

from oracle import rounds_oracle as R

S = 1_000_000       # one second in microseconds


def test_step_longer_than_processing_closed_form():
    """Rounds on the step grid; every arrival waits step/2 on average, then needs the rest of two rounds:
    mean latency = step/2 + step + proc exactly."""
    step, proc = 1 * S, 300_000
    rec, st = R.run([0], step, 1500, 100, 3000, [proc] * 12)
    assert [r["start_us"] for r in rec] == [(k + 1) * step for k in range(12)]
    assert all(r["end_us"] - r["start_us"] == proc for r in rec)
    assert st["mean_latency_us"] == step / 2 + step + proc
    assert st["mean_proc_us"] == proc and st["max_proc_us"] == proc and st["rounds"] == 12


def test_best_effort_closed_form():
    """Step below the processing time: rounds run back to back, s_k = s_0 + k p.  An arrival waits p/2 on
    average and is materialized two rounds later: 2.5 p (the very first, shorter interval aside)."""
    step, p = 10_000, 400_000
    K = 9
    rec, st = R.run([0], step, 1500, 100, 3000, [p] * K)
    assert [r["start_us"] for r in rec] == [step + k * p for k in range(K)]
    # intervals closed so far: rounds 0 .. K-2 (round k's arrivals materialize at e_{k+1})
    first = step * ((step + p + p) - step / 2)          # (0, s_0] materializes at e_1 = s_0 + 2p
    rest = (K - 2) * p * (2.5 * p)
    assert abs(st["mean_latency_us"] - (first + rest) / (step + (K - 2) * p)) < 1e-6


def test_round_start_is_max_of_grid_and_previous_end():
    rec, _ = R.run([0], 1 * S, 1500, 100, 3000, [200_000, 1_700_000, 100_000, 50_000])
    assert [r["start_us"] for r in rec] == [1 * S, 2 * S, 3_700_000, 4_700_000]


def test_buffer_sawtooth_worked_by_hand():
    """1 s steps, trim at 15 s keeping 1 s of materialized context: the buffer grows by 100 frames a round
    to 1500, then everything older than the previous snapshot except 100 frames goes: 1500 -> 300."""
    rec, _ = R.run([0], 1 * S, 1500, 100, 3000, [100_000] * 32)
    n = [r["n_frames"][0] for r in rec]
    assert n[:15] == [100 * (k + 1) for k in range(15)]
    assert n[15:28] == [300 + 100 * k for k in range(13)]
    assert n[28] == 300
    ff = [r["first_frame"][0] for r in rec]
    assert ff[:15] == [0] * 15 and ff[15] == 1300 and ff[28] == 2600


def test_frames_are_conserved_and_bounded():
    rng = np.random.default_rng(3)
    starts = [int(x) for x in rng.integers(0, 20 * S, size=7)]
    procs = [int(x) for x in rng.integers(20_000, 900_000, size=200)]
    rec, st = R.run(starts, 250_000, 1200, 150, 3000, procs)
    for r in rec:
        for i, t0 in enumerate(starts):
            n, ff = r["n_frames"][i], r["first_frame"][i]
            ingested = (r["start_us"] - t0) // R.FRAME_US if r["start_us"] > t0 else 0
            assert ff + n == ingested                      # dropped + held = ingested
            assert 0 <= n <= 3000
    # with trimming on, a buffer exceeds trim_frames by at most what two rounds can add
    worst_gap = max(b["start_us"] - a["start_us"] for a, b in zip(rec, rec[1:]))
    assert max(max(r["n_frames"]) for r in rec) <= 1200 + 2 * (worst_gap // R.FRAME_US) + 150 + 2
    assert st["frames_total"] == sum(sum(r["n_frames"]) for r in rec)


def test_window_cap_drops_the_oldest_audio():
    rec, _ = R.run([0], 40 * S, 3000, 0, 3000, [1000, 1000])
    assert rec[0]["n_frames"] == [3000] and rec[0]["first_frame"] == [1000]     # 40 s arrived, 30 s fit


def test_late_stream_is_inactive_then_counts_from_its_own_start():
    rec, st = R.run([0, 2_500_000], 1 * S, 1500, 100, 3000, [100_000] * 6)
    assert [r["n_frames"][1] for r in rec] == [0, 0, 50, 150, 250, 350]
    # closed intervals after 6 rounds: stream 0 has five of 1 s at 1.5 step + proc = 1.6 s; stream 1 has
    # (2.5 s, 3 s] materialized at e_3 = 4.1 s (4.1 - 2.75 = 1.35 s) and two full ones at 1.6 s
    expect = (5 * 1.6 + 0.5 * 1.35 + 2 * 1.6) / 7.5 * S
    assert abs(st["mean_latency_us"] - expect) < 1e-6
