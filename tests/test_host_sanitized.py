"""The library's host logic under AddressSanitizer + UndefinedBehaviorSanitizer (CPU only).

All sources of the library are rebuilt with both sanitizers on the host side and linked into
tests/host_sanitize_driver.cpp, a small command interpreter over the host-only entry points of the C ABI
(batch planning and validation, processing-round bookkeeping, the beam-pruning state machine, and every entry
point's refusal of bad arguments).  The scenarios of the other host tests are replayed through it: the results
must equal the oracles' and the run must end without a sanitizer report."""
import os
import subprocess

import numpy as np
import pytest

from oracle import beam_prune_oracle as P
from oracle import encoder_oracle as O
from oracle import rounds_oracle as R
from paper_2412_11272_amd import build as B
from tests.test_beam_prune_pins import BEAM, PUNCT, SPECIAL_FROM, filter_flag, load_cases

HERE = os.path.dirname(os.path.abspath(__file__))
CFG = "80 384 4 6 1536 50 8 20000 3050 0 1e-5"


@pytest.fixture(scope="module")
def driver():
    exe = os.path.join(B.OBJ_DIR, "asan", "host_sanitize_driver")
    os.makedirs(os.path.dirname(exe), exist_ok=True)
    return B.build_sanitized_host_driver(os.path.join(HERE, "host_sanitize_driver.cpp"), exe)


def _run(exe, commands):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], input="\n".join(commands) + "\n", capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, f"driver exit {r.returncode}\n{r.stderr[-4000:]}"
    assert "Sanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-4000:]
    return r.stdout.splitlines()


def _vec(v):
    return f"{len(v)} " + " ".join(str(int(x)) for x in v)


def test_planning_and_validation(driver):
    cmds = [f"cfgcheck {CFG}", "cfgcheck 81 384 4 6 1536 50 8 20000 3050 0 1e-5", "cfgcheck 80 384 4 5 1536 50 8 20000 3050 0 1e-5",
            f"plan {CFG} {_vec([100, 3000, 1, 2, 1450])}",
            f"plan {CFG} {_vec([100] * 9)}",                       # more streams than max_streams
            f"plan {CFG} {_vec([3001])}",                          # longer than max_frames_per_stream with the hush
            f"plan {CFG} {_vec([0, 5])}",                          # an empty stream
            f"plan {CFG} {_vec([3000] * 7)}",                      # over max_total_frames
            f"plan {CFG} {_vec([])}", "invalid"]
    out = _run(driver, cmds)
    assert out[0] == "0" and out[1] == "-1" and out[2] == "-1"
    lens = [O.stem_length(t + 50) for t in (100, 3000, 1, 2, 1450)]
    assert out[3].split() == [str(x) for x in [0, sum(t + 50 for t in (100, 3000, 1, 2, 1450)), sum(lens), 0] + np.cumsum(lens).tolist()]
    assert [l.split()[0] for l in out[4:9]] == ["-2", "-2", "-1", "-2", "-1"]
    rcs, tail = out[9].split(" | ")
    assert all(int(x) < 0 for x in rcs.split()), rcs          # every bad call is refused with an error code
    assert tail == "text"


def test_beam_pruning_sessions(driver):
    rng = np.random.default_rng(77)
    cases = [(c["ref"], c["tok"], filter_flag(c)) for c in load_cases()]
    for _ in range(300):
        ref = [int(t) for t in rng.integers(0, 110, size=int(rng.integers(0, 80)))]
        tok = [int(t) for t in rng.integers(0, 130, size=int(rng.integers(0, 120)))]
        if ref and rng.random() < 0.7:
            a = int(rng.integers(0, len(ref)))
            tok = ([100] if rng.random() < 0.5 else []) + [t if rng.random() > 0.03 else int(rng.integers(0, 95)) for t in ref[a:]] + tok[:10]
        cases.append((ref, tok, bool(rng.random() < 0.5)))
    cmds = [f"beam {BEAM} {SPECIAL_FROM} {int(f)} {_vec(PUNCT)} {_vec(ref)} {_vec(tok)}" for ref, tok, f in cases]
    out = _run(driver, cmds)
    assert len(out) == 2 * len(cases)
    for i, (ref, tok, f) in enumerate(cases):
        beams, events = P.run_session(BEAM, ref, SPECIAL_FROM, PUNCT, tok, f)
        want = ["0"] + [str(b) for b in beams] + [str(e) for e in events]
        assert out[2 * i].split() == ["S"] + want, i
        assert out[2 * i + 1].split() == ["T"] + want, i


def test_round_bookkeeping(driver):
    rng = np.random.default_rng(5)
    scenarios = [([0], 1_000_000, 1500, 100, 3000, [100_000] * 32), ([0], 10_000, 1500, 100, 3000, [400_000] * 9),
                 ([0], 40_000_000, 3000, 0, 3000, [1000, 1000]), ([0, 2_500_000], 1_000_000, 1500, 100, 3000, [100_000] * 6)]
    for _ in range(4):
        S = int(rng.integers(1, 65))
        scenarios.append(([int(x) for x in rng.integers(0, 30_000_000, size=S)], int(rng.choice([10_000, 500_000, 2_000_000])),
                          int(rng.choice([300, 1500, 3000])), int(rng.choice([0, 100, 400])), 3000,
                          [int(x) for x in rng.integers(5_000, 1_500_000, size=200)]))
    cmds = [f"rounds {len(st)} {step} {trim} {keep} {mx} {' '.join(map(str, st))} {_vec(procs)}" for st, step, trim, keep, mx, procs in scenarios]
    cmds.append("rounds 1 0 1500 100 3000 0 0")                 # step 0 is refused
    out = _run(driver, cmds)
    pos = 0
    for st, step, trim, keep, mx, procs in scenarios:
        ref, ref_st = R.run(st, step, trim, keep, mx, procs)
        for k in range(len(procs)):
            got = out[pos].split()
            pos += 1
            assert got[:4] == ["R", "0", str(ref[k]["start_us"]), str(ref[k]["end_us"])], k
            assert [int(x) for x in got[4:]] == ref[k]["n_frames"] + ref[k]["first_frame"], k
        q = out[pos].split()
        pos += 1
        assert q[:6] == ["Q", "0", str(ref_st["rounds"]), str(ref_st["frames_total"]), str(ref_st["max_proc_us"]), str(ref_st["last_round_end_us"])]
        assert float(q[6]) == ref_st["mean_proc_us"]
        assert abs(float(q[7]) - ref_st["mean_latency_us"]) <= 1e-12 * max(1.0, ref_st["mean_latency_us"])
    assert out[pos] == "E -1"
