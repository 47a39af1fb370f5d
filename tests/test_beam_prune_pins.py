"""Pins for oracle/beam_prune_oracle.py: sessions worked by hand from the paper's rules
(tests/golden/beam_prune_cases.txt) and the properties those rules imply."""
import os

import numpy as np

from oracle import beam_prune_oracle as P

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "beam_prune_cases.txt")
BEAM, SPECIAL_FROM, PUNCT = 5, 100, (90, 91)


def load_cases(path=GOLDEN):
    cases, cur = [], None
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, *vals = line.split()
        if key == "case":
            cur = {"name": vals[0]}
            cases.append(cur)
        else:
            cur[key] = [int(v) for v in vals]
    return cases


def filter_flag(case) -> bool:
    """Cases carry "filter 0" when they are worked under the literal rule (reference matched as it stands)."""
    return bool(case.get("filter", [1])[0])


def test_hand_worked_sessions():
    cases = load_cases()
    assert len(cases) == 11
    assert sum(1 for c in cases if not filter_flag(c)) == 3
    for c in cases:
        beams, events = P.run_session(BEAM, c["ref"], SPECIAL_FROM, PUNCT, c["tok"], filter_flag(c))
        assert beams == c["beam"], c["name"]
        assert events == c["ev"], c["name"]


def test_the_two_readings_differ_only_through_exempt_tokens_in_the_reference():
    rng = np.random.default_rng(5)
    differ = 0
    for _ in range(200):
        ref = _random_session(rng, 30)
        tok = ref[int(rng.integers(0, 10)):] + [int(t) for t in rng.integers(0, 80, size=5)]
        # no exempt token in the reference: the literal and the filtering rule are the same machine
        assert P.run_session(BEAM, ref, SPECIAL_FROM, PUNCT, tok, True) == P.run_session(BEAM, ref, SPECIAL_FROM, PUNCT, tok, False)
        mixed_ref = []
        for t in ref:
            if rng.random() < 0.2:
                mixed_ref.append(int(rng.choice([90, 91, 100, 160])))
            mixed_ref.append(t)
        a, _ = P.run_session(BEAM, mixed_ref, SPECIAL_FROM, PUNCT, tok, True)
        b, _ = P.run_session(BEAM, mixed_ref, SPECIAL_FROM, PUNCT, tok, False)
        # the literal rule can only fall back earlier: an ordinary token that meets an exempt reference token mismatches
        assert sum(a) <= sum(b)
        differ += a != b
    assert differ > 100


def _random_session(rng, n_ref):
    ref = [int(t) for t in rng.integers(0, 80, size=n_ref)]
    return ref


def test_a_verbatim_repeat_never_leaves_beam_one_inside_the_reference():
    rng = np.random.default_rng(1)
    for _ in range(50):
        ref = _random_session(rng, int(rng.integers(1, 60)))
        start = int(rng.integers(0, len(ref)))
        # re-decoding the reference from the first occurrence of ref[start]
        first = ref.index(ref[start])
        tok = ref[first:]
        beams, events = P.run_session(BEAM, ref, SPECIAL_FROM, PUNCT, tok)
        assert beams == [1] * len(tok)
        assert events == [P.ALIGNED] + [P.MATCHED] * (len(tok) - 1)


def test_exempt_tokens_never_change_the_outcome_for_ordinary_tokens():
    rng = np.random.default_rng(2)
    for _ in range(50):
        ref = _random_session(rng, 30)
        tok = [int(t) for t in rng.integers(0, 80, size=40)]
        if rng.random() < 0.5:
            tok[:10] = ref[5:15]
        beams0, ev0 = P.run_session(BEAM, ref, SPECIAL_FROM, PUNCT, tok)
        # sprinkle timestamps and punctuation between the ordinary tokens
        mixed, keep = [], []
        for t in tok:
            while rng.random() < 0.4:
                mixed.append(int(rng.choice([90, 91, 100, 150, 101])))
            keep.append(len(mixed))
            mixed.append(t)
        beams1, ev1 = P.run_session(BEAM, ref, SPECIAL_FROM, PUNCT, mixed)
        assert [ev1[i] for i in keep] == ev0
        assert [beams1[i] for i in keep] == beams0
        assert all(ev1[i] in (P.SKIPPED, P.FULL) for i in range(len(mixed)) if i not in set(keep))


def test_beam_is_one_until_a_single_fallback_and_full_afterwards():
    rng = np.random.default_rng(3)
    for _ in range(100):
        ref = _random_session(rng, int(rng.integers(0, 40)))
        tok = [int(t) for t in rng.integers(0, 120, size=50)]
        beams, events = P.run_session(BEAM, ref, SPECIAL_FROM, PUNCT, tok)
        falls = [i for i, e in enumerate(events) if e in (P.FB_ALIGN, P.FB_MISMATCH, P.FB_END)]
        assert len(falls) <= 1
        if falls:
            f = falls[0]
            assert beams[:f + 1] == [1] * (f + 1) and beams[f + 1:] == [BEAM] * (len(tok) - f - 1)
            assert all(e == P.FULL for e in events[f + 1:])
        else:
            assert beams == [1] * len(tok)
        s = P.summary(BEAM, beams)
        n1 = beams.count(1)
        assert s["reduce_ratio"] == n1 / len(tok) and s["avg_beam"] == (n1 + BEAM * (len(tok) - n1)) / len(tok)


def test_beam_size_one_has_nothing_to_prune():
    beams, _ = P.run_session(1, [1, 2, 3], SPECIAL_FROM, PUNCT, [9, 9, 9])
    assert beams == [1, 1, 1] and P.summary(1, beams)["reduce_ratio"] == 0.0


def test_exempt_tokens_inside_the_reference_do_not_matter_either():
    rng = np.random.default_rng(4)
    for _ in range(50):
        ref = _random_session(rng, 30)
        tok = ref[int(rng.integers(0, 10)):] + [int(t) for t in rng.integers(0, 80, size=5)]
        mixed_ref = []
        for t in ref:
            while rng.random() < 0.3:
                mixed_ref.append(int(rng.choice([90, 91, 100, 160])))
            mixed_ref.append(t)
        assert P.run_session(BEAM, ref, SPECIAL_FROM, PUNCT, tok) == P.run_session(BEAM, mixed_ref, SPECIAL_FROM, PUNCT, tok)
