"""The library's beam-pruning state machine (host code behind the C ABI) against the oracle: bit-exact
on the hand-worked sessions and on random ones, stepwise and whole-session entry points alike."""
import numpy as np
import pytest

from oracle import beam_prune_oracle as P
from paper_2412_11272_amd import binding as wf
from tests.test_beam_prune_pins import BEAM, PUNCT, SPECIAL_FROM, filter_flag, load_cases


def test_library_on_the_hand_worked_sessions():
    for c in load_cases():
        bp = wf.BeamPruner(BEAM, c["ref"], SPECIAL_FROM, PUNCT, filter_reference=filter_flag(c))
        try:
            beams, events = bp.session(c["tok"])
            assert beams.tolist() == c["beam"], c["name"]
            assert events.tolist() == c["ev"], c["name"]
        finally:
            bp.close()


@pytest.mark.parametrize("filt", [True, False], ids=["filtered-reference", "literal-reference"])
@pytest.mark.parametrize("seed", range(6))
def test_library_matches_oracle_on_random_sessions(seed, filt):
    rng = np.random.default_rng(500 + seed)
    bp = wf.BeamPruner(BEAM, [], SPECIAL_FROM, PUNCT, filter_reference=filt)
    try:
        for _ in range(200):
            ref = [int(t) for t in rng.integers(0, 110, size=int(rng.integers(0, 80)))]   # ordinary, punctuation and special ids
            n = int(rng.integers(0, 120))
            tok = [int(t) for t in rng.integers(0, 130, size=n)]
            if ref and rng.random() < 0.7:                        # overlap with the reference, lightly perturbed
                a = int(rng.integers(0, len(ref)))
                body = [t if rng.random() > 0.03 else int(rng.integers(0, 95)) for t in ref[a:]]
                tok = ([100] if rng.random() < 0.5 else []) + body + tok[:10]
            rb, re = P.run_session(BEAM, ref, SPECIAL_FROM, PUNCT, tok, filt)
            bp.reset(ref)
            beams, events = bp.session(tok)
            assert beams.tolist() == rb and events.tolist() == re
            bp.reset(ref)                                         # same thing one step at a time
            run_with = 1
            for t, (b, e) in zip(tok, zip(rb, re)):
                assert run_with == b
                ev, run_with = bp.step(t)
                assert ev == e
    finally:
        bp.close()


def test_argument_errors():
    with pytest.raises(wf.WfError):
        wf.BeamPruner(0, [1, 2], 100)
    bp = wf.BeamPruner(5, [1, 2], 100)
    try:
        beams, events = bp.session([])
        assert len(beams) == 0 and len(events) == 0
    finally:
        bp.close()
