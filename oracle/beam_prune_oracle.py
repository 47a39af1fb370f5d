"""CPU oracle for the beam-pruning state machine.  TEST INFRASTRUCTURE ONLY.

Follows the paper's Section "Beam pruning" (new design: search-based reference alignment, selective
transcript token matching and beam reduction, fallback mechanism) step by step, in its order.  The
reference is the token list the previous processing round produced; one call of step() is one decoding
step of the current round and receives that step's highest-probability token.

  1. The beam size starts at 1.
  2. Alignment (first decoding step that yields an ordinary token): search the reference for the first
     occurrence of the token.  Found at i: remember i + 1 as the reference index, beam stays 1.
     Not found: fallback.
  3. Matching (later steps): the best token is compared with the reference token at the index.  Equal:
     beam stays 1, the index advances by one.  Different: fallback.
  4. Selectivity: if the best token is a punctuation, timestamp or any other special token, the step is
     skipped: beam stays 1, the index does not move (this also holds before alignment).  That is the
     whole exemption the paper states: it concerns the CURRENT best token (filter_reference=False takes
     it literally and matches against the reference exactly as the previous round left it).  With
     filter_reference=True (the default) the same kinds of token are also left out of the reference list:
     the paper's stated purpose of the rule is that misplaced timestamps and punctuation must not disturb
     the matching, which they would if an ordinary token could meet a punctuation token on the reference
     side.  This is an extension, not something the paper says.
  5. Fallback: the beam returns to the original size.

Readings where the paper is silent: alignment waits for the first ordinary token (Whisper-style outputs
begin with a timestamp token, which rule 4 exempts from matching); after the match at i the next step is
compared with reference token i + 1; an ordinary token arriving when the reference is used up is new
content with nothing to verify against, so it falls back; a fallback lasts until the decoding session
ends.  beam_for_step[t] is the beam size step t ran with (step 0 runs with 1; a fallback decided at
step t shows from step t + 1 on).

Events: 0 skipped (special / punctuation), 1 aligned, 2 matched, 3 fallback: alignment failed,
4 fallback: mismatch, 5 fallback: reference used up, 6 already at the original beam size.

Only tests may import this; the library's implementation (csrc/beam_prune.hip) shares no code with it.
Pins: tests/test_beam_prune_pins.py and the hand-worked sessions in tests/golden/beam_prune_cases.txt.
"""
from __future__ import annotations

from typing import Iterable, List, Sequence, Tuple

SKIPPED, ALIGNED, MATCHED, FB_ALIGN, FB_MISMATCH, FB_END, FULL = range(7)


class BeamPruner:
    def __init__(self, beam_size: int, reference: Sequence[int], special_from: int, punctuation: Iterable[int] = (),
                 filter_reference: bool = True):
        assert beam_size >= 1
        self.full = int(beam_size)
        self.special_from = int(special_from)
        self.punct = set(int(t) for t in punctuation)
        self.ref = [int(t) for t in reference if not (filter_reference and self.is_exempt(int(t)))]
        self.beam = 1
        self.idx = None            # reference index; None until aligned
        self.fallen = False

    def is_exempt(self, tok: int) -> bool:
        return tok >= self.special_from or tok in self.punct

    def step(self, best_token: int) -> Tuple[int, int]:
        """Feed the best token of one decoding step.  Returns (event, beam size for the next step)."""
        tok = int(best_token)
        if self.fallen:
            return FULL, self.beam
        if self.is_exempt(tok):
            return SKIPPED, self.beam
        if self.idx is None:
            for i, r in enumerate(self.ref):
                if r == tok:
                    self.idx = i + 1
                    return ALIGNED, self.beam
            return self._fall(FB_ALIGN)
        if self.idx >= len(self.ref):
            return self._fall(FB_END)
        if self.ref[self.idx] == tok:
            self.idx += 1
            return MATCHED, self.beam
        return self._fall(FB_MISMATCH)

    def _fall(self, event: int) -> Tuple[int, int]:
        self.fallen = True
        self.beam = self.full
        return event, self.beam


def run_session(beam_size: int, reference: Sequence[int], special_from: int, punctuation: Iterable[int],
                best_tokens: Sequence[int], filter_reference: bool = True):
    """Returns (beam_for_step, events): beam_for_step[t] = beam size step t ran with."""
    p = BeamPruner(beam_size, reference, special_from, punctuation, filter_reference)
    beams: List[int] = []
    events: List[int] = []
    for t in best_tokens:
        beams.append(p.beam)
        ev, _ = p.step(t)
        events.append(ev)
    return beams, events


def summary(beam_size: int, beams: Sequence[int]) -> dict:
    """The two figures the paper's beam-pruning table reports: share of decoding steps with a reduced beam
    and the average beam size."""
    n = len(beams)
    return {"steps": n, "reduce_ratio": sum(1 for b in beams if b < beam_size) / n if n else 0.0,
            "avg_beam": sum(beams) / n if n else 0.0}
