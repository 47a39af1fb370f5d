"""CPU oracle for the processing-round bookkeeping of many concurrent streams.  TEST INFRASTRUCTURE ONLY.

Plain Python integers (microseconds and 10 ms frames), one step at a time, following the paper's
description of online operation (Section "Operations": processing rounds take a snapshot of the audio
buffer; a segment is materialized only when two consecutive rounds produce it (LocalAgreement-2); the
buffer is periodically trimmed of samples that have been materialized; a word's latency is its wait
until the next round starts plus at least two rounds of processing) and of the step length (Section
"Key Implementation Details": the interval between two consecutive rounds; when it drops below a
round's processing latency the rounds run back to back on the most recent snapshot, "best effort").

The paper fixes no trimming rule beyond that (it depends on the transcript); the reading taken here,
which needs no decoder: audio that arrived before the PREVIOUS round's snapshot has been seen by two
consecutive rounds once the current round ends, so it counts as materialized; once a buffer holds at
least trim_frames frames, its materialized part is dropped except for keep_frames frames of left
context.  A buffer never exceeds max_frames (the model's 30 s window): older audio falls off.

Rules, all in integers:
  * stream i ingests audio continuously from start_us[i]; its buffer begins at buf_start[i];
  * round k starts at s_k: s_0 = min(start_us) + step, s_{k+1} = max(s_k + step, e_k), e_k = s_k + proc_k
    with proc_k supplied by the caller (a measured duration);
  * snapshot: n_i = floor((s_k - buf_start[i]) / 10 ms) frames (0 if the stream has not started), capped
    at max_frames by advancing buf_start[i]; first_frame_i = (buf_start[i] - start_us[i]) / 10 ms;
  * after round k: for every stream with n_i >= trim_frames, committed = floor((s_{k-1} - buf_start[i]) / 10 ms)
    (0 for k = 0 or if negative); buf_start[i] += max(0, committed - keep_frames) * 10 ms;
  * latency: audio of stream i that arrived in (max(s_{k-1}, start_i), s_k] is first seen by round k and
    materialized at e_{k+1}; its mean latency is e_{k+1} minus the interval's midpoint.

Only tests and bench.py's reporting may import this; the product (csrc/rounds.hip) shares no code with it.
Pins: tests/test_rounds_oracle_pins.py (closed forms for constant processing time in both regimes,
conservation of frames, buffer bounds).
"""
from __future__ import annotations

from typing import List, Sequence, Tuple

FRAME_US = 10_000


class RoundSim:
    def __init__(self, start_us: Sequence[int], step_us: int, trim_frames: int, keep_frames: int, max_frames: int):
        assert step_us >= 1 and 1 <= trim_frames <= max_frames and 0 <= keep_frames
        self.start = [int(t) for t in start_us]
        self.buf_start = list(self.start)
        self.step, self.trim, self.keep, self.max_frames = int(step_us), int(trim_frames), int(keep_frames), int(max_frames)
        self.k = 0                       # index of the next round to begin
        self.s_prev = None               # s_{k-1}
        self.s_cur = None                # s_k while a round is open
        self.e_prev = None               # e_{k-1}
        self.n_cur: List[int] = []
        self.pending: List[Tuple[int, int]] = []   # (lo_i, s_k) intervals of the previous round, awaiting e_{k+1}
        self.lat2 = 0                    # sum of len * (2 e - lo - hi)
        self.len_total = 0
        self.frames_total = 0
        self.proc_total = 0
        self.proc_max = 0
        self.dropped = [0] * len(self.start)

    def begin(self) -> Tuple[int, List[int], List[int]]:
        """Open the next round.  Returns (s_k, n_frames per stream, first_frame per stream)."""
        assert self.s_cur is None
        if self.k == 0:
            s = min(self.start) + self.step
        else:
            s = max(self.s_prev + self.step, self.e_prev)
        n, first = [], []
        for i in range(len(self.start)):
            cnt = (s - self.buf_start[i]) // FRAME_US if s > self.buf_start[i] else 0
            if cnt > self.max_frames:
                self.buf_start[i] += (cnt - self.max_frames) * FRAME_US
                self.dropped[i] += cnt - self.max_frames
                cnt = self.max_frames
            n.append(cnt)
            first.append((self.buf_start[i] - self.start[i]) // FRAME_US)
        self.s_cur, self.n_cur = s, n
        return s, n, first

    def end(self, proc_us: int) -> int:
        """Close the open round, which took proc_us.  Returns e_k."""
        assert self.s_cur is not None and proc_us >= 0
        s, e = self.s_cur, self.s_cur + int(proc_us)
        # the previous round's arrivals are now materialized
        for lo, hi in self.pending:
            self.lat2 += (hi - lo) * (2 * e - lo - hi)
            self.len_total += hi - lo
        self.pending = []
        for i in range(len(self.start)):
            lo = max(self.s_prev, self.start[i]) if self.s_prev is not None else self.start[i]
            if s > lo:
                self.pending.append((lo, s))
        # trimming
        for i in range(len(self.start)):
            if self.n_cur[i] >= self.trim and self.s_prev is not None:
                committed = (self.s_prev - self.buf_start[i]) // FRAME_US if self.s_prev > self.buf_start[i] else 0
                drop = max(0, committed - self.keep)
                self.buf_start[i] += drop * FRAME_US
                self.dropped[i] += drop
        self.frames_total += sum(self.n_cur)
        self.proc_total += int(proc_us)
        self.proc_max = max(self.proc_max, int(proc_us))
        self.s_prev, self.e_prev, self.s_cur = s, e, None
        self.k += 1
        return e

    def stats(self) -> dict:
        return {"rounds": self.k,
                "mean_latency_us": self.lat2 / (2 * self.len_total) if self.len_total else 0.0,
                "mean_proc_us": self.proc_total / self.k if self.k else 0.0,
                "max_proc_us": self.proc_max,
                "frames_total": self.frames_total,
                "last_round_end_us": self.e_prev if self.e_prev is not None else 0}


def run(start_us: Sequence[int], step_us: int, trim_frames: int, keep_frames: int, max_frames: int, proc_us: Sequence[int]):
    """Run len(proc_us) rounds with the given processing times.  Returns (per-round records, stats)."""
    sim = RoundSim(start_us, step_us, trim_frames, keep_frames, max_frames)
    rec = []
    for p in proc_us:
        s, n, first = sim.begin()
        e = sim.end(p)
        rec.append({"start_us": s, "end_us": e, "n_frames": n, "first_frame": first})
    return rec, sim.stats()
