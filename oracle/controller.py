"""Plain statement of the paper's feedback scheduler (Sec. III-B, Algorithm 1) and of the rule that maps a
decode reservation to a pre-established partition (Sec. III-C).  TEST INFRASTRUCTURE ONLY: the library's
controller (C++) shares no code with this file, and only tests, the smoke test and the benchmark's baseline leg
may import it.

What it computes.  Each control interval the scheduler looks at the mean time per decode step it measured
(the TPOT of Sec. III-B), compares it with a band [theta_low, theta_high], and when the mean lies strictly
outside the band moves two knobs by one increment each, in opposite directions and each inside its own range:
the decode reservation R_min (up when decode is too slow, never above S nor below R_base) and the token budget
B_prefill under which a resume prefill may join the decode queue (down when decode is too slow, within
[B_min, B_max]).  The request classifier and the partition (R_min for decode, the rest for prefill) then use
the new values.  `tick()` is that interval; its order of steps is Algorithm 1's.

Readings where the paper is silent (each also listed with the library's design notes):
  * dK = 0 (no decode step in the interval) makes TPOT_step 0/0; the interval then changes nothing.
  * B_min, B_max, R_base are used by the listing but absent from its input line; they are parameters here.
  * The listing admits any request with len <= B to Q_D; Sec. III-A sends every cold prefill to the
    prefill queue whatever its length.  `classify` follows Sec. III-A for cold prefills and the listing for
    resume prefills.
  * Times are microseconds, R counts allocation units of the device (S of them).

Pins (tests/test_controller_pins.py): the paper's worked example of the partition rule (a 37 % target takes the
40 % partition, Sec. III-C); a trajectory worked by hand from the listing (tests/golden/controller_trace.txt);
closed forms (steps to saturation under a constant overload, the dead band between the thresholds); clamps.
The paper publishes no trace of its controller, so parity with the authors' implementation is unpinned.
"""
from __future__ import annotations

from dataclasses import dataclass

DECODE, RESUME, COLD = 0, 1, 2          # request types
Q_D, Q_P = 0, 1                         # the two queues of Algorithm 1


@dataclass
class Params:
    S: int                  # allocation units on the device
    r_base: int             # floor of the decode reservation
    r_init: int
    b_init: int
    delta_r: int
    delta_b: int
    b_min: int
    b_max: int
    theta_low_us: float
    theta_high_us: float


class Controller:
    def __init__(self, p: Params):
        if not (0 < p.r_base <= p.r_init <= p.S and 0 <= p.b_min <= p.b_init <= p.b_max
                and p.delta_r >= 0 and p.delta_b >= 0 and p.theta_low_us <= p.theta_high_us):
            raise ValueError("inconsistent controller parameters")
        self.p = p
        self.r_min = p.r_init
        self.b_prefill = p.b_init
        self.dL = 0.0
        self.dK = 0
        self.tpot_us = float("nan")

    def record_decode(self, step_us: float) -> None:
        self.dL += step_us
        self.dK += 1

    def tick(self):
        """One control interval.  Returns (r_min, b_prefill, tpot_us or nan when no step was recorded)."""
        p = self.p
        if self.dK == 0:
            self.tpot_us = float("nan")
        else:
            self.tpot_us = self.dL / self.dK
            if self.tpot_us > p.theta_high_us:
                self.b_prefill = max(p.b_min, self.b_prefill - p.delta_b)
                self.r_min = min(p.S, self.r_min + p.delta_r)
            elif self.tpot_us < p.theta_low_us:
                self.b_prefill = min(p.b_max, self.b_prefill + p.delta_b)
                self.r_min = max(p.r_base, self.r_min - p.delta_r)
        self.dL = 0.0
        self.dK = 0
        return self.r_min, self.b_prefill, self.tpot_us

    def classify(self, req_type: int, length: int) -> int:
        if req_type == DECODE:
            return Q_D
        if req_type == RESUME and length <= self.b_prefill:
            return Q_D
        return Q_P

    def partition(self):
        return self.r_min, self.p.S - self.r_min


def level_for(S: int, g: int, r_min: int) -> int:
    """Partitions are pre-established at g, 2g, ... units (the last one S even when g does not divide S).
    Returns the decode size of the smallest one that holds at least r_min units (Sec. III-C), the largest if
    none does."""
    levels = list(range(g, S, g)) + [S]
    for lv in levels:
        if lv >= r_min:
            return lv
    return S
