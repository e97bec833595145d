"""Pins for the scheduler oracle (oracle/controller.py): values the paper prints, a hand-worked trajectory,
closed forms and invariants.  CPU only."""
import math
import os
import random

import pytest

from oracle import controller as OC

HERE = os.path.dirname(__file__)
P0 = dict(S=32, r_base=4, r_init=8, b_init=256, delta_r=4, delta_b=64, b_min=64, b_max=512,
          theta_low_us=200.0, theta_high_us=300.0)


def read_trace():
    rows = []
    for line in open(os.path.join(HERE, "golden", "controller_trace.txt")):
        if line.startswith("#") or not line.strip():
            continue
        steps, r, b, tpot = [x.strip() for x in line.split("|")]
        rows.append(([] if steps == "-" else [float(x) for x in steps.split(",")], int(r), int(b), float(tpot)))
    return rows


def run_trace(make, rows):
    c = make(OC.Params(**P0))
    out = []
    for steps, _, _, _ in rows:
        for s in steps:
            c.record_decode(s)
        out.append(c.tick())
    return out


def test_hand_worked_trajectory():
    rows = read_trace()
    assert len(rows) >= 25
    for (steps, r, b, tpot), got in zip(rows, run_trace(OC.Controller, rows)):
        assert got[0] == r and got[1] == b, (steps, got)
        assert (math.isnan(tpot) and math.isnan(got[2])) or got[2] == tpot


def test_partition_rule_paper_example():
    # Sec. III-C: ten partitions at 10 % .. 100 %; a 37 % target takes the 40 % partition.
    assert OC.level_for(100, 10, 37) == 40
    # the neighbours of that example, and the ends of the range
    assert OC.level_for(100, 10, 40) == 40
    assert OC.level_for(100, 10, 41) == 50
    assert OC.level_for(100, 10, 1) == 10
    assert OC.level_for(100, 10, 100) == 100
    assert OC.level_for(100, 10, 250) == 100          # nothing larger exists
    # a granularity that does not divide S: the last partition is the whole device
    assert [OC.level_for(32, 5, r) for r in (5, 6, 30, 31, 32)] == [5, 10, 30, 32, 32]


def test_level_is_smallest_sufficient_brute_force():
    for S in (8, 32, 100):
        for g in (1, 3, 4, 10):
            levels = sorted(set(list(range(g, S, g)) + [S]))
            for r in range(0, S + 1):
                want = min(l for l in levels if l >= r)
                assert OC.level_for(S, g, r) == want


def test_saturation_closed_form():
    # constant overload: R reaches S after ceil((S - R0) / dR) intervals and stays; B reaches B_min likewise
    for dr, db in ((1, 10), (4, 64), (5, 100), (7, 33)):
        p = OC.Params(**{**P0, "delta_r": dr, "delta_b": db})
        c = OC.Controller(p)
        n_r = math.ceil((p.S - p.r_init) / dr)
        n_b = math.ceil((p.b_init - p.b_min) / db)
        for i in range(1, max(n_r, n_b) + 3):
            c.record_decode(10 * p.theta_high_us)
            r, b, _ = c.tick()
            assert r == min(p.S, p.r_init + i * dr)
            assert b == max(p.b_min, p.b_init - i * db)
            assert (r == p.S) == (i >= n_r) and (b == p.b_min) == (i >= n_b)


def test_relaxation_closed_form():
    p = OC.Params(**{**P0, "r_init": 30, "b_init": 64})
    c = OC.Controller(p)
    for i in range(1, 12):
        c.record_decode(1.0)
        r, b, _ = c.tick()
        assert r == max(p.r_base, 30 - 4 * i) and b == min(p.b_max, 64 + 64 * i)


def test_dead_band_and_thresholds_are_strict():
    c = OC.Controller(OC.Params(**P0))
    for t in (200.0, 250.0, 300.0):                   # at a threshold nothing moves: both tests are strict
        c.record_decode(t)
        assert c.tick()[:2] == (8, 256)
    c.record_decode(math.nextafter(300.0, 1e9))
    assert c.tick()[:2] == (12, 192)
    c.record_decode(math.nextafter(200.0, 0.0))
    assert c.tick()[:2] == (8, 256)


def test_interval_without_decode_changes_nothing_and_counters_reset():
    c = OC.Controller(OC.Params(**P0))
    assert c.tick()[:2] == (8, 256) and math.isnan(c.tpot_us)
    c.record_decode(1000.0)
    c.tick()
    # the overload of the last interval is not seen again
    assert c.tick()[:2] == (12, 192)
    c.record_decode(250.0)
    assert c.tick() == (12, 192, 250.0)


def test_tpot_is_the_mean_not_the_last_or_the_max():
    c = OC.Controller(OC.Params(**P0))
    for s in (1000.0, 10.0, 10.0, 10.0):              # mean 257.5: inside the band although one step is far above
        c.record_decode(s)
    assert c.tick() == (8, 256, 257.5)
    for s in (10.0, 10.0, 10.0, 1200.0):              # mean 307.5: above, although the median is far below
        c.record_decode(s)
    assert c.tick() == (12, 192, 307.5)


def test_invariants_random():
    rnd = random.Random(7)
    for _ in range(50):
        p = OC.Params(S=rnd.randint(4, 64), r_base=1, r_init=1, b_init=0, delta_r=rnd.randint(0, 9),
                      delta_b=rnd.randint(0, 300), b_min=0, b_max=rnd.randint(0, 2000),
                      theta_low_us=100.0, theta_high_us=rnd.choice([100.0, 150.0, 400.0]))
        p.r_base = rnd.randint(1, p.S)
        p.r_init = rnd.randint(p.r_base, p.S)
        p.b_min = rnd.randint(0, p.b_max)
        p.b_init = rnd.randint(p.b_min, p.b_max)
        c = OC.Controller(p)
        r0, b0 = c.r_min, c.b_prefill
        for _ in range(200):
            for _ in range(rnd.randint(0, 3)):
                c.record_decode(rnd.uniform(0, 600))
            r, b, t = c.tick()
            assert p.r_base <= r <= p.S and p.b_min <= b <= p.b_max
            assert abs(r - r0) <= p.delta_r and abs(b - b0) <= p.delta_b
            # R and B move in opposite directions or not at all
            assert (r - r0) * (b - b0) <= 0
            if not math.isnan(t):
                if t > p.theta_high_us:
                    assert r >= r0 and b <= b0
                elif t < p.theta_low_us:
                    assert r <= r0 and b >= b0
                else:
                    assert (r, b) == (r0, b0)
            assert c.partition() == (r, p.S - r)
            r0, b0 = r, b


def test_classification():
    c = OC.Controller(OC.Params(**P0))
    assert c.classify(OC.DECODE, 1) == OC.Q_D
    assert c.classify(OC.DECODE, 10 ** 6) == OC.Q_D           # a decode is never rerouted
    assert c.classify(OC.RESUME, 256) == OC.Q_D               # len <= B
    assert c.classify(OC.RESUME, 257) == OC.Q_P
    assert c.classify(OC.COLD, 10) == OC.Q_P                  # cold prefills always take the prefill queue
    c.record_decode(1000.0)
    c.tick()                                                  # B 256 -> 192
    assert c.classify(OC.RESUME, 256) == OC.Q_P and c.classify(OC.RESUME, 192) == OC.Q_D


def test_bad_parameters_rejected():
    for bad in (dict(r_base=0), dict(r_init=2), dict(r_init=40), dict(b_init=1000), dict(b_min=300),
                dict(theta_low_us=400.0), dict(delta_r=-1)):
        with pytest.raises(ValueError):
            OC.Controller(OC.Params(**{**P0, **bad}))


# ---- does the suite have teeth?  plant mistakes in a copy of the oracle's source ----
MUTANTS = {
    "sign_of_r_step": ("self.r_min = min(p.S, self.r_min + p.delta_r)", "self.r_min = min(p.S, self.r_min - p.delta_r)"),
    "no_upper_clamp": ("self.r_min = min(p.S, self.r_min + p.delta_r)", "self.r_min = self.r_min + p.delta_r"),
    "floor_is_zero": ("self.r_min = max(p.r_base, self.r_min - p.delta_r)", "self.r_min = max(0, self.r_min - p.delta_r)"),
    "b_moves_with_r": ("self.b_prefill = max(p.b_min, self.b_prefill - p.delta_b)", "self.b_prefill = min(p.b_max, self.b_prefill + p.delta_b)"),
    "threshold_not_strict": ("if self.tpot_us > p.theta_high_us:", "if self.tpot_us >= p.theta_high_us:"),
    "low_uses_high": ("elif self.tpot_us < p.theta_low_us:", "elif self.tpot_us < p.theta_high_us:"),
    "tpot_is_sum": ("self.tpot_us = self.dL / self.dK", "self.tpot_us = self.dL"),
    "counters_not_reset": ("        self.dL = 0.0\n        self.dK = 0\n        return", "        return"),
    "cold_by_length": ("if req_type == RESUME and length <= self.b_prefill:", "if length <= self.b_prefill:"),
    "budget_strict": ("length <= self.b_prefill", "length < self.b_prefill"),
    "level_rounds_down": ("if lv >= r_min:", "if lv + g > r_min:"),
}


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pins_catch_planted_mistake(name):
    src = open(OC.__file__).read()
    a, b = MUTANTS[name]
    assert src.count(a) >= 1
    ns = {"__name__": "mutant"}
    mutated = src.replace(a, b)
    import sys
    import types
    mod = types.ModuleType("mutant_" + name)
    sys.modules[mod.__name__] = mod          # dataclasses looks the module up
    try:
        exec(compile(mutated, "mutant", "exec"), mod.__dict__)
        failed = []
        rows = read_trace()
        try:
            for (steps, r, b_, tpot), got in zip(rows, run_trace(mod.Controller, rows)):
                assert got[0] == r and got[1] == b_
                assert (math.isnan(tpot) and math.isnan(got[2])) or got[2] == tpot
        except Exception:
            failed.append("trace")
        try:
            assert mod.level_for(100, 10, 37) == 40 and mod.level_for(100, 10, 41) == 50
        except Exception:
            failed.append("level")
        try:
            c = mod.Controller(mod.Params(**P0))
            assert c.classify(mod.RESUME, 256) == mod.Q_D and c.classify(mod.RESUME, 257) == mod.Q_P
            assert c.classify(mod.COLD, 10) == mod.Q_P
        except Exception:
            failed.append("classify")
        assert failed, f"no pin noticed the planted mistake {name}"
    finally:
        del sys.modules[mod.__name__]
