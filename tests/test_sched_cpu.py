"""The library's controller and partition rule (C++) against the oracle (oracle/controller.py) and against the
hand-worked trajectory.  Host logic only: no GPU."""
import math
import os
import random
import threading

import pytest

from oracle import controller as OC
from paper_2603_10342_amd import binding as B
from test_controller_pins import P0, read_trace


def same_tpot(a, b):
    return (math.isnan(a) and math.isnan(b)) or a == b


def test_hand_worked_trajectory_native():
    c = B.Controller(**P0)
    for steps, r, b, tpot in read_trace():
        for s in steps:
            c.record_decode(s)
        st = c.tick()
        assert (st["r_min"], st["b_prefill"]) == (r, b) and same_tpot(st["tpot_us"], tpot)
    assert c.get()["intervals"] == len(read_trace())


def test_native_equals_oracle_on_random_runs():
    rnd = random.Random(20260310342)
    for case in range(200):
        S = rnd.randint(1, 64)
        r_base = rnd.randint(1, S)
        b_max = rnd.randint(0, 4096)
        b_min = rnd.randint(0, b_max)
        lo = rnd.uniform(50, 400)
        params = dict(S=S, r_base=r_base, r_init=rnd.randint(r_base, S), b_init=rnd.randint(b_min, b_max),
                      delta_r=rnd.randint(0, 8), delta_b=rnd.randint(0, 512), b_min=b_min, b_max=b_max,
                      theta_low_us=lo, theta_high_us=lo + rnd.choice([0.0, 1.0, 77.7, 300.0]))
        o = OC.Controller(OC.Params(**params))
        n = B.Controller(**params)
        raised = lowered = 0
        for it in range(60):
            for _ in range(rnd.choice([0, 1, 1, 2, 5, 17])):
                t = rnd.choice([rnd.uniform(0, 1000), lo, params["theta_high_us"], 0.1 + 0.2])
                o.record_decode(t)
                n.record_decode(t)
            r0 = o.r_min
            want = o.tick()
            got = n.tick()
            assert (got["r_min"], got["b_prefill"]) == want[:2], (case, it, params)
            assert same_tpot(got["tpot_us"], want[2])            # same sums in the same order: bit-equal
            if not math.isnan(want[2]):
                raised += want[2] > params["theta_high_us"]
                lowered += want[2] < params["theta_low_us"]
            for typ in (OC.DECODE, OC.RESUME, OC.COLD):
                for ln in (0, 1, want[1] - 1, want[1], want[1] + 1, 10 ** 6):
                    if ln >= 0:
                        assert n.classify(typ, ln) == o.classify(typ, ln)
        st = n.get()
        assert (st["intervals"], st["raised"], st["lowered"]) == (60, raised, lowered)
        n.close()


def test_partition_rule_native_equals_oracle_and_paper_example():
    assert B.ag_partition_level_for(100, 10, 37) == 40          # the paper's example, Sec. III-C
    for S in (1, 7, 32, 100):
        for g in range(1, S + 1):
            for r in range(-2, S + 5):
                assert B.ag_partition_level_for(S, g, r) == OC.level_for(S, g, r), (S, g, r)
    for S, g in ((32, 0), (32, -1), (4, 5)):
        with pytest.raises(B.AgError):
            B.ag_partition_level_for(S, g, 1)


def test_bad_parameters_and_arguments():
    for bad in (dict(r_base=0), dict(r_init=2), dict(r_init=40), dict(b_init=1000), dict(b_min=300),
                dict(theta_low_us=400.0), dict(delta_r=-1), dict(delta_b=-1), dict(theta_high_us=float("nan"))):
        with pytest.raises(B.AgError):
            B.Controller(**{**P0, **bad})
    c = B.Controller(**P0)
    for t in (-1.0, float("nan")):
        with pytest.raises(B.AgError):
            c.record_decode(t)
    with pytest.raises(B.AgError):
        c.classify(7, 1)
    with pytest.raises(B.AgError):
        c.classify(B.AG_REQ_RESUME, -1)
    l = B.lib()
    assert l.ag_ctl_tick(None, None) == B.AG_ERR_INVALID_ARG
    assert l.ag_ctl_create(None, None) == B.AG_ERR_INVALID_ARG
    assert l.ag_slots_count(None) < 0 and l.ag_slots_bind(None, 1, None) == B.AG_ERR_INVALID_ARG


def test_concurrent_reports_lose_no_step():
    # the decode thread reports while the scheduler closes intervals: every step lands in exactly one interval
    c = B.Controller(**{**P0, "theta_low_us": 0.0, "theta_high_us": 1e12})
    n_threads, per = 4, 5000
    seen = []
    stop = threading.Event()

    def reporter():
        for _ in range(per):
            c.record_decode(2.0)

    def ticker():
        while not stop.is_set():
            st = c.tick()
            if not math.isnan(st["tpot_us"]):
                seen.append(st["tpot_us"])

    ts = [threading.Thread(target=reporter) for _ in range(n_threads)]
    tk = threading.Thread(target=ticker)
    tk.start()
    for t in ts:
        t.start()
    for t in ts:
        t.join()
    stop.set()
    tk.join()
    assert all(x == 2.0 for x in seen)                   # a mean of equal steps, whatever the cut
    # count what is left in the open interval: closing it must account for the rest
    # (steps are counted through a controller with wide thresholds, so nothing moved)
    assert c.get()["r_min"] == P0["r_init"]
