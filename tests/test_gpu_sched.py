"""The table of pre-established partitions on the device (paper Sec. III-C): every entry's two streams split
the CUs as documented, a rebinding is a lookup that later launches obey, and the attention kernels give the
oracle's result on whichever entry is bound."""
import time

import numpy as np
import pytest
import torch

from gpu_helpers import DevBatch, check_close, make_cache, to_f64
from helpers import fresh_pools, make_batch, oracle_append, oracle_attn
from oracle import controller as OC
from oracle import oracle as O
from paper_2603_10342_amd import binding as B
from paper_2603_10342_amd import inputs as I
from test_gpu_streams import where_it_ran

pytestmark = pytest.mark.gpu


def test_every_entry_partitions_the_device():
    info = B.ag_device_info()
    n_xcd = info["num_xcd"] or 8
    per = info["num_cus"] // n_xcd
    everything = where_it_ran(None, 16384)
    slots = B.Slots(8)
    try:
        assert slots.units() == per and slots.count() == per // 8
        for i in range(slots.count()):
            e = slots.get(i)
            assert e["decode_units"] == min(per, 8 * (i + 1))
            dec = where_it_ran(e["decode_stream"])
            assert len(dec) == e["decode_units"] * n_xcd
            for x in range(n_xcd):                       # the first `units` CUs of every XCD
                assert sum(1 for (xx, _) in dec if xx == x) == e["decode_units"]
            if e["decode_units"] < per:
                pre = where_it_ran(e["prefill_stream"])
                assert not (dec & pre) and (dec | pre) == everything
            else:
                assert e["prefill_stream"] is None and dec == everything
        with pytest.raises(B.AgError):
            slots.get(slots.count())
    finally:
        slots.close()


def test_granularity_that_does_not_divide_the_device_and_bad_granularity():
    info = B.ag_device_info()
    per = info["num_cus"] // (info["num_xcd"] or 8)
    slots = B.Slots(12)
    try:
        sizes = [slots.get(i)["decode_units"] for i in range(slots.count())]
        assert sizes == [12, 24, per]
    finally:
        slots.close()
    for g in (0, -3, per + 1):
        with pytest.raises(B.AgError):
            B.Slots(g)


def test_finest_granularity_gives_one_entry_per_cu_of_an_xcd():
    info = B.ag_device_info()
    n_xcd = info["num_xcd"] or 8
    per = info["num_cus"] // n_xcd
    slots = B.Slots(1)
    try:
        assert slots.count() == per
        for i in (0, 2, per - 2, per - 1):
            e = slots.get(i)
            assert e["decode_units"] == i + 1
            assert len(where_it_ran(e["decode_stream"], 2048)) == (i + 1) * n_xcd
            if i < per - 1:
                assert len(where_it_ran(e["prefill_stream"], 4096)) == (per - i - 1) * n_xcd
    finally:
        slots.close()


def test_bind_follows_the_partition_rule_and_later_launches_obey_it():
    info = B.ag_device_info()
    n_xcd = info["num_xcd"] or 8
    slots = B.Slots(4)
    try:
        S = slots.units()
        for r in (1, 4, 5, 11, 12, 13, 29, 32, 50):
            i = slots.bind(r)
            assert slots.current() == i
            e = slots.get(i)
            assert e["decode_units"] == OC.level_for(S, 4, r)
            assert len(where_it_ran(e["decode_stream"], 2048)) == e["decode_units"] * n_xcd
        # rebinding is a host-side lookup: far below the 50 us the paper allows for a context switch
        t0 = time.perf_counter()
        n = 2000
        for k in range(n):
            slots.bind(1 + (k * 7) % S)
        per_bind_us = (time.perf_counter() - t0) / n * 1e6
        assert per_bind_us < 50.0
    finally:
        slots.close()


def test_decode_and_resume_are_right_on_every_bound_entry():
    """Both request classes on both streams of the bound entry: a decode step, and a resume prefill whose chunks
    (130 and 70 rows on 700- and 300-token prefixes) run the matrix-core tile kernel."""
    g = I.Geometry(8, 2, 128, 16, 1024, I.BF16)
    c = I.make_decode(batch=6, lo=300, hi=1500, num_pages=1024, geom=g, seed=91, sigma_qk=1.0, sigma_v=1.0)
    cache = make_cache(g)
    kp, vp = fresh_pools(g)
    fill, step = DevBatch(c.fill), DevBatch(c.step)
    for b in (c.fill, c.step):
        oracle_append(kp, vp, b)
    ref = O.decode(kp, vp, g.dtype, c.step.q, c.block_tables, c.ctx_lens, g.num_q_heads, g.scale)
    ws = torch.empty(B.ag_attn_decode_workspace_bytes(6, 8, 128, step.max_ctx) // 4, dtype=torch.float32, device="cuda")
    B.ag_kv_append(cache, fill.k_new, fill.v_new, fill.bt, fill.prefix, fill.new, fill.cu, fill.total)
    B.ag_kv_append(cache, step.k_new, step.v_new, step.bt, step.prefix, step.new, step.cu, step.total)
    # a resume batch on a cache of its own
    bt_r = I.deal_block_tables(I.rng_for(92, 0), [830, 370], 16, g.num_pages)
    r_fill = make_batch(g, [0, 0], [700, 300], seed=92, bt=bt_r)
    r_chunk = make_batch(g, [700, 300], [130, 70], seed=92, bt=bt_r, stream=2)
    cache_r = make_cache(g)
    kpr, vpr = fresh_pools(g)
    rf, rc = DevBatch(r_fill), DevBatch(r_chunk)
    for b, d in ((r_fill, rf), (r_chunk, rc)):
        B.ag_kv_append(cache_r, d.k_new, d.v_new, d.bt, d.prefix, d.new, d.cu, d.total)
        oracle_append(kpr, vpr, b)
    ref_r = oracle_attn(kpr, vpr, r_chunk)
    torch.cuda.synchronize()
    slots = B.Slots(8)
    try:
        for r in (3, 16, 32):
            e = slots.get(slots.bind(r))
            for name in ("decode_stream", "prefill_stream"):
                s = e[name]
                if not s:
                    continue
                out = torch.full_like(step.q, float("nan"))
                B.ag_attn_decode(cache, step.q, out, step.bt, step.ctx, step.max_ctx, g.num_q_heads, g.scale, ws, stream=s)
                out_r = torch.full_like(rc.q, float("nan"))
                B.ag_attn_resume(cache_r, rc.q, out_r, rc.bt, rc.prefix, rc.new, rc.cu, rc.total, rc.max_new, rc.max_ctx,
                                 g.num_q_heads, g.scale, stream=s)
                torch.cuda.synchronize()
                check_close(to_f64(out, g.dtype), ref, g.dtype, f"decode on {name} of entry for R={r}")
                check_close(to_f64(out_r, g.dtype), ref_r, g.dtype, f"resume on {name} of entry for R={r}")
    finally:
        torch.cuda.synchronize()
        slots.close()
