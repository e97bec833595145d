"""The mixed configuration as it is meant (paper Sec. III-C: a prefill thread and a decode thread submit to
their own partitions at the same time, and a decode never consumes partially written KV; Algorithm 1: "launch
decode jobs from Q_D and prefill jobs from Q_P"): decode steps run on a decode-masked stream from one host
thread while the prefill loop (2 cold prefills of 8192 tokens + 8 resume prefills of 512 tokens on 4096-token
prefixes) runs on the complementary stream from another, on one shared cache, and the outputs PRODUCED DURING
THE OVERLAP are compared with the oracle: every row of every overlapped decode step, and for the prefills the
first / last / a seeded interior row of every 32-row block of every session, on every loop."""
import threading
import time

import numpy as np
import pytest
import torch

from gpu_helpers import DevBatch, check_close, gpu_append, make_cache, to_f64
from helpers import fresh_pools, oracle_append, oracle_attn
from oracle import oracle as O
from paper_2603_10342_amd import binding as B
from paper_2603_10342_amd import inputs as I
from test_gpu_fullsize import check_rows, pools_equal_on_device, sample_rows

pytestmark = pytest.mark.gpu

DECODE_CUS_PER_XCD = 8          # 64 of 256 CUs for decode, the rest for prefill
PREFILL_LOOPS = 4
MAX_DECODE_STEPS = 600


def test_config5_outputs_match_the_oracle_while_both_partitions_are_busy():
    info = B.ag_device_info()
    total, n_xcd = info["num_cus"], info["num_xcd"] or 8
    per = total // n_xcd
    m = I.make_mixed()
    g = m.geom
    cache = make_cache(g)                                   # NaN-poisoned pools
    kp, vp = fresh_pools(g)
    for b in (m.resume_fill, m.decode_fill):                # the cached prefixes and decode contexts
        gpu_append(cache, DevBatch(b))
    for b in (m.resume_fill, m.decode_fill, m.cold, m.resume, m.decode):
        oracle_append(kp, vp, b)
    cold, res, dec = DevBatch(m.cold), DevBatch(m.resume), DevBatch(m.decode)
    nb = m.decode.batch
    ws = torch.full((B.ag_attn_decode_workspace_bytes(nb, g.num_q_heads, g.head_dim, dec.max_ctx) // 4,), float("nan"),
                    dtype=torch.float32, device="cuda")
    dec_outs = torch.full((MAX_DECODE_STEPS,) + tuple(dec.q.shape), float("nan"), dtype=dec.q.dtype, device="cuda")
    cold_outs = [torch.full_like(cold.q, float("nan")) for _ in range(PREFILL_LOOPS)]
    res_outs = [torch.full_like(res.q, float("nan")) for _ in range(PREFILL_LOOPS)]
    torch.cuda.synchronize()

    sd = B.ag_stream_create_cumask(B.ag_cumask_build(total, n_xcd, 0, DECODE_CUS_PER_XCD))
    sp = B.ag_stream_create_cumask(B.ag_cumask_build(total, n_xcd, DECODE_CUS_PER_XCD, per - DECODE_CUS_PER_XCD))
    errors = []
    go, done = threading.Event(), threading.Event()
    pre_span = [0.0, 0.0]
    steps = []                                              # (host t0, host t1) of every decode step

    def prefill_thread():
        try:
            ps = torch.cuda.ExternalStream(sp)
            go.wait()
            pre_span[0] = time.perf_counter()
            for k in range(PREFILL_LOOPS):                  # enqueued back to back: the partition stays busy throughout
                B.ag_kv_append(cache, cold.k_new, cold.v_new, cold.bt, cold.prefix, cold.new, cold.cu, cold.total, stream=sp)
                B.ag_attn_prefill(cache, cold.q, cold_outs[k], cold.bt, cold.new, cold.cu, cold.total, cold.max_new,
                                  g.num_q_heads, g.scale, stream=sp)
                B.ag_kv_append(cache, res.k_new, res.v_new, res.bt, res.prefix, res.new, res.cu, res.total, stream=sp)
                B.ag_attn_resume(cache, res.q, res_outs[k], res.bt, res.prefix, res.new, res.cu, res.total, res.max_new,
                                 res.max_ctx, g.num_q_heads, g.scale, stream=sp)
            ps.synchronize()
            pre_span[1] = time.perf_counter()
        except Exception as e:                              # noqa: BLE001 - reported by the main thread
            errors.append(e)
        finally:
            done.set()

    def decode_thread():
        try:
            ds = torch.cuda.ExternalStream(sd)
            i = 0
            after = 0
            while i < MAX_DECODE_STEPS and after < 3:       # a few steps before, all steps during, three steps after
                if i == 3:
                    go.set()
                t0 = time.perf_counter()
                B.ag_kv_append(cache, dec.k_new, dec.v_new, dec.bt, dec.prefix, dec.new, dec.cu, dec.total, stream=sd)
                B.ag_attn_decode(cache, dec.q, dec_outs[i], dec.bt, dec.ctx, dec.max_ctx, g.num_q_heads, g.scale, ws, stream=sd)
                ds.synchronize()                            # a decode step is serial: its token feeds the next step
                steps.append((t0, time.perf_counter()))
                i += 1
                if done.is_set():
                    after += 1
        except Exception as e:                              # noqa: BLE001
            errors.append(e)
        finally:
            go.set()

    tp, td = threading.Thread(target=prefill_thread), threading.Thread(target=decode_thread)
    try:
        tp.start()
        td.start()
        td.join()
        tp.join()
        torch.cuda.synchronize()
    finally:
        torch.cuda.synchronize()
        B.ag_stream_destroy(sd)
        B.ag_stream_destroy(sp)
    assert not errors, errors

    # Steps that ran wholly inside the span in which the prefill partition had work (0.2 ms after the first
    # prefill launch was enqueued up to the moment its stream drained): these overlapped with prefill kernels.
    inside = [i for i, (t0, t1) in enumerate(steps) if t0 > pre_span[0] + 2e-4 and t1 < pre_span[1]]
    assert len(inside) >= 8, (len(steps), len(inside), pre_span[1] - pre_span[0])
    assert len(steps) < MAX_DECODE_STEPS

    # decode: every row of every step, overlapped or not (the context is fixed, so every step has one answer)
    ref = O.decode(kp, vp, g.dtype, m.decode.q, m.decode.block_tables, m.decode.ctx_lens, g.num_q_heads, g.scale)
    first = dec_outs[inside[0]]
    check_close(to_f64(first, g.dtype), ref, g.dtype, f"decode step {inside[0]} (during prefill)")
    for i in range(len(steps)):                             # fixed merge order: bit-identical across steps
        assert torch.equal(dec_outs[i].view(torch.int16), first.view(torch.int16)), f"decode step {i} differs"

    # prefill: every loop's output (all were produced while decode steps ran beside them)
    rows_c = sample_rows(m.cold, I.rng_for(I.config_seed(5), 9))
    rows_r = sample_rows(m.resume, I.rng_for(I.config_seed(5), 10))
    check_rows(to_f64(cold_outs[0], g.dtype), m.cold, rows_c, oracle_attn(kp, vp, m.cold, rows=rows_c), "cold beside decode")
    check_rows(to_f64(res_outs[0], g.dtype), m.resume, rows_r, oracle_attn(kp, vp, m.resume, rows=rows_r), "resume beside decode")
    for k in range(1, PREFILL_LOOPS):
        assert torch.equal(cold_outs[k].view(torch.int16), cold_outs[0].view(torch.int16)), f"cold loop {k} differs"
        assert torch.equal(res_outs[k].view(torch.int16), res_outs[0].view(torch.int16)), f"resume loop {k} differs"
    assert bool(torch.isfinite(cold_outs[0].float()).all()) and bool(torch.isfinite(res_outs[0].float()).all())
    pools_equal_on_device(cache, kp, vp, g.dtype)
