"""The page manager with a device: a prefill on one CU-masked stream, committed, then a decode on another
stream that acquires the sessions first (paper Sec. III-C: mutex for the buffers, events between the two
threads' kernels, decode never reads partly written KV)."""
import numpy as np
import pytest
import torch

from gpu_helpers import DevBatch, check_close, i32, make_cache, to_dev, to_f64
from helpers import fresh_pools, oracle_append, oracle_attn
from oracle import oracle as O
from paper_2603_10342_amd import binding as B
from paper_2603_10342_amd import inputs as I

pytestmark = pytest.mark.gpu


def test_prefill_commit_then_decode_acquire_across_streams():
    g = I.Geometry(8, 2, 128, 16, 512, I.BF16)
    prompt = [700, 333, 1200, 64]
    nb = len(prompt)
    max_pages = 96
    pager = B.Pager(g.num_pages, g.page_size, 8, max_pages)
    slots = B.Slots(8)
    e = slots.get(slots.bind(8))
    s_dec, s_pre = e["decode_stream"], e["prefill_stream"]
    try:
        sess = [pager.open() for _ in range(nb)]
        starts = [pager.reserve(s, n) for s, n in zip(sess, prompt)]
        assert starts == [0] * nb
        bt = pager.export(sess)
        # the prompt's data, drawn for exactly this block table
        cold = I.draw_batch(g, bt, [0] * nb, prompt, 4242, 1, sigma_qk=1.0, sigma_v=1.0)
        kp, vp = fresh_pools(g)
        oracle_append(kp, vp, cold)
        ref_cold = oracle_attn(kp, vp, cold)
        cache = make_cache(g)
        d = DevBatch(cold)
        torch.cuda.synchronize()
        # prefill thread's work, on the prefill partition
        B.ag_kv_append(cache, d.k_new, d.v_new, d.bt, d.prefix, d.new, d.cu, d.total, stream=s_pre)
        B.ag_attn_prefill(cache, d.q, d.out, d.bt, d.new, d.cu, d.total, d.max_new, g.num_q_heads, g.scale, stream=s_pre)
        for s in sess:
            pager.commit(s, s_pre)
        assert [pager.lengths(s)["sealed"] for s in sess] == prompt
        # decode thread: one more token per session, on the decode partition
        dstart = [pager.reserve(s, 1) for s in sess]
        assert dstart == prompt
        bt2 = pager.export(sess)
        for r, n in enumerate(prompt):                   # sealed pages kept their place
            assert np.array_equal(bt2[r, :n // 16], bt[r, :n // 16])
        step = I.draw_batch(g, bt2, prompt, [1] * nb, 4242, 2, sigma_qk=1.0, sigma_v=1.0)
        oracle_append(kp, vp, step)
        ref_dec = O.decode(kp, vp, g.dtype, step.q, bt2, np.asarray(prompt, np.int32) + 1, g.num_q_heads, g.scale)
        ds = DevBatch(step)
        ws = torch.empty(B.ag_attn_decode_workspace_bytes(nb, g.num_q_heads, 128, ds.max_ctx) // 4, dtype=torch.float32, device="cuda")
        out = torch.full_like(ds.q, float("nan"))
        before = pager.stats()
        sealed = [pager.acquire(s, s_dec) for s in sess]
        after = pager.stats()
        assert sealed == prompt
        # every acquire either made the decode stream wait or found the prefill already complete
        assert after["waits_issued"] + after["waits_skipped"] - before["waits_issued"] - before["waits_skipped"] == nb
        B.ag_kv_append(cache, ds.k_new, ds.v_new, ds.bt, ds.prefix, ds.new, ds.cu, ds.total, stream=s_dec)
        B.ag_attn_decode(cache, ds.q, out, ds.bt, ds.ctx, ds.max_ctx, g.num_q_heads, g.scale, ws, stream=s_dec)
        for s in sess:
            pager.commit(s, s_dec)
        torch.cuda.synchronize()
        check_close(to_f64(d.out, g.dtype), ref_cold, g.dtype, "prefill on the prefill partition")
        check_close(to_f64(out, g.dtype), ref_dec, g.dtype, "decode after acquire")
        # same stream as the last commit, or an event that has completed: no wait is issued
        w0 = pager.stats()["waits_issued"]
        pager.acquire(sess[0], s_dec)
        pager.acquire(sess[1], s_pre)                    # other stream, but the device is idle: event complete
        assert pager.stats()["waits_issued"] == w0
        for s in sess:
            pager.close(s)
        assert pager.stats()["free_pages"] == g.num_pages
    finally:
        torch.cuda.synchronize()
        pager.destroy()
        slots.close()


def test_a_reader_behind_a_long_writer_is_made_to_wait():
    """The writer stream is kept busy by a long prefill; the acquire must issue a wait, and the reader's result
    must still see every appended value."""
    g = I.Geometry(8, 2, 128, 16, 2048, I.BF16)
    pager = B.Pager(g.num_pages, g.page_size, 4, 600)
    slots = B.Slots(16)
    e = slots.get(slots.bind(16))
    s_dec, s_pre = e["decode_stream"], e["prefill_stream"]
    try:
        n = 8000
        s = pager.open()
        pager.reserve(s, n)
        bt = pager.export([s])
        cold = I.draw_batch(g, bt, [0], [n], 777, 1, sigma_qk=1.0, sigma_v=1.0)
        kp, vp = fresh_pools(g)
        oracle_append(kp, vp, cold)
        cache = make_cache(g)
        d = DevBatch(cold)
        q1 = d.q[-1:].contiguous()
        ctx = i32([n])
        ref = O.decode(kp, vp, g.dtype, cold.q[-1:], bt, np.asarray([n], np.int32), g.num_q_heads, g.scale)
        ws = torch.empty(B.ag_attn_decode_workspace_bytes(1, g.num_q_heads, 128, n) // 4, dtype=torch.float32, device="cuda")
        out = torch.full_like(q1, float("nan"))
        torch.cuda.synchronize()
        B.ag_kv_append(cache, d.k_new, d.v_new, d.bt, d.prefix, d.new, d.cu, d.total, stream=s_pre)
        for _ in range(3):                               # keeps the writer's stream busy past the acquire
            B.ag_attn_prefill(cache, d.q, d.out, d.bt, d.new, d.cu, d.total, d.max_new, g.num_q_heads, g.scale, stream=s_pre)
        pager.commit(s, s_pre)
        w0 = pager.stats()["waits_issued"]
        assert pager.acquire(s, s_dec) == n
        issued = pager.stats()["waits_issued"] - w0
        B.ag_attn_decode(cache, q1, out, d.bt, ctx, n, g.num_q_heads, g.scale, ws, stream=s_dec)
        torch.cuda.synchronize()
        assert issued == 1
        check_close(to_f64(out, g.dtype), ref, g.dtype, "decode behind a long prefill")
        pager.close(s)
    finally:
        torch.cuda.synchronize()
        pager.destroy()
        slots.close()


def test_pages_of_a_closed_session_are_not_rewritten_under_a_reader_still_in_flight():
    """Session A's decode is queued behind a long kernel on the reader's stream and released; A is closed and
    session B, which gets A's pages back from the free list, has its prompt appended into them on the writer's
    stream.  Launch order is fixed: long kernel, A's decode, release, close(A), B's append.  close must have
    waited for A's decode, so A's result is the oracle's and B's append lands afterwards."""
    g = I.Geometry(8, 2, 128, 16, 1024, I.BF16)
    pager = B.Pager(g.num_pages, g.page_size, 4, 600)
    slots = B.Slots(16)
    e = slots.get(slots.bind(16))
    s_dec, s_pre = e["decode_stream"], e["prefill_stream"]
    try:
        n = 8000
        a = pager.open()
        pager.reserve(a, n)
        bt_a = pager.export([a])
        fill = I.draw_batch(g, bt_a, [0], [n], 901, 1, sigma_qk=1.0, sigma_v=1.0)
        kp, vp = fresh_pools(g)
        oracle_append(kp, vp, fill)
        ref = O.decode(kp, vp, g.dtype, fill.q[-1:], bt_a, np.asarray([n], np.int32), g.num_q_heads, g.scale)
        cache = make_cache(g)
        d = DevBatch(fill)
        q1, ctx = d.q[-1:].contiguous(), i32([n])
        ws = torch.empty(B.ag_attn_decode_workspace_bytes(1, g.num_q_heads, 128, n) // 4, dtype=torch.float32, device="cuda")
        out = torch.full_like(q1, float("nan"))
        busy_out = torch.empty_like(d.q)
        B.ag_kv_append(cache, d.k_new, d.v_new, d.bt, d.prefix, d.new, d.cu, d.total, stream=s_pre)
        pager.commit(a, s_pre)
        torch.cuda.synchronize()
        # reader's stream: a long prefill first (it only reads A's pages), then A's decode
        pager.acquire(a, s_dec)
        for _ in range(3):
            B.ag_attn_prefill(cache, d.q, busy_out, d.bt, d.new, d.cu, d.total, d.max_new, g.num_q_heads, g.scale, stream=s_dec)
        B.ag_attn_decode(cache, q1, out, d.bt, ctx, n, g.num_q_heads, g.scale, ws, stream=s_dec)
        pager.release(a, s_dec)
        w0 = pager.stats()["close_waits"]
        pager.close(a)                                   # must not return while the decode can still read the pages
        assert pager.stats()["close_waits"] - w0 >= 1
        b = pager.open()
        pager.reserve(b, n)
        bt_b = pager.export([b])
        assert set(bt_b[0, :n // 16].tolist()) == set(bt_a[0, :n // 16].tolist())      # the same physical pages
        other = I.draw_batch(g, bt_b, [0], [n], 902, 1, sigma_qk=4.0, sigma_v=4.0)
        do = DevBatch(other)
        B.ag_kv_append(cache, do.k_new, do.v_new, do.bt, do.prefix, do.new, do.cu, do.total, stream=s_pre)
        pager.commit(b, s_pre)
        torch.cuda.synchronize()
        check_close(to_f64(out, g.dtype), ref, g.dtype, "decode of the closed session")
        pager.close(b)
        assert pager.stats()["free_pages"] == g.num_pages
    finally:
        torch.cuda.synchronize()
        pager.destroy()
        slots.close()
