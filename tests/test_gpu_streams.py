"""CU-masked streams (the counterpart of the paper's pre-created SM partitions, Sec. III-C), the ordering rule
between a writer stream and a reader stream (Sec. III-C, memory management), and the profiling aid."""
import numpy as np
import pytest
import torch

from gpu_helpers import DevBatch, check_close, gpu_append, i32, make_cache, to_f64
from helpers import fresh_pools, make_batch, oracle_append
from oracle import oracle as O
from paper_2603_10342_amd import binding as B
from paper_2603_10342_amd import inputs as I

pytestmark = pytest.mark.gpu


def where_it_ran(stream, n_wg=4096):
    ids = torch.zeros(n_wg, dtype=torch.int32, device="cuda")
    B.ag_probe_placement(ids, 20000, stream)
    torch.cuda.synchronize()
    v = ids.cpu().numpy().astype(np.int64)
    cu = v & 0xFFFF
    xcd = (v >> 16) & 0xF
    return set(zip(xcd.tolist(), cu.tolist()))


def test_masks_built_by_the_library_partition_the_cus_evenly_over_xcds():
    info = B.ag_device_info()
    total, n_xcd = info["num_cus"], info["num_xcd"] or 8
    per = total // n_xcd
    everything = where_it_ran(None, 16384)
    assert len(everything) == total
    for k in (4, 8, 12):
        sd = B.ag_stream_create_cumask(B.ag_cumask_build(total, n_xcd, 0, k))
        sp = B.ag_stream_create_cumask(B.ag_cumask_build(total, n_xcd, k, per - k))
        try:
            dec, pre = where_it_ran(sd), where_it_ran(sp)
        finally:
            B.ag_stream_destroy(sd)
            B.ag_stream_destroy(sp)
        assert len(dec) == k * n_xcd and len(pre) == (per - k) * n_xcd
        assert not (dec & pre) and (dec | pre) == everything
        for x in range(n_xcd):
            assert sum(1 for (xx, _) in dec if xx == x) == k


def test_append_on_one_masked_stream_then_decode_on_another_with_an_event_between():
    """The writer records an event after ag_kv_append; the reader waits for it before ag_attn_decode: the decode
    must see every appended value (paper: decoding never consumes partially written KV)."""
    info = B.ag_device_info()
    total, n_xcd = info["num_cus"], info["num_xcd"] or 8
    per = total // n_xcd
    sw = B.ag_stream_create_cumask(B.ag_cumask_build(total, n_xcd, 8, per - 8))
    sr = B.ag_stream_create_cumask(B.ag_cumask_build(total, n_xcd, 0, 8))
    try:
        g = I.Geometry(8, 2, 128, 16, 1024, I.BF16)
        c = I.make_decode(batch=8, lo=900, hi=1800, num_pages=1024, geom=g, seed=37, sigma_qk=1.0, sigma_v=1.0)
        cache = make_cache(g)
        kp, vp = fresh_pools(g)
        fill, step = DevBatch(c.fill), DevBatch(c.step)
        for b in (c.fill, c.step):
            oracle_append(kp, vp, b)
        ref = O.decode(kp, vp, g.dtype, c.step.q, c.block_tables, c.ctx_lens, g.num_q_heads, g.scale)
        ws = torch.empty(B.ag_attn_decode_workspace_bytes(8, 8, 128, step.max_ctx) // 4, dtype=torch.float32, device="cuda")
        out = torch.full_like(step.q, float("nan"))
        torch.cuda.synchronize()
        ev = torch.cuda.Event()
        writer, reader = torch.cuda.ExternalStream(sw), torch.cuda.ExternalStream(sr)
        B.ag_kv_append(cache, fill.k_new, fill.v_new, fill.bt, fill.prefix, fill.new, fill.cu, fill.total, stream=sw)
        B.ag_kv_append(cache, step.k_new, step.v_new, step.bt, step.prefix, step.new, step.cu, step.total, stream=sw)
        ev.record(writer)
        reader.wait_event(ev)
        B.ag_attn_decode(cache, step.q, out, step.bt, step.ctx, step.max_ctx, g.num_q_heads, g.scale, ws, stream=sr)
        reader.synchronize()
        check_close(to_f64(out, g.dtype), ref, g.dtype, "decode after cross-stream append")
    finally:
        torch.cuda.synchronize()
        B.ag_stream_destroy(sw)
        B.ag_stream_destroy(sr)


def test_profiling_bracket_times_the_main_kernel():
    g = I.Geometry(8, 2, 128, 16, 512, I.BF16)
    c = I.make_decode(batch=4, lo=500, hi=900, num_pages=512, geom=g, seed=41)
    cache = make_cache(g, poison=False)
    gpu_append(cache, DevBatch(c.fill))
    d = DevBatch(c.step)
    gpu_append(cache, d)
    ws = torch.empty(B.ag_attn_decode_workspace_bytes(4, 8, 128, d.max_ctx) // 4, dtype=torch.float32, device="cuda")
    B.ag_prof_enable(8)
    try:
        for _ in range(5):
            B.ag_attn_decode(cache, d.q, d.out, d.bt, d.ctx, d.max_ctx, g.num_q_heads, g.scale, ws)
        r = B.ag_prof_collect()
        assert r["n"] == 5 and 0.5 < r["min_us"] <= r["mean_us"] <= r["max_us"] < 1e4
        assert B.ag_prof_collect()["n"] == 0
    finally:
        B.ag_prof_disable()
    with pytest.raises(B.AgError):
        B.ag_prof_collect()


def test_misaligned_append_source_is_rejected():
    g = I.Geometry(8, 2, 128, 16, 64, I.BF16)
    b = make_batch(g, [0], [20], seed=43)
    d = DevBatch(b)
    cache = make_cache(g)
    k_off = torch.empty(d.k_new.numel() + 8, dtype=d.k_new.dtype, device="cuda")[1:1 + d.k_new.numel()].view_as(d.k_new)
    with pytest.raises(B.AgError) as e:
        B.ag_kv_append(cache, k_off, d.v_new, d.bt, d.prefix, d.new, d.cu, d.total)
    assert e.value.status == B.AG_ERR_INVALID_ARG
