"""ag_decode_step - append of the step's token, attention and merge in ONE launch - against the oracle (pools
bit for bit, outputs within the bf16 gates) and against ag_kv_append + ag_attn_decode, whose pools and outputs it
must reproduce bit for bit.  The workspace's counters are zeroed once and must come back zero from every call."""
import numpy as np
import pytest
import torch

from gpu_helpers import DevBatch, check_close, gpu_append, i32, make_cache, pools_match, to_dev, to_f64
from helpers import fresh_pools, make_batch, oracle_append
from oracle import oracle as O
from paper_2603_10342_amd import binding as B
from paper_2603_10342_amd import inputs as I
from test_gpu_fullsize import pools_equal_on_device

pytestmark = pytest.mark.gpu


def step_workspace(nb, g, max_ctx, dirty_tail=True):
    n = B.ag_decode_step_workspace_bytes(nb, g.num_q_heads, g.head_dim, max_ctx) // 4
    ws = torch.zeros(n, dtype=torch.float32, device="cuda")
    counters = B.AG_DECODE_STEP_COUNTER_BYTES // 4                    # floats covered by the counter region
    if dirty_tail:
        ws[counters:] = float("nan")                                  # only the counters have to start at zero
    return ws, counters


def both_ways(g, fill, step, ws=None, stream=None):
    """The step through ag_decode_step on one poisoned cache and through ag_kv_append + ag_attn_decode on another.
    Returns (cache_step, out_step, cache_two, out_two, ws, counters)."""
    df, ds = DevBatch(fill), DevBatch(step)
    nb = step.batch
    c1, c2 = make_cache(g), make_cache(g)
    for c in (c1, c2):
        gpu_append(c, df)
    counters = None
    if ws is None:
        ws, counters = step_workspace(nb, g, ds.max_ctx)
    out1, out2 = torch.full_like(ds.q, float("nan")), torch.full_like(ds.q, float("nan"))
    torch.cuda.synchronize()                                           # `stream` may be another stream than the fills'
    B.ag_decode_step(c1, ds.k_new, ds.v_new, ds.q, out1, ds.bt, ds.ctx, ds.max_ctx, g.num_q_heads, g.scale, ws, stream=stream)
    B.ag_kv_append(c2, ds.k_new, ds.v_new, ds.bt, ds.prefix, ds.new, ds.cu, ds.total, stream=stream)
    ws2 = torch.full((B.ag_attn_decode_workspace_bytes(nb, g.num_q_heads, g.head_dim, ds.max_ctx) // 4,), float("nan"),
                     dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    # on the same stream: the shares, hence the bits, follow the number of CUs the stream may use
    B.ag_attn_decode(c2, ds.q, out2, ds.bt, ds.ctx, ds.max_ctx, g.num_q_heads, g.scale, ws2, stream=stream)
    torch.cuda.synchronize()
    return c1, out1, c2, out2, ws, counters


def same_bits(x, y):
    return torch.equal(x.contiguous().view(torch.int16), y.contiguous().view(torch.int16))


@pytest.mark.parametrize("hq,hkv", [(8, 2), (4, 4), (16, 1), (32, 8)])
def test_step_at_boundary_lengths_equals_oracle_and_the_two_calls(hq, hkv):
    g = I.Geometry(hq, hkv, 128, 16, 768, I.BF16)
    ctx = np.array([1, 2, 15, 16, 17, 31, 32, 33, 127, 128, 129, 511, 512, 513, 1023, 1024, 1500, 64], np.int32)
    bt = I.deal_block_tables(I.rng_for(21, 0), ctx, 16, g.num_pages)
    fill = make_batch(g, np.zeros_like(ctx), ctx - 1, seed=21, bt=bt, sigma_qk=1.0, sigma_v=1.0)
    step = make_batch(g, ctx - 1, np.ones_like(ctx), seed=21, bt=bt, stream=2, sigma_qk=1.0, sigma_v=1.0)
    kp, vp = fresh_pools(g)
    for b in (fill, step):
        oracle_append(kp, vp, b)
    ref = O.decode(kp, vp, g.dtype, step.q, bt, ctx, g.num_q_heads, g.scale)
    c1, out1, c2, out2, ws, counters = both_ways(g, fill, step)
    pools_match(c1, kp, vp, g.dtype)                                   # the append half: bit-exact, nothing else touched
    check_close(to_f64(out1, g.dtype), ref, g.dtype, "decode step")
    assert same_bits(out1, out2)
    assert same_bits(c1.k_pool, c2.k_pool) and same_bits(c1.v_pool, c2.v_pool)
    assert bool((ws[:counters] == 0).all())                            # the counters came back zero


def test_steps_in_a_row_share_one_workspace_and_a_smaller_batch_follows():
    """Three growing steps of 40 sessions, then a step of 7 other sessions, all through one workspace that was
    zeroed once: every call must leave the counters as the next one needs them."""
    g = I.Geometry(32, 8, 128, 16, 8192, I.BF16)
    rng = I.rng_for(23, 0)
    ctx0 = I.uniform_lens(rng, 200, 2600, 40)
    bt = I.deal_block_tables(rng, ctx0 + 8, 16, g.num_pages)
    cache = make_cache(g)
    kp, vp = fresh_pools(g)
    fill = make_batch(g, np.zeros_like(ctx0), ctx0, seed=23, bt=bt, sigma_qk=1.0, sigma_v=1.0)
    gpu_append(cache, DevBatch(fill))
    oracle_append(kp, vp, fill)
    ws, counters = step_workspace(40, g, int(ctx0.max()) + 8)
    for i in range(3):
        step = make_batch(g, ctx0 + i, np.ones_like(ctx0), seed=23, bt=bt, stream=3 + i, sigma_qk=1.0, sigma_v=1.0)
        ds = DevBatch(step)
        out = torch.full_like(ds.q, float("nan"))
        B.ag_decode_step(cache, ds.k_new, ds.v_new, ds.q, out, ds.bt, ds.ctx, ds.max_ctx, g.num_q_heads, g.scale, ws)
        torch.cuda.synchronize()
        oracle_append(kp, vp, step)
        ref = O.decode(kp, vp, g.dtype, step.q, bt, ctx0 + i + 1, g.num_q_heads, g.scale)
        check_close(to_f64(out, g.dtype), ref, g.dtype, f"step {i}")
        assert bool((ws[:counters] == 0).all()), f"counters after step {i}"
    pools_equal_on_device(cache, kp, vp, g.dtype)
    # a smaller batch (other sessions, other lengths) through the same workspace
    small = I.make_decode(batch=7, lo=1, hi=900, num_pages=8192, geom=g, seed=24, sigma_qk=1.0, sigma_v=1.0)
    cache2 = make_cache(g)
    kp2, vp2 = fresh_pools(g)
    gpu_append(cache2, DevBatch(small.fill))
    for b in (small.fill, small.step):
        oracle_append(kp2, vp2, b)
    ds = DevBatch(small.step)
    out = torch.full_like(ds.q, float("nan"))
    B.ag_decode_step(cache2, ds.k_new, ds.v_new, ds.q, out, ds.bt, ds.ctx, ds.max_ctx, g.num_q_heads, g.scale, ws)
    torch.cuda.synchronize()
    ref = O.decode(kp2, vp2, g.dtype, small.step.q, small.block_tables, small.ctx_lens, g.num_q_heads, g.scale)
    check_close(to_f64(out, g.dtype), ref, g.dtype, "smaller batch")
    pools_equal_on_device(cache2, kp2, vp2, g.dtype)
    assert bool((ws[:counters] == 0).all())


def test_empty_sessions_get_zero_rows_and_nothing_appended():
    g = I.Geometry(8, 2, 128, 16, 256, I.BF16)
    ctx = np.array([0, 41, 0, 600], np.int32)
    bt = I.deal_block_tables(I.rng_for(25, 0), [16, 41, 16, 600], 16, g.num_pages)
    fill = make_batch(g, [0, 0, 0, 0], [0, 40, 0, 599], seed=25, bt=bt, sigma_qk=1.0, sigma_v=1.0)
    kv = make_batch(g, [0, 40, 0, 599], [1, 1, 1, 1], seed=25, bt=bt, stream=2, sigma_qk=1.0, sigma_v=1.0)   # rows 0, 2 must be ignored
    cache = make_cache(g)
    kp, vp = fresh_pools(g)
    gpu_append(cache, DevBatch(fill))
    oracle_append(kp, vp, fill)
    live = make_batch(g, [40, 599], [1, 1], seed=25, bt=bt[[1, 3]], stream=2)
    live.k_new, live.v_new, live.q = kv.k_new[[1, 3]], kv.v_new[[1, 3]], kv.q[[1, 3]]
    oracle_append(kp, vp, live)
    ref = O.decode(kp, vp, g.dtype, live.q, bt[[1, 3]], [41, 600], g.num_q_heads, g.scale)
    d = DevBatch(kv)
    ws, counters = step_workspace(4, g, 600)
    out = torch.full_like(d.q, float("nan"))
    B.ag_decode_step(cache, d.k_new, d.v_new, d.q, out, d.bt, i32(ctx), 600, g.num_q_heads, g.scale, ws)
    torch.cuda.synchronize()
    got = to_f64(out, g.dtype)
    assert np.all(got[0] == 0) and np.all(got[2] == 0)
    check_close(got[[1, 3]], ref, g.dtype, "live sessions")
    pools_match(cache, kp, vp, g.dtype)                                # the empty sessions' pages stay untouched (NaN)


def test_config2_and_config5_decode_shapes_in_full():
    for make, what in ((I.make_decode, "config 2"), (lambda: I.make_mixed(), "config 5")):
        c = make()
        g = c.geom
        fill, step = (c.fill, c.step) if what == "config 2" else (c.decode_fill, c.decode)
        kp, vp = fresh_pools(g)
        for b in (fill, step):
            oracle_append(kp, vp, b)
        ref = O.decode(kp, vp, g.dtype, step.q, step.block_tables, step.ctx_lens, g.num_q_heads, g.scale)
        c1, out1, c2, out2, ws, counters = both_ways(g, fill, step)
        check_close(to_f64(out1, g.dtype), ref, g.dtype, what)
        assert same_bits(out1, out2), what
        pools_equal_on_device(c1, kp, vp, g.dtype)
        assert bool((ws[:counters] == 0).all())
        del c1, c2


def test_step_on_a_cu_masked_stream_and_replayed_from_a_graph():
    info = B.ag_device_info()
    total, n_xcd = info["num_cus"], info["num_xcd"] or 8
    g = I.Geometry(32, 8, 128, 16, 4096, I.BF16)
    c = I.make_decode(batch=20, lo=100, hi=3000, num_pages=4096, geom=g, seed=27, sigma_qk=1.0, sigma_v=1.0)
    kp, vp = fresh_pools(g)
    for b in (c.fill, c.step):
        oracle_append(kp, vp, b)
    ref = O.decode(kp, vp, g.dtype, c.step.q, c.block_tables, c.ctx_lens, g.num_q_heads, g.scale)
    sd = B.ag_stream_create_cumask(B.ag_cumask_build(total, n_xcd, 0, 5))      # 40 CUs: the grid follows the mask
    try:
        c1, out1, c2, out2, ws, counters = both_ways(g, c.fill, c.step, stream=sd)
        torch.cuda.synchronize()
        check_close(to_f64(out1, g.dtype), ref, g.dtype, "masked stream")
        assert same_bits(out1, out2)
    finally:
        torch.cuda.synchronize()
        B.ag_stream_destroy(sd)
    # graph: the step (which rewrites the same slot with the same token) replayed four times
    ds = DevBatch(c.step)
    out = torch.zeros_like(ds.q)
    B.ag_decode_step(c1, ds.k_new, ds.v_new, ds.q, out, ds.bt, ds.ctx, ds.max_ctx, g.num_q_heads, g.scale, ws)
    torch.cuda.synchronize()
    eager = out.clone()                                                # on an unmasked stream, as the capture below
    check_close(to_f64(eager, g.dtype), ref, g.dtype, "eager")
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        B.ag_decode_step(c1, ds.k_new, ds.v_new, ds.q, out, ds.bt, ds.ctx, ds.max_ctx, g.num_q_heads, g.scale, ws,
                         stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    for r in range(4):
        out.fill_(float("nan"))
        ws[counters:].uniform_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert same_bits(out, eager), f"replay {r}"
        assert bool((ws[:counters] == 0).all())
