"""Parity at the benchmark configurations' full sizes, through the same entry points and launch shapes
bench.py times.  The oracle checks every decode row (cheap) and, for the prefills, the first, the last and a
seeded interior row of EVERY block of 32 consecutive query rows of every session - the rows one wave of the
matrix-core kernel owns, so every wave of every workgroup of the launched grid is compared on all its heads -
plus the edges around tile boundaries; KV pools are compared bit for bit."""
import numpy as np
import pytest
import torch

from gpu_helpers import (DevBatch, check_close, gpu_append, gpu_decode, gpu_merged, gpu_prefill, gpu_resume, make_cache,
                         to_dev)
from helpers import fresh_pools, oracle_append, oracle_attn
from oracle import oracle as O
from paper_2603_10342_amd import inputs as I

pytestmark = pytest.mark.gpu


def pools_equal_on_device(cache, kp, vp, dtype):
    """Upload the oracle's pools and compare on the GPU (NaN-poisoned slots compare as raw bits)."""
    for dev_pool, host in ((cache.k_pool_token_major(), kp), (cache.v_pool_token_major(), vp)):
        ref = to_dev(host, dtype)
        assert torch.equal(dev_pool.contiguous().view(torch.int16), ref.view(torch.int16))
        del ref


def sample_rows(b, rng, block=32, edges=(0, 1, 31, 32, 63, 64, 127, 128, 129, 255, 256)):
    """(session, row) pairs: for every session, the first, the last and one seeded interior row of each block of
    `block` consecutive rows, and the rows around the first tile boundaries and the session's end."""
    rs, ri = [], []
    for s in range(b.batch):
        n = int(b.new_lens[s])
        picks = {e for e in edges if e < n} | {n - 1, n - 2, n - 128, n // 2}
        for r0 in range(0, n, block):
            r1 = min(r0 + block, n) - 1
            picks |= {r0, r1, int(rng.integers(r0, r1 + 1))}
        for i in sorted(p for p in picks if 0 <= p < n):
            rs.append(s)
            ri.append(i)
    return np.array(rs, np.int32), np.array(ri, np.int32)


def check_rows(got_full, b, rows, ref, what):
    idx = b.cu_new[rows[0]].astype(np.int64) + rows[1]
    check_close(got_full[idx], ref, b.geom.dtype, what)


def test_config2_decode_full():
    c = I.make_decode()
    g = c.geom
    cache = make_cache(g)
    kp, vp = fresh_pools(g)
    for b in (c.fill, c.step):
        gpu_append(cache, DevBatch(b))
        oracle_append(kp, vp, b)
    torch.cuda.synchronize()
    pools_equal_on_device(cache, kp, vp, g.dtype)
    d = DevBatch(c.step)
    got = gpu_decode(cache, d.q, d.bt, d.ctx, d.max_ctx, g)
    ref = O.decode(kp, vp, g.dtype, c.step.q, c.block_tables, c.ctx_lens, g.num_q_heads, g.scale)
    check_close(got, ref, g.dtype, "config 2 decode")


def test_config3_cold_prefill_every_wave_block():
    b = I.make_cold()
    g = b.geom
    cache = make_cache(g)
    kp, vp = fresh_pools(g)
    d = DevBatch(b)
    gpu_append(cache, d)
    oracle_append(kp, vp, b)
    torch.cuda.synchronize()
    pools_equal_on_device(cache, kp, vp, g.dtype)
    got = gpu_prefill(cache, d)
    assert np.isfinite(got).all()
    rows = sample_rows(b, I.rng_for(I.config_seed(3), 9))
    ref = oracle_attn(kp, vp, b, rows=rows)
    check_rows(got, b, rows, ref, "config 3 cold prefill")


def test_config4_resume_prefill_every_wave_block():
    c = I.make_resume()
    g = c.geom
    cache = make_cache(g)
    kp, vp = fresh_pools(g)
    for b in (c.fill, c.chunk):
        gpu_append(cache, DevBatch(b))
        oracle_append(kp, vp, b)
    torch.cuda.synchronize()
    pools_equal_on_device(cache, kp, vp, g.dtype)
    d = DevBatch(c.chunk)
    got = gpu_resume(cache, d)
    assert np.isfinite(got).all()
    rows = sample_rows(c.chunk, I.rng_for(I.config_seed(4), 9))
    ref = oracle_attn(kp, vp, c.chunk, rows=rows)
    check_rows(got, c.chunk, rows, ref, "config 4 resume prefill")


def test_config5_shapes_one_call_after_another():
    m = I.make_mixed()
    g = m.geom
    cache = make_cache(g)
    kp, vp = fresh_pools(g)
    for b in (m.resume_fill, m.decode_fill, m.cold, m.resume, m.decode):
        gpu_append(cache, DevBatch(b))
        oracle_append(kp, vp, b)
    torch.cuda.synchronize()
    pools_equal_on_device(cache, kp, vp, g.dtype)
    dc, dr, dd = DevBatch(m.cold), DevBatch(m.resume), DevBatch(m.decode)
    got = gpu_prefill(cache, dc)
    rows = sample_rows(m.cold, I.rng_for(I.config_seed(5), 9))
    check_rows(got, m.cold, rows, oracle_attn(kp, vp, m.cold, rows=rows), "config 5 cold")
    got = gpu_resume(cache, dr)
    rows = sample_rows(m.resume, I.rng_for(I.config_seed(5), 10))
    check_rows(got, m.resume, rows, oracle_attn(kp, vp, m.resume, rows=rows), "config 5 resume")
    got = gpu_decode(cache, dd.q, dd.bt, dd.ctx, dd.max_ctx, g)
    ref = O.decode(kp, vp, g.dtype, m.decode.q, m.decode.block_tables, m.decode.ctx_lens, g.num_q_heads, g.scale)
    check_close(got, ref, g.dtype, "config 5 decode")


def test_decode_queue_merged_full():
    """The merged workload bench.py times (64 decodes + 8 resume chunks on long prefixes): every row."""
    c = I.make_decode_queue()
    g = c.geom
    cache = make_cache(g)
    kp, vp = fresh_pools(g)
    for b in (c.fill, c.chunk):
        gpu_append(cache, DevBatch(b))
        oracle_append(kp, vp, b)
    torch.cuda.synchronize()
    pools_equal_on_device(cache, kp, vp, g.dtype)
    got = gpu_merged(cache, DevBatch(c.chunk))
    check_close(got, oracle_attn(kp, vp, c.chunk), g.dtype, "decode queue, merged")
