"""Seeded random shapes through every attention entry point against the oracle: session counts, prefix and
chunk lengths, head groupings and block tables drawn at random (small enough for the oracle, large enough to
cross tile, page, split and item boundaries at unplanned places)."""
import numpy as np
import pytest
import torch

from gpu_helpers import (DevBatch, check_close, gpu_append, gpu_decode, gpu_merged, gpu_prefill, gpu_resume, make_cache,
                         pools_match)
from helpers import fresh_pools, make_batch, oracle_append, oracle_attn
from oracle import oracle as O
from paper_2603_10342_amd import inputs as I

pytestmark = pytest.mark.gpu


def draw_case(seed):
    rng = np.random.default_rng(1000 + seed)
    hkv = int(rng.choice([1, 2, 4, 8]))
    G = int(rng.choice([1, 2, 4, 8]))
    batch = int(rng.integers(1, 7))
    prefix = [int(x) for x in rng.choice([0, 1, 15, 16, 17, 63, 64, 65, 200, 777, 1500, 2900], size=batch)]
    new = [int(x) for x in rng.choice([0, 1, 2, 3, 5, 8, 9, 31, 32, 33, 100, 129, 260], size=batch)]
    if sum(new) == 0:
        new[0] = 7
    sigma = float(rng.choice([0.3, 1.0, 2.0]))
    return hkv * G, hkv, prefix, new, sigma


@pytest.mark.parametrize("seed", range(24))
def test_random_shapes(seed):
    hq, hkv, prefix, new, sigma = draw_case(seed)
    total_pages = sum(-(-(p + n + 1) // 16) for p, n in zip(prefix, new)) + 8
    g = I.Geometry(hq, hkv, 128, 16, total_pages, I.BF16)
    caps = [p + n + 1 for p, n in zip(prefix, new)]               # room for one decode token after the chunk
    bt = I.deal_block_tables(I.rng_for(seed, 0), caps, 16, g.num_pages)
    cache = make_cache(g)
    kp, vp = fresh_pools(g)
    if sum(prefix):
        fill = make_batch(g, [0] * len(prefix), prefix, seed=seed, bt=bt, sigma_qk=sigma, sigma_v=1.0)
        gpu_append(cache, DevBatch(fill))
        oracle_append(kp, vp, fill)
    chunk = make_batch(g, prefix, new, seed=seed, bt=bt, stream=2, sigma_qk=sigma, sigma_v=1.0)
    d = DevBatch(chunk)
    gpu_append(cache, d)
    oracle_append(kp, vp, chunk)
    pools_match(cache, kp, vp, g.dtype)
    ref = oracle_attn(kp, vp, chunk)
    what = f"seed {seed}: hq {hq} hkv {hkv} prefix {prefix} new {new}"
    check_close(gpu_resume(cache, d), ref, g.dtype, "resume, " + what)
    check_close(gpu_merged(cache, d), ref, g.dtype, "merged, " + what)
    if not sum(prefix):
        check_close(gpu_prefill(cache, d), ref, g.dtype, "prefill, " + what)
    # one decode token on top of every session that has a context
    ctx = np.asarray([p + n for p, n in zip(prefix, new)], np.int32)
    live = [i for i, c in enumerate(ctx) if c > 0]
    step = make_batch(g, [int(ctx[i]) for i in live], [1] * len(live), seed=seed, bt=np.ascontiguousarray(bt[live]),
                      stream=3, sigma_qk=sigma, sigma_v=1.0)
    ds = DevBatch(step)
    gpu_append(cache, ds)
    oracle_append(kp, vp, step)
    refd = O.decode(kp, vp, g.dtype, step.q, step.block_tables, step.ctx_lens, g.num_q_heads, g.scale)
    check_close(gpu_decode(cache, ds.q, ds.bt, ds.ctx, ds.max_ctx, g), refd, g.dtype, "decode, " + what)
    check_close(gpu_merged(cache, ds), refd, g.dtype, "merged as decode, " + what)
