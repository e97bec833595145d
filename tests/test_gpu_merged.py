"""The decode queue's batch in one launch (paper Sec. III-A; Algorithm 1's Q_D): decodes and short resume
prefills together, against the oracle's resume semantics."""
import numpy as np
import pytest
import torch

from gpu_helpers import (DevBatch, check_close, gpu_append, gpu_decode, gpu_merged, gpu_resume, make_cache, to_f64)
from helpers import fresh_pools, make_batch, oracle_append, oracle_attn
from paper_2603_10342_amd import binding as B
from paper_2603_10342_amd import inputs as I

pytestmark = pytest.mark.gpu


def geom(pages=1024, hq=8, hkv=2, d=128, ps=16, dtype=I.BF16):
    return I.Geometry(hq, hkv, d, ps, pages, dtype)


def filled(g, prefix, new, seed):
    """Caches on both sides with the prefixes in place and the chunk appended; returns (cache, kp, vp, chunk)."""
    bt = I.deal_block_tables(I.rng_for(seed, 0), [a + b for a, b in zip(prefix, new)], g.page_size, g.num_pages)
    fill = make_batch(g, [0] * len(prefix), prefix, seed=seed, bt=bt, sigma_qk=1.0, sigma_v=1.0)
    chunk = make_batch(g, prefix, new, seed=seed, bt=bt, stream=2, sigma_qk=1.0, sigma_v=1.0)
    cache = make_cache(g)
    kp, vp = fresh_pools(g)
    for b in (fill, chunk):
        if b.total_new:
            gpu_append(cache, DevBatch(b))
            oracle_append(kp, vp, b)
    return cache, kp, vp, chunk


MIXES = {
    # decodes among resumes of every row count around the item size (4 rows at G = 4), ragged contexts
    "decodes_and_short_resumes": ([700, 1, 2047, 300, 129, 0, 5000, 15, 16, 1023], [1, 1, 1, 5, 4, 7, 3, 2, 17, 33]),
    # a session without rows in the middle, a chunk that is the whole (short) context, one long chunk
    "empty_and_cold_like": ([100, 40, 0, 900, 0], [1, 0, 9, 64, 130]),
    # contexts that end exactly on page / step / part boundaries
    "boundaries": ([15, 16, 31, 127, 128, 255, 511, 1024, 2047, 4095], [1, 1, 1, 1, 1, 1, 1, 1, 1, 1]),
    "only_resumes": ([2000, 1000], [48, 64]),
    # a chunk long enough for the call to hand the launch to the prefill kernel (same semantics), next to decodes
    "handed_to_the_prefill_kernel": ([500, 1200, 77], [1, 150, 1]),
    # ... and the longest chunk the merged kernel keeps (four full rows items and a remainder)
    "longest_kept": ([500, 1200, 77], [1, 143, 1]),
}


@pytest.mark.parametrize("name", sorted(MIXES))
def test_merged_batch_matches_oracle(name):
    prefix, new = MIXES[name]
    g = geom(pages=2048, hq=8, hkv=2)
    cache, kp, vp, chunk = filled(g, prefix, new, seed=300 + len(name))
    ref = oracle_attn(kp, vp, chunk)
    got = gpu_merged(cache, DevBatch(chunk))
    check_close(got, ref, g.dtype, name)


@pytest.mark.parametrize("hq,hkv", [(4, 4), (8, 4), (32, 8), (16, 2), (16, 1), (6, 2), (40, 8)])
def test_merged_batch_group_sizes(hq, hkv):
    """G = 1, 2, 4, 8, 16 fill the 16 columns exactly; 3 and 5 leave one unused."""
    g = geom(pages=1024, hq=hq, hkv=hkv)
    cache, kp, vp, chunk = filled(g, [333, 1500, 64, 0], [1, 6, 19, 3], seed=41 + hq)
    check_close(gpu_merged(cache, DevBatch(chunk)), oracle_attn(kp, vp, chunk), g.dtype, f"G={hq // hkv}")


def test_merged_equals_the_resume_and_decode_paths_within_tolerance_and_is_reproducible():
    g = geom(pages=2048, hq=32, hkv=8)
    prefix, new = [1800, 2500, 999, 3000], [1, 1, 24, 1]
    cache, kp, vp, chunk = filled(g, prefix, new, seed=77)
    d = DevBatch(chunk)
    ref = oracle_attn(kp, vp, chunk)
    a = gpu_merged(cache, d)
    b = gpu_merged(cache, d)
    assert np.array_equal(a, b)                       # fixed merge order: bit-reproducible
    check_close(a, ref, g.dtype, "merged")
    check_close(gpu_resume(cache, d), ref, g.dtype, "resume path, same batch")
    # the three decodes alone through the decode entry point
    rows = [0, 1, 26]
    dec = gpu_decode(cache, d.q[rows].contiguous(), d.bt[[0, 1, 3]].contiguous(), d.ctx[[0, 1, 3]].contiguous(),
                     d.max_ctx, g)
    check_close(dec, ref[rows], g.dtype, "decode path, the decodes of the batch")


def test_merged_long_context_many_splits():
    g = geom(pages=4096, hq=8, hkv=2)
    cache, kp, vp, chunk = filled(g, [30000, 12345], [6, 1], seed=5)
    check_close(gpu_merged(cache, DevBatch(chunk)), oracle_attn(kp, vp, chunk), g.dtype, "30k context")


def test_merged_on_a_small_partition_shares_span_several_runs_of_page_ids():
    """On 8 CUs the launch has 16 workgroups, so a share is hundreds of steps (a wave's steps then come in several
    runs of 64 pages) and tens of tiles, and crosses sessions, heads and items."""
    g = geom(pages=4096, hq=8, hkv=2)
    cache, kp, vp, chunk = filled(g, [30000, 12345, 5000, 0], [6, 1, 70, 1], seed=15)
    d = DevBatch(chunk)
    ref = oracle_attn(kp, vp, chunk)
    info = B.ag_device_info()
    total, n_xcd = info["num_cus"], info["num_xcd"] or 8
    st = B.ag_stream_create_cumask(B.ag_cumask_build(total, n_xcd, 0, 1))
    try:
        ws = torch.full((B.ag_attn_merged_workspace_bytes(d.total, g.num_q_heads, d.max_ctx) // 4,), float("nan"),
                        dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        B.ag_attn_merged(cache, d.q, d.out, d.bt, d.prefix, d.new, d.cu, d.total, d.max_new, d.max_ctx,
                         g.num_q_heads, g.scale, ws, stream=st)
        torch.cuda.synchronize()
    finally:
        B.ag_stream_destroy(st)
    check_close(to_f64(d.out, g.dtype), ref, g.dtype, "8-CU partition")
    check_close(gpu_merged(cache, d), ref, g.dtype, "whole device, same batch")


def test_merged_more_sessions_than_one_pass_of_the_plan():
    """300 sessions (the plan scans 256 at a time): decodes, empty sessions, short and long chunks in any order."""
    g = geom(pages=8192, hq=8, hkv=2)
    rng = I.rng_for(4242, 0)
    prefix = [int(x) for x in rng.integers(0, 400, size=300)]
    new = [int(x) for x in rng.choice([0, 1, 1, 1, 1, 2, 5, 9, 17, 40], size=300)]
    prefix[7], new[7] = 0, 33                          # a cold-like chunk
    prefix[290], new[290] = 2500, 1                    # a long decode behind the first pass
    cache, kp, vp, chunk = filled(g, prefix, new, seed=91)
    check_close(gpu_merged(cache, DevBatch(chunk)), oracle_attn(kp, vp, chunk), g.dtype, "300 sessions")


def test_merged_names_the_planted_key_under_the_causal_limit():
    """Each row's query points at one key; rows of one item differ in which keys they may see, so a wrong
    per-column limit (the item's instead of the row's) would let a row name a key from its future."""
    g = geom(pages=512, hq=8, hkv=2)
    p, n = 200, 12
    l = p + n
    rng = np.random.default_rng(23)
    k = rng.standard_normal((l, 2, 128)).astype(np.float32)
    k /= np.linalg.norm(k, axis=-1, keepdims=True)
    k = I.bf16_bits_to_f32(I.f32_to_bf16_bits(k))
    v = np.repeat(I.position_bits(np.arange(l), 128)[:, None, :], 2, axis=1)
    # every row's query is the key ONE PAST its own position where that exists (invisible: must not win),
    # plus a weaker pull towards its own position (visible: must win)
    tgt_future = np.minimum(p + np.arange(n) + 1, l - 1)
    tgt_self = p + np.arange(n)
    q = np.zeros((n, 8, 128), np.float32)
    for i in range(n):
        for h in range(8):
            q[i, h] = 400.0 * k[tgt_future[i], h // 4] + 200.0 * k[tgt_self[i], h // 4]
    bt = I.deal_block_tables(I.rng_for(23, 0), [l], 16, g.num_pages)
    fill = make_batch(g, [0], [p], seed=23, bt=bt, k=k[:p], v=v[:p])
    chunk = make_batch(g, [p], [n], seed=23, bt=bt, stream=2, q=q, k=k[p:], v=v[p:])
    cache = make_cache(g)
    kp, vp = fresh_pools(g)
    for b in (fill, chunk):
        gpu_append(cache, DevBatch(b))
        oracle_append(kp, vp, b)
    got = gpu_merged(cache, DevBatch(chunk))
    check_close(got, oracle_attn(kp, vp, chunk), g.dtype, "planted")
    want = I.position_bits(tgt_self, 128)
    for i in range(n - 1):                           # the last row's "future" key is itself
        for h in range(8):
            assert np.array_equal(got[i, h] > 0.5, want[i] > 0.5), (i, h)


def test_merged_other_shapes_take_the_general_path():
    for g in (geom(pages=256, d=64), geom(pages=256, ps=8), geom(pages=128, hq=4, hkv=2, d=64, dtype=I.F32)):
        cache, kp, vp, chunk = filled(g, [70, 200], [1, 9], seed=9)
        check_close(gpu_merged(cache, DevBatch(chunk)), oracle_attn(kp, vp, chunk), g.dtype, str(g))


def test_merged_errors_from_the_host_layer():
    g = geom(pages=256)
    cache, kp, vp, chunk = filled(g, [70, 200], [1, 9], seed=9)
    d = DevBatch(chunk)
    small = torch.empty(16, dtype=torch.float32, device="cuda")
    with pytest.raises(B.AgError) as e:
        B.ag_attn_merged(cache, d.q, d.out, d.bt, d.prefix, d.new, d.cu, d.total, d.max_new, d.max_ctx, g.num_q_heads,
                         g.scale, small)
    assert e.value.status == B.AG_ERR_WORKSPACE
    ws = torch.empty(B.ag_attn_merged_workspace_bytes(d.total, g.num_q_heads, d.max_ctx) // 4, dtype=torch.float32, device="cuda")
    with pytest.raises(B.AgError):
        B.ag_attn_merged(cache, d.q, d.out, d.bt, d.prefix, d.new, d.cu, d.total, d.total + 1, d.max_ctx, g.num_q_heads,
                         g.scale, ws)
    # nothing to do is not an error and touches nothing
    out = torch.full_like(d.q, 7.0)
    B.ag_attn_merged(cache, d.q, out, d.bt, d.prefix, d.new, d.cu, 0, 0, d.max_ctx, g.num_q_heads, g.scale, ws)
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())
