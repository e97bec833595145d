"""GPU parity: the HIP path, called through the C ABI, against the fp64 oracle
on the same seeded inputs.  Pools start NaN-poisoned, so any read of an
unwritten slot or an unreferenced page turns an output into NaN.

Tolerances (tests/gpu_helpers.py): bf16 max-abs 2e-2 and mean-abs 2e-3 (the
stated gate) plus relative Frobenius 1e-2 and a per-row bound; fp32 1e-5
absolute and relative; KV append bit-exact.
"""
import numpy as np
import pytest
import torch

from gpu_helpers import (DevBatch, check_close, gpu_append, gpu_decode, gpu_prefill, gpu_resume, i32, make_cache,
                         pools_match, run_phase, to_dev)
from helpers import fresh_pools, make_batch, oracle_append, oracle_attn
from oracle import oracle as O
from paper_2603_10342_amd import binding as B
from paper_2603_10342_amd import inputs as I

pytestmark = pytest.mark.gpu


def slm(pages=256, hq=8, hkv=2, d=128, dtype=I.BF16):
    return I.Geometry(hq, hkv, d, 16, pages, dtype)


# ------------------------------------------------------------------ config 1
def test_tiny_fp32_cold_resume_decode():
    c = I.make_tiny()
    g = c.geom
    cache = make_cache(g)
    kp, vp = fresh_pools(g)
    got, ref = run_phase(cache, kp, vp, c.cold, "cold")
    check_close(got, ref, g.dtype, "cold")
    pools_match(cache, kp, vp, g.dtype)
    got, ref = run_phase(cache, kp, vp, c.resume, "resume")
    check_close(got, ref, g.dtype, "resume")
    for i, step in enumerate(c.decode_steps):
        got, ref = run_phase(cache, kp, vp, step, "decode")
        check_close(got, ref, g.dtype, f"decode step {i}")
    pools_match(cache, kp, vp, g.dtype)


def test_tiny_in_bf16_uses_the_general_kernels():
    c = I.make_tiny(dtype=I.BF16, sigma_qk=1.0, sigma_v=1.0)
    g = c.geom
    cache = make_cache(g)
    kp, vp = fresh_pools(g)
    for b, kind in [(c.cold, "cold"), (c.resume, "resume"), (c.decode_steps[0], "decode")]:
        got, ref = run_phase(cache, kp, vp, b, kind)
        check_close(got, ref, g.dtype, kind)
    pools_match(cache, kp, vp, g.dtype)


# ------------------------------------------------------------------ append
@pytest.mark.parametrize("dtype", [I.F32, I.BF16])
@pytest.mark.parametrize("d", [64, 128])
def test_append_is_bit_exact(dtype, d):
    g = I.Geometry(8, 4, d, 16, 96, dtype)
    lens_a = [5, 16, 17, 0, 100]
    lens_b = [12, 1, 30, 7, 0]
    bt = I.deal_block_tables(I.rng_for(3, 0), [a + b + 40 for a, b in zip(lens_a, lens_b)], 16, 96)
    cache = make_cache(g)
    kp, vp = fresh_pools(g)
    first = make_batch(g, [0] * 5, lens_a, seed=3, bt=bt)
    second = make_batch(g, lens_a, lens_b, seed=3, bt=bt, stream=2)
    third = make_batch(g, [a + b for a, b in zip(lens_a, lens_b)], [1] * 5, seed=3, bt=bt, stream=3)
    for b in (first, second, third):
        gpu_append(cache, DevBatch(b))
        oracle_append(kp, vp, b)
    torch.cuda.synchronize()
    pools_match(cache, kp, vp, dtype)          # NaN-poisoned elsewhere: untouched slots must stay untouched


# ------------------------------------------------------------------ decode (matrix-core path)
@pytest.mark.parametrize("hq,hkv", [(8, 2), (4, 4), (16, 1), (6, 2)])
def test_decode_boundary_lengths(hq, hkv):
    g = slm(pages=640, hq=hq, hkv=hkv)
    ctx = np.array([1, 15, 16, 17, 31, 32, 33, 127, 128, 129, 511, 512, 513, 1023, 1024, 1500, 64, 2], np.int32)
    bt = I.deal_block_tables(I.rng_for(5, 0), ctx, 16, g.num_pages)
    fill = make_batch(g, np.zeros_like(ctx), ctx - 1, seed=5, bt=bt)
    step = make_batch(g, ctx - 1, np.ones_like(ctx), seed=5, bt=bt, stream=2)
    cache = make_cache(g)
    kp, vp = fresh_pools(g)
    gpu_append(cache, DevBatch(fill))
    oracle_append(kp, vp, fill)
    got, ref = run_phase(cache, kp, vp, step, "decode")
    check_close(got, ref, g.dtype, "decode")
    pools_match(cache, kp, vp, g.dtype)


def test_decode_zero_length_context_gives_zeros():
    g = slm()
    ctx = np.array([0, 40, 0], np.int32)
    bt = I.deal_block_tables(I.rng_for(6, 0), [16, 40, 16], 16, g.num_pages)
    fill = make_batch(g, [0, 0, 0], [0, 40, 0], seed=6, bt=bt)
    cache = make_cache(g)
    kp, vp = fresh_pools(g)
    d = DevBatch(fill)
    gpu_append(cache, d)
    oracle_append(kp, vp, fill)
    q = to_dev(I.normal_values(6, 9, 0, (3, g.num_q_heads, g.head_dim), 1.0, g.dtype), g.dtype)
    got = gpu_decode(cache, q, d.bt, i32(ctx), 40, g)
    assert np.all(got[0] == 0) and np.all(got[2] == 0)
    ref = O.decode(kp, vp, g.dtype, I.normal_values(6, 9, 0, (3, g.num_q_heads, g.head_dim), 1.0, g.dtype)[1:2],
                   bt[1:2], [40], g.num_q_heads, g.scale)
    check_close(got[1:2], ref, g.dtype, "decode")


@pytest.mark.parametrize("gain", [1.0, 4.0])
def test_decode_sharp_logits(gain):
    """Q, K ~ N(0, gain^2): logits of std ~ gain (x sqrt(D)/sqrt(D)), softmax far from flat, |O| ~ |V|."""
    g = slm(pages=1024)
    ctx = np.array([700, 2049, 513, 96], np.int32)
    bt = I.deal_block_tables(I.rng_for(7, 0), ctx, 16, g.num_pages)
    fill = make_batch(g, np.zeros_like(ctx), ctx - 1, seed=7, bt=bt, sigma_qk=1.0, sigma_v=1.0)
    step = make_batch(g, ctx - 1, np.ones_like(ctx), seed=7, bt=bt, stream=2, sigma_qk=gain, sigma_v=1.0)
    cache = make_cache(g)
    kp, vp = fresh_pools(g)
    gpu_append(cache, DevBatch(fill))
    oracle_append(kp, vp, fill)
    got, ref = run_phase(cache, kp, vp, step, "decode")
    check_close(got, ref, g.dtype, "decode sharp")
    assert np.abs(ref).mean() > 0.02          # outputs are O(|V|) here: the absolute gate has teeth


def test_decode_names_the_planted_position():
    """V rows spell their logical position in binary; each head's query is planted on one key."""
    g = slm(pages=512, hq=8, hkv=2)
    ctx = np.array([1000, 517, 33], np.int32)
    bt = I.deal_block_tables(I.rng_for(8, 0), ctx, 16, g.num_pages)
    rng = np.random.default_rng(8)
    ks, vs, qs, tg = [], [], [], []
    for l in ctx:
        k = rng.standard_normal((l, 2, 128)).astype(np.float32)
        k = I.bf16_bits_to_f32(I.f32_to_bf16_bits(k))
        t = rng.integers(0, l, size=(1, 8))
        t[0, 0], t[0, 1] = l - 1, 0            # the ends of the context
        qs.append(I.planted_queries(k, t, 4, gain=40.0))
        ks.append(k)
        vs.append(np.repeat(I.position_bits(np.arange(l), 128)[:, None, :], 2, axis=1))
        tg.append(t[0])
    fill = make_batch(g, np.zeros_like(ctx), ctx, seed=8, bt=bt, k=np.concatenate(ks), v=np.concatenate(vs))
    cache = make_cache(g)
    kp, vp = fresh_pools(g)
    d = DevBatch(fill)
    gpu_append(cache, d)
    oracle_append(kp, vp, fill)
    qn = I.store(np.concatenate(qs), g.dtype)
    got = gpu_decode(cache, to_dev(qn, g.dtype), d.bt, i32(ctx), int(ctx.max()), g)
    ref = O.decode(kp, vp, g.dtype, qn, bt, ctx, g.num_q_heads, g.scale)
    check_close(got, ref, g.dtype, "decode planted")
    for s in range(3):
        for h in range(8):
            named = int((np.rint(got[s, h, :16]).astype(int) * (1 << np.arange(16))).sum())
            assert named == tg[s][h], (s, h, named, tg[s][h])


def _decode_against_oracle(g, ctx, seed, max_ctx=None, pad_pages=0, ws_fill=None):
    """Fill every session's whole context, then decode with fresh queries; sessions of length 0 must give zeros."""
    ctx = np.asarray(ctx, np.int32)
    bt = I.deal_block_tables(I.rng_for(seed, 0), np.maximum(ctx, 1), 16, g.num_pages)
    if pad_pages > bt.shape[1]:
        bt = np.concatenate([bt, np.zeros((bt.shape[0], pad_pages - bt.shape[1]), np.int32)], axis=1)
    fill = make_batch(g, np.zeros_like(ctx), ctx, seed=seed, bt=bt, sigma_qk=1.0, sigma_v=1.0)
    cache = make_cache(g)
    kp, vp = fresh_pools(g)
    d = DevBatch(fill)
    gpu_append(cache, d)
    oracle_append(kp, vp, fill)
    qn = I.normal_values(seed, 9, 0, (len(ctx), g.num_q_heads, g.head_dim), 1.0, g.dtype)
    max_ctx = int(ctx.max()) if max_ctx is None else max_ctx
    q = to_dev(qn, g.dtype)
    if ws_fill is None:
        got = gpu_decode(cache, q, d.bt, i32(ctx), max_ctx, g)
    else:
        nbytes = B.ag_attn_decode_workspace_bytes(len(ctx), g.num_q_heads, g.head_dim, max_ctx)
        ws = torch.full((nbytes // 4,), ws_fill, dtype=torch.float32, device="cuda")
        out = torch.full_like(q, float("nan"))
        B.ag_attn_decode(cache, q, out, d.bt, i32(ctx), max_ctx, g.num_q_heads, g.scale, ws)
        torch.cuda.synchronize()
        from gpu_helpers import to_f64
        got = to_f64(out, g.dtype)
    live = np.nonzero(ctx > 0)[0]
    assert np.all(got[ctx == 0] == 0)
    ref = O.decode(kp, vp, g.dtype, qn[live], bt[live], ctx[live], g.num_q_heads, g.scale)
    check_close(got[live], ref, g.dtype, "decode")


@pytest.mark.parametrize("hq,hkv", [(8, 2), (4, 4), (16, 1)])
def test_decode_shares_that_span_many_short_sessions(hq, hkv):
    """300 sessions of 0..200 tokens: more sessions than one pass of the plan's scan covers, and every
    workgroup's share (at least 8 steps of 32 tokens) runs over several (session, head) pairs, some empty."""
    g = slm(pages=2600, hq=hq, hkv=hkv)
    rng = np.random.default_rng(41)
    ctx = rng.integers(1, 201, size=300)
    ctx[rng.integers(0, 300, size=40)] = 0
    ctx[[0, 255, 256, 299]] = [0, 33, 0, 1]            # empty sessions at the ends of the scan's passes
    _decode_against_oracle(g, ctx, seed=41)


def test_decode_bounds_far_above_the_lengths():
    """max_ctx (which sizes the grid and the workspace) 100x the longest context, on a dirty workspace."""
    g = slm(pages=600)
    _decode_against_oracle(g, [300, 17, 0, 1024, 95], seed=42, max_ctx=32768, pad_pages=2048, ws_fill=float("nan"))
    _decode_against_oracle(g, [300, 17, 0, 1024, 95], seed=42, max_ctx=32768, pad_pages=2048, ws_fill=1e30)


def test_decode_one_share_per_workgroup_boundaries():
    """Lengths chosen so that shares end exactly on, one step before and one step after a pair's end."""
    g = slm(pages=4200, hq=8, hkv=2)
    # 1024 workgroup slots: F = 2 * sum(steps); with these lengths q = 8 steps and pairs of 8, 16, 9, 7, 17 steps
    _decode_against_oracle(g, [256, 512, 288, 224, 544, 8192 + 31, 8192], seed=43)


def test_decode_is_reproducible_and_ignores_stale_workspace():
    g = slm(pages=512)
    c = I.make_decode(batch=6, lo=100, hi=1200, num_pages=512, geom=g, seed=9)
    cache = make_cache(g)
    gpu_append(cache, DevBatch(c.fill))
    d = DevBatch(c.step)
    gpu_append(cache, d)
    a = gpu_decode(cache, d.q, d.bt, d.ctx, d.max_ctx, g)
    b = gpu_decode(cache, d.q, d.bt, d.ctx, d.max_ctx, g)
    assert np.array_equal(a, b)


# ------------------------------------------------------------------ prefill / resume (matrix-core path)
@pytest.mark.parametrize("lens", [[1], [31, 32, 33], [127, 128, 129], [300, 0, 64, 200], [513]])
def test_cold_prefill_ragged(lens):
    g = slm(pages=256)
    b = make_batch(g, [0] * len(lens), lens, seed=11, sigma_qk=1.0, sigma_v=1.0)
    cache = make_cache(g)
    kp, vp = fresh_pools(g)
    got, ref = run_phase(cache, kp, vp, b, "cold")
    check_close(got, ref, g.dtype, f"cold {lens}")
    pools_match(cache, kp, vp, g.dtype)


@pytest.mark.parametrize("hq,hkv", [(4, 4), (16, 2), (3, 1)])
def test_cold_prefill_head_groupings(hq, hkv):
    g = slm(pages=128, hq=hq, hkv=hkv)
    b = make_batch(g, [0, 0], [200, 77], seed=12, sigma_qk=1.0, sigma_v=1.0)
    cache = make_cache(g)
    kp, vp = fresh_pools(g)
    got, ref = run_phase(cache, kp, vp, b, "cold")
    check_close(got, ref, g.dtype, "cold gqa")


@pytest.mark.parametrize("hq,hkv", [(4, 2), (8, 2), (16, 2), (3, 1)])
def test_long_chunks_with_head_groups_sharing_a_workgroup(hq, hkv):
    """Chunks of 512 rows and more take the 256-row workgroups; groups of 2, 4 and 8 heads share one (a wave is
    one head x 32 tokens), a group of 3 does not.  Cold, then a resume on top, ragged ends included."""
    g = slm(pages=256, hq=hq, hkv=hkv)
    bt = I.deal_block_tables(I.rng_for(14, 0), [1130, 78, 546], 16, g.num_pages)
    cold = make_batch(g, [0, 0, 0], [600, 77, 513], seed=14, bt=bt, sigma_qk=1.0, sigma_v=1.0)
    cache = make_cache(g)
    kp, vp = fresh_pools(g)
    got, ref = run_phase(cache, kp, vp, cold, "cold")
    check_close(got, ref, g.dtype, "cold, shared workgroups")
    more = make_batch(g, [600, 77, 513], [530, 1, 33], seed=14, bt=bt, stream=2, sigma_qk=1.0, sigma_v=1.0)
    got, ref = run_phase(cache, kp, vp, more, "resume")
    check_close(got, ref, g.dtype, "resume, shared workgroups")


@pytest.mark.parametrize("hq,hkv", [(8, 2), (3, 1)])
def test_resume_over_many_short_sessions(hq, hkv):
    """150 sessions with chunks of 0..40 rows on prefixes of 0..100 tokens: the workgroups' tile list is
    resolved from the lengths in passes of 64 sessions, and many sessions bring no tile at all."""
    g = slm(pages=1400, hq=hq, hkv=hkv)
    rng = np.random.default_rng(44)
    p = rng.integers(0, 101, size=150)
    n = rng.integers(0, 41, size=150)
    n[rng.integers(0, 150, size=30)] = 0
    n[[0, 63, 64, 127, 128, 149]] = [0, 40, 0, 1, 33, 0]        # around the passes' boundaries
    bt = I.deal_block_tables(I.rng_for(44, 0), np.maximum(p + n, 1), 16, g.num_pages)
    fill = make_batch(g, np.zeros_like(p), p, seed=44, bt=bt, sigma_qk=1.0, sigma_v=1.0)
    cache = make_cache(g)
    kp, vp = fresh_pools(g)
    gpu_append(cache, DevBatch(fill))
    oracle_append(kp, vp, fill)
    chunk = make_batch(g, p, n, seed=44, bt=bt, stream=2, sigma_qk=1.0, sigma_v=1.0)
    got, ref = run_phase(cache, kp, vp, chunk, "resume")
    check_close(got, ref, g.dtype, "resume, 150 sessions")


@pytest.mark.parametrize("p,n", [([5, 16, 100], [40, 1, 130]), ([64, 63, 65], [64, 65, 63]), ([700, 0], [150, 20])])
def test_resume_prefill_offsets(p, n):
    g = slm(pages=256)
    bt = I.deal_block_tables(I.rng_for(13, 0), [a + b for a, b in zip(p, n)], 16, g.num_pages)
    fill = make_batch(g, [0] * len(p), p, seed=13, bt=bt, sigma_qk=1.0, sigma_v=1.0)
    chunk = make_batch(g, p, n, seed=13, bt=bt, stream=2, sigma_qk=1.0, sigma_v=1.0)
    cache = make_cache(g)
    kp, vp = fresh_pools(g)
    gpu_append(cache, DevBatch(fill))
    oracle_append(kp, vp, fill)
    got, ref = run_phase(cache, kp, vp, chunk, "resume")
    check_close(got, ref, g.dtype, "resume")
    pools_match(cache, kp, vp, g.dtype)


def test_resume_with_zero_prefix_equals_prefill_bitwise():
    g = slm(pages=128)
    b = make_batch(g, [0, 0], [150, 90], seed=14, sigma_qk=1.0, sigma_v=1.0)
    cache = make_cache(g)
    d = DevBatch(b)
    gpu_append(cache, d)
    a = gpu_prefill(cache, d)
    r = gpu_resume(cache, d)
    assert np.array_equal(a, r)


def test_prefill_flat_logits_as_the_configs_state():
    """Values ~ N(0, 1/D) and scale 1/sqrt(D): the configs' own distribution (outputs ~ mean of V)."""
    g = slm(pages=128)
    b = make_batch(g, [0, 0], [260, 100], seed=15, sigma_qk=None, sigma_v=None)
    cache = make_cache(g)
    kp, vp = fresh_pools(g)
    got, ref = run_phase(cache, kp, vp, b, "cold")
    check_close(got, ref, g.dtype, "cold flat")


def test_prefill_very_sharp_logits():
    g = slm(pages=128)
    b = make_batch(g, [0], [400], seed=16, sigma_qk=2.0, sigma_v=1.0)    # logit std ~ 4 * sqrt(128)/sqrt(128)
    cache = make_cache(g)
    kp, vp = fresh_pools(g)
    got, ref = run_phase(cache, kp, vp, b, "cold")
    check_close(got, ref, g.dtype, "cold sharp")


def test_prefill_names_the_planted_position():
    g = slm(pages=128, hq=8, hkv=2)
    p, n = 150, 170
    l = p + n
    rng = np.random.default_rng(17)
    k = I.bf16_bits_to_f32(I.f32_to_bf16_bits(rng.standard_normal((l, 2, 128)).astype(np.float32)))
    v = np.repeat(I.position_bits(np.arange(l), 128)[:, None, :], 2, axis=1)
    tgt = np.stack([rng.integers(0, p + i + 1, size=8) for i in range(n)])
    tgt[:, 0] = p + np.arange(n)               # the diagonal itself
    tgt[:, 1] = np.maximum(p + np.arange(n) - 1, 0)
    tgt[:, 2] = 0
    q = I.planted_queries(k, tgt, 4, gain=40.0)
    bt = I.deal_block_tables(I.rng_for(17, 0), [l], 16, g.num_pages)
    fill = make_batch(g, [0], [p], seed=17, bt=bt, k=k[:p], v=v[:p])
    chunk = make_batch(g, [p], [n], seed=17, bt=bt, q=q, k=k[p:], v=v[p:])
    cache = make_cache(g)
    kp, vp = fresh_pools(g)
    gpu_append(cache, DevBatch(fill))
    oracle_append(kp, vp, fill)
    got, ref = run_phase(cache, kp, vp, chunk, "resume")
    check_close(got, ref, g.dtype, "resume planted")
    named = (np.rint(got[:, :, :16]).astype(int) * (1 << np.arange(16))).sum(-1)
    assert np.array_equal(named, tgt)


def test_decode_equals_last_row_of_prefill_on_the_gpu():
    g = slm(pages=128)
    b = make_batch(g, [0, 0], [333, 64], seed=18, sigma_qk=1.0, sigma_v=1.0)
    cache = make_cache(g)
    d = DevBatch(b)
    gpu_append(cache, d)
    full = gpu_prefill(cache, d)
    last = torch.tensor([332, 333 + 63], device="cuda")
    dec = gpu_decode(cache, d.q[last].contiguous(), d.bt, d.ctx, d.max_ctx, g)
    # two different kernels: equal to bf16 rounding, not bitwise
    assert np.abs(dec - full[last.cpu().numpy()]).max() <= 2e-2


# ------------------------------------------------------------------ errors through the ABI
def test_host_side_errors_are_reported_before_launch():
    g = slm()
    cache = make_cache(g)
    b = make_batch(g, [0], [20], seed=19)
    d = DevBatch(b)
    with pytest.raises(B.AgError) as e:
        B.ag_attn_prefill(cache, d.q, d.out, d.bt, d.new, d.cu, d.total, d.max_new, 7, g.scale)
    assert e.value.status == B.AG_ERR_INVALID_ARG
    with pytest.raises(B.AgError) as e:
        B.ag_attn_resume(cache, d.q, d.out, d.bt, d.prefix, d.new, d.cu, d.total, d.max_new,
                         16 * d.bt.shape[1] + 1, g.num_q_heads, g.scale)
    assert e.value.status == B.AG_ERR_INVALID_ARG
    ws = torch.empty(4, dtype=torch.float32, device="cuda")
    with pytest.raises(B.AgError) as e:
        B.ag_attn_decode(cache, d.q[:1], d.out[:1], d.bt, d.ctx, 20, g.num_q_heads, g.scale, ws)
    assert e.value.status == B.AG_ERR_WORKSPACE
    bad = d.bt.clone()
    bad[0, 0] = g.num_pages
    with pytest.raises(B.AgError):
        B.ag_debug_validate(cache, bad, d.prefix, d.new, d.cu)
    torch.cuda.synchronize()


# ------------------------------------------------------------------ other page sizes and head dims (general kernels)
@pytest.mark.parametrize("ps,d,dtype", [(1, 64, I.F32), (4, 64, I.BF16), (8, 128, I.BF16), (32, 64, I.F32),
                                        (64, 128, I.BF16), (16, 256, I.BF16), (16, 8, I.F32)])
def test_general_kernels_cover_other_page_sizes_and_head_dims(ps, d, dtype):
    """Pool layouts depend on the page size (chunks of 8 keys from 16 slots up, plain below): append must stay
    bit-exact and all three classes must match the oracle for every supported combination."""
    lens_a, lens_b = [37, 5, 64], [20, 70, 1]
    pages = sum((a + b + 1 + ps - 1) // ps for a, b in zip(lens_a, lens_b)) + 3
    g = I.Geometry(4, 2, d, ps, pages, dtype)
    bt = I.deal_block_tables(I.rng_for(23, 0), [a + b + 1 for a, b in zip(lens_a, lens_b)], ps, pages)
    cold = make_batch(g, [0, 0, 0], lens_a, seed=23, bt=bt)
    res = make_batch(g, lens_a, lens_b, seed=23, bt=bt, stream=2)
    dec = make_batch(g, [a + b for a, b in zip(lens_a, lens_b)], [1, 1, 1], seed=23, bt=bt, stream=3)
    cache = make_cache(g)
    kp, vp = fresh_pools(g)
    for b, kind in [(cold, "cold"), (res, "resume"), (dec, "decode")]:
        got, ref = run_phase(cache, kp, vp, b, kind)
        check_close(got, ref, dtype, f"{kind} ps={ps} d={d}")
    pools_match(cache, kp, vp, dtype)


def test_decode_with_more_than_16_heads_per_kv_head_uses_the_general_kernel():
    g = I.Geometry(32, 1, 128, 16, 64, I.BF16)
    c = I.make_decode(batch=3, lo=20, hi=300, num_pages=64, geom=g, seed=29, sigma_qk=1.0, sigma_v=1.0)
    cache = make_cache(g)
    kp, vp = fresh_pools(g)
    gpu_append(cache, DevBatch(c.fill))
    oracle_append(kp, vp, c.fill)
    got, ref = run_phase(cache, kp, vp, c.step, "decode")
    check_close(got, ref, g.dtype, "decode G=32")


def test_long_context_decode_many_partials():
    """One session of 40000 tokens: cut into the shortest shares (157 partials per head), page ids far apart."""
    g = slm(pages=2600, hq=8, hkv=2)
    ctx = np.array([40000, 129], np.int32)
    bt = I.deal_block_tables(I.rng_for(31, 0), ctx, 16, g.num_pages)
    fill = make_batch(g, [0, 0], ctx - 1, seed=31, bt=bt, sigma_qk=1.0, sigma_v=1.0)
    step = make_batch(g, ctx - 1, [1, 1], seed=31, bt=bt, stream=2, sigma_qk=1.0, sigma_v=1.0)
    cache = make_cache(g)
    kp, vp = fresh_pools(g)
    gpu_append(cache, DevBatch(fill))
    oracle_append(kp, vp, fill)
    got, ref = run_phase(cache, kp, vp, step, "decode")
    check_close(got, ref, g.dtype, "decode 40000")
