"""Pins for the CPU oracle: everything here is fixed by mathematics or by the
paper's definition of the three request classes (Sec. I; Sec. II-A; Fig. 1),
none of it by the oracle itself.  The paper prints no numeric value for the
attention path, so there is no golden number to compare with; see
tests/golden/README.md.

Runs on the CPU only.
"""
import numpy as np
import pytest

from brute_force import dense_attention
from helpers import fresh_pools, make_batch, oracle_append, oracle_attn, session_slice
from oracle import oracle as O
from paper_2603_10342_amd import inputs as I

TIGHT = 1e-12


def geom(hq=4, hkv=2, d=16, ps=16, pages=32, dtype=I.F32):
    return I.Geometry(hq, hkv, d, ps, pages, dtype)


def run(b, poison=True, scale=None):
    kp, vp = fresh_pools(b.geom, poison)
    oracle_append(kp, vp, b)
    return oracle_attn(kp, vp, b, scale=scale)


def as64(a, dtype):
    return I.stored_to_f64(a, dtype)


# ---------------------------------------------------------------- brute force
@pytest.mark.parametrize("hq,hkv", [(1, 1), (4, 2), (4, 1), (4, 4)])
@pytest.mark.parametrize("d", [1, 8, 16])
@pytest.mark.parametrize("n", [1, 2, 15, 16, 17, 33, 64])
@pytest.mark.parametrize("dtype", [I.F32, I.BF16])
def test_cold_matches_dense_brute_force(hq, hkv, d, n, dtype):
    g = geom(hq, hkv, d, dtype=dtype)
    b = make_batch(g, [0, 0], [n, max(1, n - 1)], seed=11 + n + d)
    out = run(b)
    for s in range(b.batch):
        sl = session_slice(b, s)
        ref = dense_attention(as64(b.q[sl], dtype), as64(b.k_new[sl], dtype), as64(b.v_new[sl], dtype), 0, g.scale)
        np.testing.assert_allclose(out[sl], ref, rtol=0, atol=TIGHT)


@pytest.mark.parametrize("p,n", [(1, 1), (5, 3), (16, 16), (17, 1), (31, 2), (32, 33), (40, 24)])
def test_resume_matches_dense_brute_force(p, n):
    g = geom(4, 2, 8)
    bt = I.deal_block_tables(I.rng_for(5, 0), [p + n], g.page_size, g.num_pages)
    fill = make_batch(g, [0], [p], seed=5, bt=bt)
    chunk = make_batch(g, [p], [n], seed=5, bt=bt, stream=2)
    kp, vp = fresh_pools(g)
    oracle_append(kp, vp, fill)
    oracle_append(kp, vp, chunk)
    out = oracle_attn(kp, vp, chunk)
    k = np.concatenate([as64(fill.k_new, g.dtype), as64(chunk.k_new, g.dtype)])
    v = np.concatenate([as64(fill.v_new, g.dtype), as64(chunk.v_new, g.dtype)])
    ref = dense_attention(as64(chunk.q, g.dtype), k, v, p, g.scale)
    np.testing.assert_allclose(out, ref, rtol=0, atol=TIGHT)


def test_explicit_scale_is_used():
    g = geom()
    b = make_batch(g, [0], [20], seed=3)
    out = run(b, scale=0.37)
    ref = dense_attention(as64(b.q, g.dtype), as64(b.k_new, g.dtype), as64(b.v_new, g.dtype), 0, 0.37)
    np.testing.assert_allclose(out, ref, rtol=0, atol=TIGHT)
    assert np.abs(out - run(b)).max() > 1e-3


# ---------------------------------------------------------------- closed forms
def running_mean(v):
    return np.cumsum(v, axis=0) / np.arange(1, len(v) + 1)[:, None, None]


def test_constant_keys_give_running_mean_of_v():
    g = geom()
    n = 50
    rng = np.random.default_rng(0)
    k = np.tile(rng.standard_normal((1, g.num_kv_heads, g.head_dim)), (n, 1, 1))
    b = make_batch(g, [0], [n], seed=1, k=k)
    out = run(b)
    v = np.repeat(as64(b.v_new, g.dtype), g.num_q_heads // g.num_kv_heads, axis=1)
    np.testing.assert_allclose(out, running_mean(v), rtol=0, atol=TIGHT)


def test_zero_queries_give_running_mean_of_v():
    g = geom()
    n = 37
    b = make_batch(g, [0], [n], seed=2, q=np.zeros((n, g.num_q_heads, g.head_dim)))
    out = run(b)
    v = np.repeat(as64(b.v_new, g.dtype), 2, axis=1)
    np.testing.assert_allclose(out, running_mean(v), rtol=0, atol=TIGHT)


def test_first_row_of_a_cold_prefill_returns_v0():
    g = geom()
    b = make_batch(g, [0, 0], [9, 4], seed=4)
    out = run(b)
    for s in range(2):
        t0 = int(b.cu_new[s])
        v0 = np.repeat(as64(b.v_new[t0], g.dtype), 2, axis=0)
        np.testing.assert_array_equal(out[t0], v0)


def test_two_keys_give_the_logistic_mixture():
    g = geom(1, 1, 4)
    q = np.array([[[0, 0, 0, 0]], [[1.0, -2.0, 0.5, 3.0]]])
    k = np.array([[[0.5, 1.0, -1.0, 0.25]], [[-1.5, 0.5, 2.0, 1.0]]])
    v = np.array([[[1.0, 2.0, 3.0, 4.0]], [[-4.0, 0.0, 8.0, 0.5]]])
    b = make_batch(g, [0], [2], seed=0, q=q, k=k, v=v)
    out = run(b)
    a = g.scale * float(q[1, 0] @ k[0, 0])
    c = g.scale * float(q[1, 0] @ k[1, 0])
    sig = 1.0 / (1.0 + np.exp(-(a - c)))
    np.testing.assert_allclose(out[1, 0], sig * v[0, 0] + (1 - sig) * v[1, 0], rtol=0, atol=TIGHT)


def test_one_dominant_key_selects_its_value():
    """Sharp softmax: a planted key whose logit is >= 40 above every other returns its V row."""
    d = 64
    g = geom(4, 2, d)
    n = 40
    rng = np.random.default_rng(7)
    k = rng.standard_normal((n, 2, d))
    k = (k / np.linalg.norm(k, axis=-1, keepdims=True) * np.sqrt(d)).astype(np.float32)
    cos = np.einsum("ihd,jhd->hij", k, k) / d
    assert np.max(cos - 2 * np.eye(n)[None]) < 0.5           # so the margin below is >= 40
    targets = np.stack([rng.integers(0, i + 1, size=4) for i in range(n)])
    q = I.planted_queries(k, targets, 2, gain=80.0)
    vbits = np.repeat(I.position_bits(np.arange(n), d)[:, None, :], 2, axis=1)
    b = make_batch(g, [0], [n], seed=0, q=q, k=k, v=vbits)
    out = run(b)
    for i in range(n):
        for h in range(4):
            got = np.rint(out[i, h]).astype(int)
            assert (got[:16] * (1 << np.arange(16))).sum() == targets[i, h], (i, h)
            assert np.abs(out[i, h] - got).max() < 1e-9


# ---------------------------------------------------------------- invariants
def test_output_is_a_convex_combination_of_visible_values():
    g = geom()
    b = make_batch(g, [0], [45], seed=8, sigma_qk=3.0)
    out = run(b)
    v = np.repeat(as64(b.v_new, g.dtype), 2, axis=1)
    lo = np.minimum.accumulate(v, axis=0)
    hi = np.maximum.accumulate(v, axis=0)
    assert np.all(out >= lo - 1e-12) and np.all(out <= hi + 1e-12)


def test_linear_in_v():
    g = geom()
    b1 = make_batch(g, [0], [30], seed=9)
    rng = np.random.default_rng(1)
    v2 = rng.standard_normal(b1.v_new.shape).astype(np.float32)
    b2 = make_batch(g, [0], [30], seed=9, v=v2)
    # exactly representable sum: round both to few mantissa bits first
    va = np.round(as64(b1.v_new, g.dtype) * 256) / 256
    vb = np.round(v2.astype(np.float64) * 256) / 256
    ba = make_batch(g, [0], [30], seed=9, v=va)
    bb = make_batch(g, [0], [30], seed=9, v=vb)
    bs = make_batch(g, [0], [30], seed=9, v=va + vb)
    np.testing.assert_allclose(run(bs), run(ba) + run(bb), rtol=0, atol=TIGHT)
    assert np.abs(run(b2) - run(b1)).max() > 1e-2


def test_adding_one_vector_to_every_key_changes_nothing():
    g = geom()
    n = 33
    b = make_batch(g, [0], [n], seed=10)
    k = np.round(as64(b.k_new, g.dtype) * 64) / 64
    shift = np.round(np.random.default_rng(2).standard_normal((1, g.num_kv_heads, g.head_dim)) * 64) / 64
    b0 = make_batch(g, [0], [n], seed=10, k=k)
    b1 = make_batch(g, [0], [n], seed=10, k=k + shift)
    np.testing.assert_allclose(run(b1), run(b0), rtol=0, atol=1e-11)


def test_permuting_prefix_keys_with_their_values_changes_nothing():
    g = geom()
    p, n = 40, 6
    fill = make_batch(g, [0], [p], seed=12)
    bt = I.deal_block_tables(I.rng_for(12, 0), [p + n], g.page_size, g.num_pages)
    fill.block_tables = bt
    chunk = make_batch(g, [p], [n], seed=12, bt=bt, stream=2)

    def go(perm):
        f = make_batch(g, [0], [p], seed=12, bt=bt)
        f.k_new = fill.k_new[perm].copy()
        f.v_new = fill.v_new[perm].copy()
        kp, vp = fresh_pools(g)
        oracle_append(kp, vp, f)
        oracle_append(kp, vp, chunk)
        return oracle_attn(kp, vp, chunk)

    perm = np.random.default_rng(3).permutation(p)
    np.testing.assert_allclose(go(perm), go(np.arange(p)), rtol=0, atol=TIGHT)


# ------------------------------------------- equalities between the classes
def _three_phase(g, p, n, seed):
    """cold(p+n) in one go, versus cold(p) then resume(n), on the same tokens."""
    whole = make_batch(g, [0, 0], [p + n, p + n], seed=seed)
    kp, vp = fresh_pools(g)
    oracle_append(kp, vp, whole)
    cold = oracle_attn(kp, vp, whole)
    return whole, cold


@pytest.mark.parametrize("p,n", [(16, 16), (20, 13), (1, 30), (47, 1)])
def test_resume_equals_tail_rows_of_cold_prefill(p, n):
    g = geom(4, 2, 16, pages=64)
    whole, cold = _three_phase(g, p, n, seed=21)
    bt = whole.block_tables
    kp, vp = fresh_pools(g)
    parts = []
    for s in range(2):
        parts.append(session_slice(whole, s))
    first = np.concatenate([np.arange(sl.start, sl.start + p) for sl in parts])
    last = np.concatenate([np.arange(sl.start + p, sl.stop) for sl in parts])
    fill = I.Batch(g, bt, [0, 0], [p, p], whole.q[first], whole.k_new[first], whole.v_new[first])
    chunk = I.Batch(g, bt, [p, p], [n, n], whole.q[last], whole.k_new[last], whole.v_new[last])
    oracle_append(kp, vp, fill)
    head = oracle_attn(kp, vp, fill)
    oracle_append(kp, vp, chunk)
    tail = oracle_attn(kp, vp, chunk)
    np.testing.assert_allclose(tail, cold[last], rtol=0, atol=TIGHT)
    np.testing.assert_allclose(head, cold[first], rtol=0, atol=TIGHT)


def test_decode_equals_last_row_of_prefill_and_resume_of_one():
    g = geom(4, 2, 16, pages=64)
    lens = [37, 48]
    whole = make_batch(g, [0, 0], lens, seed=22)
    kp, vp = fresh_pools(g)
    oracle_append(kp, vp, whole)
    cold = oracle_attn(kp, vp, whole)
    last = np.array([int(whole.cu_new[s + 1]) - 1 for s in range(2)])
    dec = O.decode(kp, vp, g.dtype, np.ascontiguousarray(whole.q[last]), whole.block_tables, lens,
                   g.num_q_heads, g.scale)
    np.testing.assert_allclose(dec, cold[last], rtol=0, atol=TIGHT)
    one = I.Batch(g, whole.block_tables, [l - 1 for l in lens], [1, 1], np.ascontiguousarray(whole.q[last]),
                  np.ascontiguousarray(whole.k_new[last]), np.ascontiguousarray(whole.v_new[last]))
    np.testing.assert_allclose(oracle_attn(kp, vp, one), dec, rtol=0, atol=0)


def test_resume_with_empty_prefix_is_cold():
    g = geom()
    b = make_batch(g, [0], [25], seed=23)
    ref = dense_attention(as64(b.q, g.dtype), as64(b.k_new, g.dtype), as64(b.v_new, g.dtype), 0, g.scale)
    np.testing.assert_allclose(run(b), ref, rtol=0, atol=TIGHT)


def test_row_subset_equals_full_result():
    g = geom()
    b = make_batch(g, [0, 0], [30, 18], seed=24)
    kp, vp = fresh_pools(g)
    oracle_append(kp, vp, b)
    full = oracle_attn(kp, vp, b)
    rs = np.array([1, 0, 0, 1], np.int32)
    ri = np.array([17, 0, 29, 3], np.int32)
    sub = oracle_attn(kp, vp, b, rows=(rs, ri))
    for r in range(4):
        np.testing.assert_array_equal(sub[r], full[int(b.cu_new[rs[r]]) + ri[r]])


# ---------------------------------------------------------------- paging
@pytest.mark.parametrize("dtype", [I.F32, I.BF16])
def test_append_matches_a_dictionary_model(dtype):
    g = geom(4, 2, 8, ps=16, pages=40, dtype=dtype)
    lens_a = [5, 16, 17, 0]
    lens_b = [12, 1, 30, 7]          # crosses page boundaries, starts mid-page, starts on a boundary
    bt = I.deal_block_tables(I.rng_for(31, 0), [a + b for a, b in zip(lens_a, lens_b)], 16, 40)
    first = make_batch(g, [0] * 4, lens_a, seed=31, bt=bt)
    second = make_batch(g, lens_a, lens_b, seed=31, bt=bt, stream=2)
    kp, vp = fresh_pools(g)
    sentinel_k, sentinel_v = kp.copy(), vp.copy()
    oracle_append(kp, vp, first)
    oracle_append(kp, vp, second)
    model = {}
    for b in (first, second):
        for s in range(4):
            for i in range(int(b.new_lens[s])):
                for h in range(2):
                    model[(s, int(b.prefix_lens[s]) + i, h)] = (b.k_new[b.cu_new[s] + i, h], b.v_new[b.cu_new[s] + i, h])
    written = np.zeros(kp.shape[:3], bool)
    for (s, pos, h), (kr, vr) in model.items():
        page, slot = bt[s, pos // 16], pos % 16
        np.testing.assert_array_equal(kp[page, h, slot], kr)
        np.testing.assert_array_equal(vp[page, h, slot], vr)
        written[page, h, slot] = True
    # nothing else was touched (bit compare: NaN patterns included)
    raw = np.uint32 if dtype == I.F32 else np.uint16
    assert np.array_equal(kp.view(raw)[~written], sentinel_k.view(raw)[~written])
    assert np.array_equal(vp.view(raw)[~written], sentinel_v.view(raw)[~written])


def test_physical_page_permutation_leaves_output_bit_identical():
    g = geom(4, 2, 16, pages=48)
    lens = [33, 47]
    outs = []
    for seed in (41, 42):
        bt = I.deal_block_tables(I.rng_for(seed, 0), lens, 16, 48)
        b = make_batch(g, [0, 0], lens, seed=40, bt=bt)
        outs.append(run(b))
    np.testing.assert_array_equal(outs[0], outs[1])


def test_identity_block_table_reads_a_contiguous_cache():
    g = geom(2, 1, 8, pages=4)
    n = 50
    bt = np.arange(4, dtype=np.int32)[None, :]
    b = make_batch(g, [0], [n], seed=43, bt=bt)
    kp, vp = fresh_pools(g)
    oracle_append(kp, vp, b)
    # [page][1 head][slot][d] with identity pages == plain [token][d]
    np.testing.assert_array_equal(kp.reshape(-1, 8)[:n], b.k_new[:, 0])
    out = oracle_attn(kp, vp, b)
    ref = dense_attention(as64(b.q, g.dtype), as64(b.k_new, g.dtype), as64(b.v_new, g.dtype), 0, g.scale)
    np.testing.assert_allclose(out, ref, rtol=0, atol=TIGHT)


@pytest.mark.parametrize("l", [1, 15, 16, 17, 31, 32, 33])
def test_boundary_lengths_never_read_a_poisoned_slot(l):
    g = geom(4, 2, 8)
    b = make_batch(g, [0], [l], seed=44 + l)
    out = run(b, poison=True)
    assert np.isfinite(out).all()
    ref = dense_attention(as64(b.q, g.dtype), as64(b.k_new, g.dtype), as64(b.v_new, g.dtype), 0, g.scale)
    np.testing.assert_allclose(out, ref, rtol=0, atol=TIGHT)


def test_two_sessions_may_read_the_same_physical_pages():
    g = geom(4, 2, 8)
    b = make_batch(g, [0], [40], seed=45)
    kp, vp = fresh_pools(g)
    oracle_append(kp, vp, b)
    bt2 = np.concatenate([b.block_tables, b.block_tables])
    q2 = np.concatenate([b.q[-1:], b.q[-1:]])
    dec = O.decode(kp, vp, g.dtype, q2, bt2, [40, 25], g.num_q_heads, g.scale)
    full = oracle_attn(kp, vp, b)
    np.testing.assert_array_equal(dec[0], full[-1])
    assert np.isfinite(dec[1]).all()


def test_out_of_range_page_is_an_error_not_a_read():
    g = geom()
    b = make_batch(g, [0], [20], seed=46)
    kp, vp = fresh_pools(g)
    oracle_append(kp, vp, b)
    bad = b.block_tables.copy()
    bad[0, 1] = g.num_pages
    with pytest.raises(O.OracleError):
        O.attn(kp, vp, g.dtype, b.q, bad, b.prefix_lens, b.new_lens, b.cu_new, g.num_q_heads, g.scale)
    with pytest.raises(O.OracleError):
        O.kv_append(kp, vp, g.dtype, b.k_new, b.v_new, bad, b.prefix_lens, b.new_lens, b.cu_new)


# ---------------------------------------------------------------- GQA
def test_heads_of_one_group_with_equal_queries_agree_and_groups_differ():
    g = geom(4, 2, 16)
    n = 20
    rng = np.random.default_rng(5)
    q = np.repeat(rng.standard_normal((n, 1, 16)), 4, axis=1)
    b = make_batch(g, [0], [n], seed=50, q=q)
    out = run(b)
    np.testing.assert_array_equal(out[:, 0], out[:, 1])
    np.testing.assert_array_equal(out[:, 2], out[:, 3])
    assert np.abs(out[:, 1] - out[:, 2]).max() > 1e-3


def test_bf16_inputs_are_widened_exactly():
    g32 = geom(dtype=I.F32)
    g16 = geom(dtype=I.BF16)
    b16 = make_batch(g16, [0], [30], seed=51)
    b32 = make_batch(g32, [0], [30], seed=51, q=I.bf16_bits_to_f32(b16.q), k=I.bf16_bits_to_f32(b16.k_new),
                     v=I.bf16_bits_to_f32(b16.v_new), bt=b16.block_tables)
    np.testing.assert_array_equal(run(b16), run(b32))


# ------------------------------------------------ the tiny benchmark config
def test_tiny_config_phases_agree_with_one_cold_prefill_of_everything():
    """Config 1's cold(256) -> resume(32) -> 16 decode steps, against a single
    cold prefill over all 304 tokens of each session."""
    c = I.make_tiny()
    g = c.geom
    kp, vp = fresh_pools(g)
    outs = []
    for b in [c.cold, c.resume] + c.decode_steps:
        oracle_append(kp, vp, b)
        outs.append(oracle_attn(kp, vp, b))
    assert np.isfinite(np.concatenate(outs)).all()
    per_session = [np.concatenate([o[session_slice(b, s)] for o, b in zip(outs, [c.cold, c.resume] + c.decode_steps)])
                   for s in range(2)]
    for s in range(2):
        parts = [c.cold, c.resume] + c.decode_steps
        q = np.concatenate([as64(b.q[session_slice(b, s)], g.dtype) for b in parts])
        k = np.concatenate([as64(b.k_new[session_slice(b, s)], g.dtype) for b in parts])
        v = np.concatenate([as64(b.v_new[session_slice(b, s)], g.dtype) for b in parts])
        ref = dense_attention(q, k, v, 0, g.scale)
        np.testing.assert_allclose(per_session[s], ref, rtol=0, atol=TIGHT)
