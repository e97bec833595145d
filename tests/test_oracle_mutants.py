"""Does the pin suite have teeth?  Each case plants one plausible mistake in a
COPY of the oracle's C source (the committed source is untouched), builds it,
and checks that at least one pin from test_oracle_pins fails against it.
The mistakes: a dropped scale, an off-by-one causal mask, prefix ignored by the
mask, the wrong GQA mapping, a wrong slot/page index, K and V pools swapped, a
missing normalisation, and an append that lands one slot off.
CPU only.
"""
import os

import numpy as np
import pytest

from brute_force import dense_attention
from helpers import fresh_pools, make_batch, oracle_append, oracle_attn
from oracle import build as OB
from oracle import oracle as O
from paper_2603_10342_amd import inputs as I

MUTANTS = {
    "scale_dropped": ("x[j] = scale * dot;", "x[j] = dot;"),
    "mask_excludes_self": ("for (int64_t j = 0; j <= pos; ++j) {\n        const int64_t lp", "for (int64_t j = 0; j < pos + (pos == 0); ++j) {\n        const int64_t lp"),
    "mask_ignores_prefix": ("(int64_t)prefix_lens[s] + i, h / G, scale, x,", "(int64_t)i, h / G, scale, x,"),
    "gqa_interleaved": ("(int64_t)prefix_lens[s] + i, h / G, scale, x,", "(int64_t)prefix_lens[s] + i, h % c->num_kv_heads, scale, x,"),
    "slot_uses_page_index": ("const size_t ko = pool_offset(c, page, g, (int)(j % ps));", "const size_t ko = pool_offset(c, page, g, (int)((j + 1) % ps));"),
    "v_read_from_k_pool": ("out[d] += w * load_elem(c->v_pool, vo + d, dt);", "out[d] += w * load_elem(c->k_pool, vo + d, dt);"),
    "not_normalised": ("for (int d = 0; d < D; ++d) out[d] /= Z;", "(void)Z;"),
    "append_off_by_one_slot": ("const int slot = (int)(pos % c->page_size);", "const int slot = (int)((pos + 1) % c->page_size);"),
    "append_ignores_prefix": ("const int64_t pos = (int64_t)prefix_lens[s] + i;", "const int64_t pos = (int64_t)i;"),
    "pool_layout_slot_major": ("return (((size_t)page * c->num_kv_heads + g) * c->page_size + slot) * (size_t)c->head_dim;",
                               "return (((size_t)page * c->page_size + slot) * c->num_kv_heads + g) * (size_t)c->head_dim;"),
}


def as64(a):
    return I.stored_to_f64(a, I.F32)


def pins(lib):
    """A condensed run of the pin suite against `lib`; returns the names of the pins that fail."""
    failed = []
    g = I.Geometry(4, 2, 16, 16, 32, I.F32)

    def check(name, cond):
        if not cond:
            failed.append(name)

    # brute force, cold + resume
    try:
        bt = I.deal_block_tables(I.rng_for(1, 0), [50, 37], 16, 32)
        fill = make_batch(g, [0, 0], [30, 20], seed=1, bt=bt)
        chunk = make_batch(g, [30, 20], [20, 17], seed=1, bt=bt, stream=2)
        kp, vp = fresh_pools(g)
        oracle_append(kp, vp, fill, lib=lib)
        cold = oracle_attn(kp, vp, fill, lib=lib)
        oracle_append(kp, vp, chunk, lib=lib)
        res = oracle_attn(kp, vp, chunk, lib=lib)
        ok_c = ok_r = True
        for s in range(2):
            fs = slice(int(fill.cu_new[s]), int(fill.cu_new[s + 1]))
            cs = slice(int(chunk.cu_new[s]), int(chunk.cu_new[s + 1]))
            ref = dense_attention(as64(fill.q[fs]), as64(fill.k_new[fs]), as64(fill.v_new[fs]), 0, g.scale)
            ok_c &= bool(np.allclose(cold[fs], ref, rtol=0, atol=1e-12))
            k = np.concatenate([as64(fill.k_new[fs]), as64(chunk.k_new[cs])])
            v = np.concatenate([as64(fill.v_new[fs]), as64(chunk.v_new[cs])])
            ref = dense_attention(as64(chunk.q[cs]), k, v, int(fill.new_lens[s]), g.scale)
            ok_r &= bool(np.allclose(res[cs], ref, rtol=0, atol=1e-12))
        check("brute_cold", ok_c)
        check("brute_resume", ok_r)
        # dictionary model of the append
        ok_d = True
        for b in (fill, chunk):
            for s in range(2):
                for i in range(int(b.new_lens[s])):
                    pos = int(b.prefix_lens[s]) + i
                    for h in range(2):
                        ok_d &= bool(np.array_equal(kp[bt[s, pos // 16], h, pos % 16], b.k_new[b.cu_new[s] + i, h]))
                        ok_d &= bool(np.array_equal(vp[bt[s, pos // 16], h, pos % 16], b.v_new[b.cu_new[s] + i, h]))
        check("append_dictionary", ok_d)
    except O.OracleError:
        failed.append("raised")
    return failed


def test_unmutated_oracle_passes_the_condensed_pins():
    assert pins(O.lib()) == []


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_planted_mistake_is_caught(name, tmp_path):
    old, new = MUTANTS[name]
    src = open(OB.SRC).read()
    assert src.count(old) == 1, f"mutation site for {name} not found exactly once"
    msrc = tmp_path / "mutant.c"
    msrc.write_text(src.replace(old, new))
    mlib = OB.build(force=True, src=str(msrc), lib=str(tmp_path / f"libmut_{name}.so"))
    failed = pins(O.lib(mlib))
    assert failed, f"no pin noticed the planted mistake '{name}'"
