"""Shared test plumbing: run a Batch through the oracle; gather a session's
logical K/V out of the pools.  No attention arithmetic here."""
import numpy as np

from oracle import oracle as O
from paper_2603_10342_amd import inputs as I


def fresh_pools(geom, poison=True):
    mk = I.nan_pool if poison else I.zero_pool
    return mk(geom.pool_shape, geom.dtype), mk(geom.pool_shape, geom.dtype)


def oracle_append(kp, vp, b, lib=None):
    O.kv_append(kp, vp, b.geom.dtype, b.k_new, b.v_new, b.block_tables, b.prefix_lens, b.new_lens, b.cu_new,
                _lib=lib)


def oracle_attn(kp, vp, b, scale=None, rows=None, lib=None):
    g = b.geom
    return O.attn(kp, vp, g.dtype, b.q, b.block_tables, b.prefix_lens, b.new_lens, b.cu_new, g.num_q_heads,
                  g.scale if scale is None else scale, rows=rows, _lib=lib)


def make_batch(geom, prefix_lens, new_lens, seed, q=None, k=None, v=None, sigma_qk=1.0, sigma_v=1.0, bt=None,
               stream=1):
    """Small batch with its own block table; optional fp32 overrides for q/k/v ([T,H,D])."""
    prefix_lens = np.asarray(prefix_lens, np.int32)
    new_lens = np.asarray(new_lens, np.int32)
    if bt is None:
        bt = I.deal_block_tables(I.rng_for(seed, 0), prefix_lens + new_lens, geom.page_size, geom.num_pages)
    b = I.draw_batch(geom, bt, prefix_lens, new_lens, seed, stream, sigma_qk=sigma_qk, sigma_v=sigma_v)
    if q is not None:
        b.q = I.store(np.asarray(q, np.float32), geom.dtype)
    if k is not None:
        b.k_new = I.store(np.asarray(k, np.float32), geom.dtype)
    if v is not None:
        b.v_new = I.store(np.asarray(v, np.float32), geom.dtype)
    return b


def session_slice(b, s):
    return slice(int(b.cu_new[s]), int(b.cu_new[s + 1]))


def rel_fro(a, ref):
    a = np.asarray(a, np.float64)
    ref = np.asarray(ref, np.float64)
    return float(np.linalg.norm(a - ref) / max(np.linalg.norm(ref), 1e-300))
