"""Seeded synthetic inputs for the paged-KV attention path.

This module only *draws data*: session lengths, block tables, and Q/K/V values
in the storage dtype.  It contains none of the attention arithmetic, imports
neither the HIP binding nor the CPU oracle, and is the one module both of them
are fed from.

The workloads stand in for the agent sessions the paper measures on (cold
prefill of a long system prompt, resume prefill of an appended tool output,
short decode; Sec. II-A/II-B and Table I): the paper's sessions come from a
public tool-use benchmark that is not reproduced here, so lengths are drawn
from the uniform ranges of the five benchmark configurations instead.

Storage conventions
  * fp32 values are numpy float32.
  * bf16 values are numpy uint16 holding the upper 16 bits of the fp32 value
    after round-to-nearest-even.  Both consumers upcast those stored bits
    exactly, so input quantisation is never part of a measured error.
  * Token-major activations: Q [T, Hq, D], K_new / V_new [T, Hkv, D], sessions
    concatenated, cu_new[B+1] the offsets.
  * KV pools: [num_pages, Hkv, page_size, D], K and V separately.
  * Block tables: int32 [B, max_pages]; unused entries are -1.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

F32 = 0
BF16 = 1

BASE_SEED = 10342 * 100


# ----------------------------------------------------------------------------
# storage-dtype helpers (format conversion only)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bits."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    nan = np.isnan(x)
    rounded = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) >> np.uint32(16)
    out = rounded.astype(np.uint16)
    if nan.any():
        out[nan] = np.uint16(0x7FC0)
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact upcast of bfloat16 bits (uint16) to float32."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def store(x: np.ndarray, dtype: int) -> np.ndarray:
    """fp32 array -> array in storage dtype (float32, or uint16 bf16 bits)."""
    if dtype == F32:
        return np.ascontiguousarray(x, dtype=np.float32)
    return f32_to_bf16_bits(x)


def stored_to_f64(a: np.ndarray, dtype: int) -> np.ndarray:
    """Exact upcast of a stored array to float64."""
    if dtype == F32:
        return np.asarray(a, dtype=np.float32).astype(np.float64)
    return bf16_bits_to_f32(a).astype(np.float64)


def np_storage_dtype(dtype: int):
    return np.float32 if dtype == F32 else np.uint16


def nan_pool(shape, dtype: int) -> np.ndarray:
    """A pool in which every slot is NaN: any read of an unwritten slot shows."""
    if dtype == F32:
        return np.full(shape, np.nan, dtype=np.float32)
    return np.full(shape, 0x7FC0, dtype=np.uint16)


def zero_pool(shape, dtype: int) -> np.ndarray:
    return np.zeros(shape, dtype=np_storage_dtype(dtype))


# ----------------------------------------------------------------------------
# counter-based random source
# ----------------------------------------------------------------------------
def rng_for(seed: int, stream: int = 0) -> np.random.Generator:
    """Philox is counter-based: (seed, stream) fully determines the sequence."""
    return np.random.Generator(np.random.Philox(key=[np.uint64(seed), np.uint64(stream)]))


_CHUNK = 1 << 22


def normal_values(seed: int, stream: int, tensor: int, shape, sigma: float, dtype: int) -> np.ndarray:
    """N(0, sigma^2) drawn in fp32, rounded once to the storage dtype.

    The array is cut into fixed chunks of 2^22 values; chunk c of tensor
    `tensor` is drawn from the Philox key (seed, stream * 2^40 + tensor * 2^32 + c),
    so the bytes do not depend on how many host threads fill it.
    """
    from concurrent.futures import ThreadPoolExecutor
    import os

    n = int(np.prod(shape))
    out = np.empty(n, dtype=np_storage_dtype(dtype))

    def fill(c):
        lo = c * _CHUNK
        hi = min(n, lo + _CHUNK)
        rng = rng_for(seed, (stream << 40) + (tensor << 32) + c)
        x = rng.standard_normal(hi - lo, dtype=np.float32)
        if sigma != 1.0:
            x *= np.float32(sigma)
        out[lo:hi] = store(x, dtype)

    chunks = range((n + _CHUNK - 1) // _CHUNK)
    workers = min(len(chunks), max(1, min(16, os.cpu_count() or 1)))
    if workers <= 1:
        for c in chunks:
            fill(c)
    else:
        with ThreadPoolExecutor(workers) as ex:
            list(ex.map(fill, chunks))
    return out.reshape(shape)


# ----------------------------------------------------------------------------
# block tables
# ----------------------------------------------------------------------------
def pages_for(length: int, page_size: int) -> int:
    return (int(length) + page_size - 1) // page_size


def deal_block_tables(rng: np.random.Generator, capacities, page_size: int, num_pages: int,
                      max_pages: Optional[int] = None) -> np.ndarray:
    """One random permutation of the physical pages, dealt to sessions in order.

    capacities[s] is the largest context session s will ever hold; it gets
    ceil(capacity / page_size) pages, disjoint from every other session's.
    """
    need = [pages_for(c, page_size) for c in capacities]
    if sum(need) > num_pages:
        raise ValueError(f"pool of {num_pages} pages cannot hold {sum(need)} pages")
    width = max(need + [1]) if max_pages is None else max_pages
    if width < max(need + [0]):
        raise ValueError("max_pages smaller than the longest session")
    perm = rng.permutation(num_pages).astype(np.int32)
    bt = np.full((len(capacities), width), -1, dtype=np.int32)
    at = 0
    for s, n in enumerate(need):
        bt[s, :n] = perm[at:at + n]
        at += n
    return bt


def cu_from_lens(lens) -> np.ndarray:
    cu = np.zeros(len(lens) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(np.asarray(lens, dtype=np.int64))
    return cu


# ----------------------------------------------------------------------------
# a batch of work for one call of the path
# ----------------------------------------------------------------------------
@dataclass
class Geometry:
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    page_size: int
    num_pages: int
    dtype: int

    @property
    def scale(self) -> float:
        return 1.0 / float(np.sqrt(self.head_dim))

    @property
    def pool_shape(self):
        return (self.num_pages, self.num_kv_heads, self.page_size, self.head_dim)

    @property
    def kv_bytes_per_token(self) -> int:
        return 2 * self.num_kv_heads * self.head_dim * (4 if self.dtype == F32 else 2)


@dataclass
class Batch:
    """Inputs of one append + attention call over B sessions.

    prefix_lens[s] tokens of session s are already cached; new_lens[s] tokens
    are appended and attended (cold prefill: prefix 0; decode: new 1).
    """
    geom: Geometry
    block_tables: np.ndarray            # int32 [B, max_pages]
    prefix_lens: np.ndarray             # int32 [B]
    new_lens: np.ndarray                # int32 [B]
    q: np.ndarray                       # [T, Hq, D] stored
    k_new: np.ndarray                   # [T, Hkv, D] stored
    v_new: np.ndarray                   # [T, Hkv, D] stored
    cu_new: np.ndarray = field(default=None)  # int32 [B+1]

    def __post_init__(self):
        self.prefix_lens = np.ascontiguousarray(self.prefix_lens, dtype=np.int32)
        self.new_lens = np.ascontiguousarray(self.new_lens, dtype=np.int32)
        if self.cu_new is None:
            self.cu_new = cu_from_lens(self.new_lens)

    @property
    def batch(self) -> int:
        return len(self.new_lens)

    @property
    def total_new(self) -> int:
        return int(self.cu_new[-1])

    @property
    def ctx_lens(self) -> np.ndarray:
        return (self.prefix_lens + self.new_lens).astype(np.int32)

    @property
    def max_pages(self) -> int:
        return int(self.block_tables.shape[1])

    def visible_pairs(self) -> int:
        """(query row, key) pairs per query head the attention must cover."""
        p = self.prefix_lens.astype(np.int64)
        n = self.new_lens.astype(np.int64)
        return int((n * p + n * (n + 1) // 2).sum())

    def attn_flops(self) -> int:
        """2*D for the score and 2*D for the value product, per visible pair and head."""
        return 4 * self.geom.head_dim * self.geom.num_q_heads * self.visible_pairs()

    def kv_read_bytes(self) -> int:
        """KV bytes a pass over every session's full context reads once."""
        return int(self.ctx_lens.astype(np.int64).sum()) * self.geom.kv_bytes_per_token


def draw_batch(geom: Geometry, block_tables: np.ndarray, prefix_lens, new_lens, seed: int,
               stream: int, sigma_qk: Optional[float] = None, sigma_v: Optional[float] = None) -> Batch:
    """Draw Q, K_new, V_new ~ N(0, sigma^2); default sigma = 1/sqrt(D) as the configs state."""
    t = int(np.sum(new_lens))
    s_qk = 1.0 / np.sqrt(geom.head_dim) if sigma_qk is None else sigma_qk
    s_v = 1.0 / np.sqrt(geom.head_dim) if sigma_v is None else sigma_v
    q = normal_values(seed, stream, 0, (t, geom.num_q_heads, geom.head_dim), s_qk, geom.dtype)
    k = normal_values(seed, stream, 1, (t, geom.num_kv_heads, geom.head_dim), s_qk, geom.dtype)
    v = normal_values(seed, stream, 2, (t, geom.num_kv_heads, geom.head_dim), s_v, geom.dtype)
    return Batch(geom, block_tables, prefix_lens, new_lens, q, k, v)


def uniform_lens(rng: np.random.Generator, lo: int, hi: int, n: int) -> np.ndarray:
    """Integers uniform on [lo, hi], both ends included."""
    return rng.integers(lo, hi + 1, size=n, dtype=np.int64).astype(np.int32)


# ----------------------------------------------------------------------------
# the five benchmark configurations
# ----------------------------------------------------------------------------
def slm_geometry(num_pages: int, dtype: int = BF16) -> Geometry:
    """32 query heads, 8 KV heads, head_dim 128, page 16: the small-LM shape of configs 2-5."""
    return Geometry(32, 8, 128, 16, num_pages, dtype)


def config_seed(config_index: int) -> int:
    return BASE_SEED + config_index


@dataclass
class TinyConfig:
    """Config 1: fp32, 4/2 heads, D 64, 2 sessions: cold 256 -> resume 32 -> 16 decode steps."""
    geom: Geometry
    block_tables: np.ndarray
    cold: Batch
    resume: Batch
    decode_steps: list


def make_tiny(seed: Optional[int] = None, dtype: int = F32, sigma_qk: Optional[float] = None,
              sigma_v: Optional[float] = None) -> TinyConfig:
    seed = config_seed(1) if seed is None else seed
    geom = Geometry(4, 2, 64, 16, 64, dtype)
    b = 2
    cap = 256 + 32 + 16
    bt = deal_block_tables(rng_for(seed, 0), [cap] * b, geom.page_size, geom.num_pages)
    kw = dict(sigma_qk=sigma_qk, sigma_v=sigma_v)
    cold = draw_batch(geom, bt, [0] * b, [256] * b, seed + 50, 1, **kw)
    resume = draw_batch(geom, bt, [256] * b, [32] * b, seed + 50, 2, **kw)
    steps = [draw_batch(geom, bt, [288 + i] * b, [1] * b, seed + 50, 3 + i, **kw) for i in range(16)]
    return TinyConfig(geom, bt, cold, resume, steps)


@dataclass
class DecodeConfig:
    """Config 2 (and the decode half of config 5): B sessions with a cached context, 1 query each.

    `fill` appends ctx-1 tokens per session (not timed); `step` appends the
    last token and holds the query.
    """
    geom: Geometry
    block_tables: np.ndarray
    ctx_lens: np.ndarray
    fill: Batch
    step: Batch


def make_decode(batch: int = 64, lo: int = 1024, hi: int = 4096, num_pages: int = 32768,
                seed: Optional[int] = None, sigma_qk: Optional[float] = None,
                sigma_v: Optional[float] = None, geom: Optional[Geometry] = None) -> DecodeConfig:
    seed = config_seed(2) if seed is None else seed
    geom = slm_geometry(num_pages) if geom is None else geom
    rng = rng_for(seed, 0)
    ctx = uniform_lens(rng, lo, hi, batch)
    bt = deal_block_tables(rng, ctx, geom.page_size, geom.num_pages)
    kw = dict(sigma_qk=sigma_qk, sigma_v=sigma_v)
    fill = draw_batch(geom, bt, np.zeros(batch, np.int32), ctx - 1, seed + 50, 1, **kw)
    step = draw_batch(geom, bt, ctx - 1, np.ones(batch, np.int32), seed + 50, 2, **kw)
    return DecodeConfig(geom, bt, ctx, fill, step)


def make_decode_queue(n_decode: int = 64, n_resume: int = 8, ctx_lo: int = 1024, ctx_hi: int = 4096,
                      p_lo: int = 2048, p_hi: int = 8192, n_lo: int = 16, n_hi: int = 64, num_pages: int = 32768,
                      seed: Optional[int] = None, sigma_qk: Optional[float] = None, sigma_v: Optional[float] = None,
                      geom: Optional[Geometry] = None) -> "ResumeConfig":
    """The decode queue of one scheduling step: n_decode sessions that decode (one row each, contexts as in
    config 2) followed by n_resume sessions whose short tool output (n_lo..n_hi rows, prefixes as in config 4)
    was admitted beside them.  `fill` builds the caches, `chunk` is the batch of the step."""
    seed = config_seed(6) if seed is None else seed
    geom = slm_geometry(num_pages) if geom is None else geom
    rng = rng_for(seed, 0)
    p = np.concatenate([uniform_lens(rng, ctx_lo, ctx_hi, n_decode) - 1, uniform_lens(rng, p_lo, p_hi, n_resume)]).astype(np.int32)
    n = np.concatenate([np.ones(n_decode, np.int32), uniform_lens(rng, n_lo, n_hi, n_resume)]).astype(np.int32)
    bt = deal_block_tables(rng, p + n, geom.page_size, geom.num_pages)
    kw = dict(sigma_qk=sigma_qk, sigma_v=sigma_v)
    fill = draw_batch(geom, bt, np.zeros(len(p), np.int32), p, seed + 50, 1, **kw)
    chunk = draw_batch(geom, bt, p, n, seed + 50, 2, **kw)
    return ResumeConfig(geom, bt, fill, chunk)


def make_cold(batch: int = 8, n: int = 4096, num_pages: Optional[int] = None,
              seed: Optional[int] = None, sigma_qk: Optional[float] = None,
              sigma_v: Optional[float] = None, geom: Optional[Geometry] = None) -> Batch:
    """Config 3: B system prompts of n tokens each, appended then attended causally."""
    seed = config_seed(3) if seed is None else seed
    if geom is None:
        geom = slm_geometry(num_pages or batch * pages_for(n, 16))
    bt = deal_block_tables(rng_for(seed, 0), [n] * batch, geom.page_size, geom.num_pages)
    return draw_batch(geom, bt, [0] * batch, [n] * batch, seed + 50, 1, sigma_qk=sigma_qk, sigma_v=sigma_v)


@dataclass
class ResumeConfig:
    """Config 4: cached prefixes (filled, not timed) plus an appended chunk that is attended."""
    geom: Geometry
    block_tables: np.ndarray
    fill: Batch
    chunk: Batch


def make_resume(batch: int = 32, p_lo: int = 2048, p_hi: int = 8192, n_lo: int = 128, n_hi: int = 1024,
                num_pages: int = 18432, seed: Optional[int] = None, sigma_qk: Optional[float] = None,
                sigma_v: Optional[float] = None, geom: Optional[Geometry] = None) -> ResumeConfig:
    seed = config_seed(4) if seed is None else seed
    geom = slm_geometry(num_pages) if geom is None else geom
    rng = rng_for(seed, 0)
    p = uniform_lens(rng, p_lo, p_hi, batch)
    n = uniform_lens(rng, n_lo, n_hi, batch)
    bt = deal_block_tables(rng, p + n, geom.page_size, geom.num_pages)
    kw = dict(sigma_qk=sigma_qk, sigma_v=sigma_v)
    fill = draw_batch(geom, bt, np.zeros(batch, np.int32), p, seed + 50, 1, **kw)
    chunk = draw_batch(geom, bt, p, n, seed + 50, 2, **kw)
    return ResumeConfig(geom, bt, fill, chunk)


@dataclass
class MixedConfig:
    """Config 5: a prefill loop (2 cold of 8192; 8 resumes of 512 on 4096) beside 64 decode sessions.

    All sessions share one pool; their block tables are disjoint slices of
    one permutation.
    """
    geom: Geometry
    cold: Batch
    resume_fill: Batch
    resume: Batch
    decode_fill: Batch
    decode: Batch


def make_mixed(num_pages: int = 36864, seed: Optional[int] = None, n_cold: int = 2, cold_len: int = 8192,
               n_resume: int = 8, resume_prefix: int = 4096, resume_len: int = 512, n_decode: int = 64,
               d_lo: int = 1024, d_hi: int = 8192, geom: Optional[Geometry] = None) -> MixedConfig:
    seed = config_seed(5) if seed is None else seed
    geom = slm_geometry(num_pages) if geom is None else geom
    rng = rng_for(seed, 0)
    ctx = uniform_lens(rng, d_lo, d_hi, n_decode)
    caps = [cold_len] * n_cold + [resume_prefix + resume_len] * n_resume + list(ctx)
    bt = deal_block_tables(rng, caps, geom.page_size, geom.num_pages)
    bt_c = np.ascontiguousarray(bt[:n_cold])
    bt_r = np.ascontiguousarray(bt[n_cold:n_cold + n_resume])
    bt_d = np.ascontiguousarray(bt[n_cold + n_resume:])
    cold = draw_batch(geom, bt_c, [0] * n_cold, [cold_len] * n_cold, seed + 50, 1)
    r_fill = draw_batch(geom, bt_r, [0] * n_resume, [resume_prefix] * n_resume, seed + 50, 2)
    res = draw_batch(geom, bt_r, [resume_prefix] * n_resume, [resume_len] * n_resume, seed + 50, 3)
    d_fill = draw_batch(geom, bt_d, np.zeros(n_decode, np.int32), ctx - 1, seed + 50, 4)
    dec = draw_batch(geom, bt_d, ctx - 1, np.ones(n_decode, np.int32), seed + 50, 5)
    return MixedConfig(geom, cold, r_fill, res, d_fill, dec)


@dataclass
class ServingConfig:
    """Config 5's sessions with tool outputs of mixed length, cut the way the scheduler's two queues cut them:
    for every admission level a (the a shortest resume chunks fit the budget B_prefill), `queue_d[a]` is the
    decode queue's batch (all decodes followed by those a chunks) and `queue_p[a]` the resume chunks left to
    the prefill queue (None when there are none).  `cold` always belongs to the prefill queue."""
    geom: Geometry
    cold: Batch
    resume_fill: Batch
    decode_fill: Batch
    resume_lens: np.ndarray
    queue_d: dict
    queue_p: dict


def make_serving(num_pages: int = 36864, seed: Optional[int] = None, n_cold: int = 2, cold_len: int = 8192,
                 resume_prefix: int = 4096, resume_lens=(16, 32, 64, 96, 128, 256, 384, 512), n_decode: int = 64,
                 d_lo: int = 1024, d_hi: int = 8192, geom: Optional[Geometry] = None) -> ServingConfig:
    seed = config_seed(7) if seed is None else seed
    geom = slm_geometry(num_pages) if geom is None else geom
    rng = rng_for(seed, 0)
    lens = np.sort(np.asarray(resume_lens, np.int32))
    n_resume = len(lens)
    ctx = uniform_lens(rng, d_lo, d_hi, n_decode)
    caps = [cold_len] * n_cold + [resume_prefix + int(n) for n in lens] + list(ctx)
    bt = deal_block_tables(rng, caps, geom.page_size, geom.num_pages)
    bt_c, bt_r, bt_d = bt[:n_cold], bt[n_cold:n_cold + n_resume], bt[n_cold + n_resume:]
    cold = draw_batch(geom, np.ascontiguousarray(bt_c), [0] * n_cold, [cold_len] * n_cold, seed + 50, 1)
    r_fill = draw_batch(geom, np.ascontiguousarray(bt_r), [0] * n_resume, [resume_prefix] * n_resume, seed + 50, 2)
    d_fill = draw_batch(geom, np.ascontiguousarray(bt_d), np.zeros(n_decode, np.int32), ctx - 1, seed + 50, 3)
    queue_d, queue_p = {}, {}
    for a in range(n_resume + 1):
        bt_q = np.ascontiguousarray(np.concatenate([bt_d, bt_r[:a]]))
        prefix = np.concatenate([ctx - 1, np.full(a, resume_prefix, np.int32)]).astype(np.int32)
        new = np.concatenate([np.ones(n_decode, np.int32), lens[:a]]).astype(np.int32)
        queue_d[a] = draw_batch(geom, bt_q, prefix, new, seed + 50, 10 + a)
        queue_p[a] = None if a == n_resume else draw_batch(
            geom, np.ascontiguousarray(bt_r[a:]), [resume_prefix] * (n_resume - a), lens[a:], seed + 50, 30 + a)
    return ServingConfig(geom, cold, r_fill, d_fill, lens, queue_d, queue_p)


# ----------------------------------------------------------------------------
# adversarial value patterns (data only)
# ----------------------------------------------------------------------------
def position_bits(positions, head_dim: int) -> np.ndarray:
    """Rows whose entry d is bit d of the logical position (0.0 / 1.0): a value
    row that names the position it was stored at."""
    pos = np.asarray(positions, dtype=np.int64)
    nb = min(head_dim, 30)
    out = np.zeros((len(pos), head_dim), np.float32)
    out[:, :nb] = ((pos[:, None] >> np.arange(nb)[None, :]) & 1).astype(np.float32)
    return out


def planted_queries(k_ctx: np.ndarray, targets: np.ndarray, group: int, gain: float) -> np.ndarray:
    """Queries that single out one key each.

    k_ctx   float32 [L, Hkv, D]: every key of one session's context, in logical order.
    targets int [N, Hq]: the logical position row i / head h must select.
    Head h is paired with KV head h // group.  The query is the target key
    rescaled so that (1/sqrt(D)) * q.k_target == gain; with keys drawn
    N(0, 1) every other logit is ~ N(0, gain^2 / D), far below.
    """
    n, hq = targets.shape
    d = k_ctx.shape[2]
    kv_of = np.arange(hq) // group
    kt = k_ctx[targets, kv_of[None, :], :]                      # [N, Hq, D]
    nrm2 = (kt.astype(np.float64) ** 2).sum(-1, keepdims=True)
    return (kt * (gain * np.sqrt(d) / nrm2)).astype(np.float32)
