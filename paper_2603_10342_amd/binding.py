"""ctypes binding of libagattn.so: same names as include/ag.h, argument
marshalling only.  Every step of the path runs in the HIP kernels behind the
C ABI; tensors are torch CUDA (ROCm) tensors used as device memory.

There is no fallback: if the library is missing or was not built, importing
`lib()` raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libagattn.so")

AG_OK, AG_ERR_INVALID_ARG, AG_ERR_UNSUPPORTED, AG_ERR_WORKSPACE, AG_ERR_HIP, AG_ERR_NO_SPACE = 0, -1, -2, -3, -4, -5
AG_F32, AG_BF16 = 0, 1

EXPORTS = [
    "ag_kv_append", "ag_attn_prefill", "ag_attn_resume", "ag_attn_decode_workspace_bytes", "ag_attn_decode",
    "ag_attn_decode_static", "ag_decode_step_workspace_bytes", "ag_decode_step",
    "ag_attn_merged_workspace_bytes", "ag_attn_merged",
    "ag_stream_create_cumask", "ag_stream_destroy", "ag_cumask_build", "ag_probe_placement", "ag_device_info",
    "ag_debug_validate", "ag_prof_enable", "ag_prof_collect", "ag_prof_disable", "ag_status_string",
    "ag_last_error", "ag_version",
    # ag_sched.h
    "ag_ctl_create", "ag_ctl_destroy", "ag_ctl_record_decode", "ag_ctl_tick", "ag_ctl_get", "ag_ctl_classify",
    "ag_partition_level_for", "ag_slots_create", "ag_slots_destroy", "ag_slots_count", "ag_slots_units",
    "ag_slots_get", "ag_slots_bind", "ag_slots_current",
    # ag_pager.h
    "ag_pager_create", "ag_pager_destroy", "ag_pager_open", "ag_pager_close", "ag_pager_reserve", "ag_pager_seal",
    "ag_pager_commit", "ag_pager_acquire", "ag_pager_release", "ag_pager_lengths", "ag_pager_export", "ag_pager_page_state",
    "ag_pager_get_stats",
]
AG_PAGE_FREE, AG_PAGE_WRITABLE, AG_PAGE_SEALED = 0, 1, 2

AG_REQ_DECODE, AG_REQ_RESUME, AG_REQ_COLD = 0, 1, 2
AG_QUEUE_DECODE, AG_QUEUE_PREFILL = 0, 1


class AgError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{message} (status {status})")
        self.status = status


class ag_ctl_params(C.Structure):
    _fields_ = [("S", C.c_int32), ("r_base", C.c_int32), ("r_init", C.c_int32), ("b_init", C.c_int32),
                ("delta_r", C.c_int32), ("delta_b", C.c_int32), ("b_min", C.c_int32), ("b_max", C.c_int32),
                ("theta_low_us", C.c_double), ("theta_high_us", C.c_double)]


class ag_ctl_state(C.Structure):
    _fields_ = [("r_min", C.c_int32), ("b_prefill", C.c_int32), ("tpot_us", C.c_double),
                ("intervals", C.c_int64), ("raised", C.c_int64), ("lowered", C.c_int64)]


class ag_pager_stats(C.Structure):
    _fields_ = [("num_pages", C.c_int32), ("free_pages", C.c_int32), ("open_sessions", C.c_int32),
                ("reserves", C.c_int64), ("failed_reserves", C.c_int64), ("commits", C.c_int64),
                ("waits_issued", C.c_int64), ("waits_skipped", C.c_int64),
                ("releases", C.c_int64), ("close_waits", C.c_int64)]


class ag_kv_cache(C.Structure):
    _fields_ = [("k_pool", C.c_void_p), ("v_pool", C.c_void_p), ("num_pages", C.c_int32),
                ("page_size", C.c_int32), ("num_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("dtype", C.c_int32)]


_lib = None


def lib():
    """Load the HIP library (built in-tree by paper_2603_10342_amd/build.py).  Fails loudly."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2603_10342_amd.build` "
                          "(or __graft_entry__.build()); there is no fallback path")
    l = C.CDLL(LIB_PATH)
    vp, i32, i32p, u32p = C.c_void_p, C.c_int32, C.c_void_p, C.POINTER(C.c_uint32)
    cp = C.POINTER(ag_kv_cache)
    l.ag_kv_append.argtypes = [cp, vp, vp, i32p, i32, i32p, i32p, i32p, i32, i32, vp]
    l.ag_attn_prefill.argtypes = [cp, vp, vp, i32p, i32, i32p, i32p, i32, i32, i32, i32, C.c_float, vp]
    l.ag_attn_resume.argtypes = [cp, vp, vp, i32p, i32, i32p, i32p, i32p, i32, i32, i32, i32, i32, C.c_float, vp]
    l.ag_attn_decode_workspace_bytes.argtypes = [i32, i32, i32, i32]
    l.ag_attn_decode_workspace_bytes.restype = C.c_size_t
    l.ag_attn_decode.argtypes = [cp, vp, vp, i32p, i32, i32p, i32, i32, i32, C.c_float, vp, C.c_size_t, vp]
    l.ag_attn_decode_static.argtypes = [cp, vp, vp, i32p, i32, i32p, i32, i32, i32, C.c_float, vp]
    l.ag_decode_step_workspace_bytes.argtypes = [i32, i32, i32, i32]
    l.ag_decode_step_workspace_bytes.restype = C.c_size_t
    l.ag_decode_step.argtypes = [cp, vp, vp, vp, vp, i32p, i32, i32p, i32, i32, i32, C.c_float, vp, C.c_size_t, vp]
    l.ag_attn_merged_workspace_bytes.argtypes = [i32, i32, i32]
    l.ag_attn_merged_workspace_bytes.restype = C.c_size_t
    l.ag_attn_merged.argtypes = [cp, vp, vp, i32p, i32, i32p, i32p, i32p, i32, i32, i32, i32, i32, C.c_float, vp,
                                 C.c_size_t, vp]
    l.ag_stream_create_cumask.argtypes = [C.POINTER(vp), u32p, i32]
    l.ag_stream_destroy.argtypes = [vp]
    l.ag_cumask_build.argtypes = [u32p, i32, i32, i32, i32, i32]
    l.ag_probe_placement.argtypes = [vp, i32, i32, vp]
    l.ag_device_info.argtypes = [C.POINTER(i32), C.POINTER(i32), C.POINTER(i32), C.c_char_p, i32]
    l.ag_debug_validate.argtypes = [cp, i32p, i32, i32p, i32p, i32p, i32, vp]
    l.ag_prof_enable.argtypes = [i32]
    l.ag_prof_collect.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(C.c_double), C.POINTER(i32)]
    l.ag_prof_disable.argtypes = []
    l.ag_ctl_create.argtypes = [C.POINTER(ag_ctl_params), C.POINTER(vp)]
    l.ag_ctl_destroy.argtypes = [vp]
    l.ag_ctl_record_decode.argtypes = [vp, C.c_double]
    l.ag_ctl_tick.argtypes = [vp, C.POINTER(ag_ctl_state)]
    l.ag_ctl_get.argtypes = [vp, C.POINTER(ag_ctl_state)]
    l.ag_ctl_classify.argtypes = [vp, i32, i32]
    l.ag_partition_level_for.argtypes = [i32, i32, i32]
    l.ag_slots_create.argtypes = [i32, C.POINTER(vp)]
    l.ag_slots_destroy.argtypes = [vp]
    l.ag_slots_count.argtypes = [vp]
    l.ag_slots_units.argtypes = [vp]
    l.ag_slots_get.argtypes = [vp, i32, C.POINTER(i32), C.POINTER(vp), C.POINTER(vp)]
    l.ag_slots_bind.argtypes = [vp, i32, C.POINTER(i32)]
    l.ag_slots_current.argtypes = [vp]
    pi32 = C.POINTER(i32)
    l.ag_pager_create.argtypes = [i32, i32, i32, i32, C.POINTER(vp)]
    l.ag_pager_destroy.argtypes = [vp]
    l.ag_pager_open.argtypes = [vp, pi32]
    l.ag_pager_close.argtypes = [vp, i32]
    l.ag_pager_reserve.argtypes = [vp, i32, i32, pi32]
    l.ag_pager_seal.argtypes = [vp, i32]
    l.ag_pager_commit.argtypes = [vp, i32, vp]
    l.ag_pager_acquire.argtypes = [vp, i32, vp, pi32]
    l.ag_pager_release.argtypes = [vp, i32, vp]
    l.ag_pager_lengths.argtypes = [vp, i32, pi32, pi32, pi32]
    l.ag_pager_export.argtypes = [vp, pi32, i32, pi32]
    l.ag_pager_page_state.argtypes = [vp, i32]
    l.ag_pager_get_stats.argtypes = [vp, C.POINTER(ag_pager_stats)]
    for name in EXPORTS:
        if name not in ("ag_attn_decode_workspace_bytes", "ag_decode_step_workspace_bytes", "ag_attn_merged_workspace_bytes", "ag_status_string", "ag_last_error", "ag_version"):
            getattr(l, name).restype = C.c_int
    l.ag_status_string.argtypes = [C.c_int]
    for name in ("ag_status_string", "ag_last_error", "ag_version"):
        getattr(l, name).restype = C.c_char_p
    _lib = l
    return l


def _check(status: int):
    if status != AG_OK:
        raise AgError(status, lib().ag_last_error().decode())


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("device pointers must come from contiguous CUDA/ROCm tensors")
    return t.data_ptr()


def _i32(t: Optional[torch.Tensor]):
    if t is not None and t.dtype != torch.int32:
        raise TypeError("length arrays and block tables are int32")
    return _ptr(t)


def _stream(stream) -> Optional[int]:
    """None -> torch's current stream; an int is a raw hipStream_t; a torch stream gives its handle."""
    if stream is None:
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


def torch_dtype(dtype: int):
    return torch.float32 if dtype == AG_F32 else torch.bfloat16


class KVCache:
    """Caller-owned paged pools plus the geometry the library needs (mirrors ag_kv_cache)."""

    def __init__(self, num_pages: int, page_size: int, num_kv_heads: int, head_dim: int, dtype: int,
                 device="cuda", fill: Optional[float] = None):
        td = torch_dtype(dtype)
        mk = torch.empty if fill is None else (lambda *a, **k: torch.full(*a, fill_value=fill, **k))
        self.k_pool = mk((num_pages, num_kv_heads, head_dim // 8, page_size, 8), dtype=td, device=device)
        vshape = (num_pages, num_kv_heads, head_dim, page_size) if page_size < 16 else \
                 (num_pages, num_kv_heads, page_size // 8, head_dim, 8)
        self.v_pool = mk(vshape, dtype=td, device=device)
        self.num_pages, self.page_size = num_pages, page_size
        self.num_kv_heads, self.head_dim, self.dtype = num_kv_heads, head_dim, dtype

    def c_struct(self) -> ag_kv_cache:
        return ag_kv_cache(self.k_pool.data_ptr(), self.v_pool.data_ptr(), self.num_pages, self.page_size,
                           self.num_kv_heads, self.head_dim, self.dtype)

    def k_pool_token_major(self) -> torch.Tensor:
        """The key pool as [page][head][slot][d] (the library stores [d/8][slot][8])."""
        return self.k_pool.permute(0, 1, 3, 2, 4).reshape(self.num_pages, self.num_kv_heads, self.page_size,
                                                           self.head_dim)

    def v_pool_token_major(self) -> torch.Tensor:
        """The value pool as [page][head][slot][d].  The library stores page sizes >= 16 as [slot chunk][d][8 keys]
        with chunk 2g + h of each 16-slot group g holding slots h*4 + {0..3}, 8 + h*4 + {0..3}; smaller pages
        as [d][slot]."""
        ps = self.page_size
        if ps < 16:
            return self.v_pool.transpose(2, 3)
        s = torch.arange(ps, device=self.v_pool.device)
        chunk = ((s >> 4) << 1) | ((s >> 2) & 1)
        pos = (s & 3) | (((s >> 3) & 1) << 2)
        flat = self.v_pool.permute(0, 1, 2, 4, 3).reshape(self.num_pages, self.num_kv_heads, ps, self.head_dim)
        return flat.index_select(2, chunk * 8 + pos)


def ag_kv_append(cache: KVCache, k_new, v_new, block_tables, prefix_lens, new_lens, cu_new, total_new: int,
                 stream=None):
    c = cache.c_struct()
    _check(lib().ag_kv_append(C.byref(c), _ptr(k_new), _ptr(v_new), _i32(block_tables), block_tables.shape[1],
                              _i32(prefix_lens), _i32(new_lens), _i32(cu_new), new_lens.shape[0], total_new,
                              _stream(stream)))


def ag_attn_prefill(cache: KVCache, q, out, block_tables, new_lens, cu_new, total_new: int, max_new: int,
                    num_q_heads: int, scale: float, stream=None):
    c = cache.c_struct()
    _check(lib().ag_attn_prefill(C.byref(c), _ptr(q), _ptr(out), _i32(block_tables), block_tables.shape[1],
                                 _i32(new_lens), _i32(cu_new), new_lens.shape[0], total_new, max_new, num_q_heads,
                                 scale, _stream(stream)))


def ag_attn_resume(cache: KVCache, q, out, block_tables, prefix_lens, new_lens, cu_new, total_new: int,
                   max_new: int, max_ctx: int, num_q_heads: int, scale: float, stream=None):
    c = cache.c_struct()
    _check(lib().ag_attn_resume(C.byref(c), _ptr(q), _ptr(out), _i32(block_tables), block_tables.shape[1],
                                _i32(prefix_lens), _i32(new_lens), _i32(cu_new), new_lens.shape[0], total_new,
                                max_new, max_ctx, num_q_heads, scale, _stream(stream)))


def ag_attn_decode_workspace_bytes(batch: int, num_q_heads: int, head_dim: int, max_ctx: int) -> int:
    return int(lib().ag_attn_decode_workspace_bytes(batch, num_q_heads, head_dim, max_ctx))


def ag_attn_decode(cache: KVCache, q, out, block_tables, ctx_lens, max_ctx: int, num_q_heads: int, scale: float,
                   workspace: torch.Tensor, stream=None):
    c = cache.c_struct()
    _check(lib().ag_attn_decode(C.byref(c), _ptr(q), _ptr(out), _i32(block_tables), block_tables.shape[1],
                                _i32(ctx_lens), ctx_lens.shape[0], max_ctx, num_q_heads, scale, _ptr(workspace),
                                workspace.numel() * workspace.element_size(), _stream(stream)))


AG_DECODE_STATIC_SCRATCH_BYTES = 32 << 20


def ag_attn_decode_static(cache: KVCache, q, out, block_tables, ctx_lens, max_ctx: int, num_q_heads: int, scale: float,
                          stream=None):
    c = cache.c_struct()
    _check(lib().ag_attn_decode_static(C.byref(c), _ptr(q), _ptr(out), _i32(block_tables), block_tables.shape[1],
                                       _i32(ctx_lens), ctx_lens.shape[0], max_ctx, num_q_heads, scale,
                                       _stream(stream)))


AG_DECODE_STEP_COUNTER_BYTES = 256 << 10


def ag_decode_step_workspace_bytes(batch: int, num_q_heads: int, head_dim: int, max_ctx: int) -> int:
    return int(lib().ag_decode_step_workspace_bytes(batch, num_q_heads, head_dim, max_ctx))


def ag_decode_step(cache: KVCache, k_new, v_new, q, out, block_tables, ctx_lens, max_ctx: int, num_q_heads: int,
                   scale: float, workspace: torch.Tensor, stream=None):
    """`workspace` must have been zero-filled once before its first use (every call leaves its counters zero)."""
    c = cache.c_struct()
    _check(lib().ag_decode_step(C.byref(c), _ptr(k_new), _ptr(v_new), _ptr(q), _ptr(out), _i32(block_tables),
                                block_tables.shape[1], _i32(ctx_lens), ctx_lens.shape[0], max_ctx, num_q_heads, scale,
                                _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)))


def ag_attn_merged_workspace_bytes(total_new: int, num_q_heads: int, max_ctx: int) -> int:
    return int(lib().ag_attn_merged_workspace_bytes(total_new, num_q_heads, max_ctx))


def ag_attn_merged(cache: KVCache, q, out, block_tables, prefix_lens, new_lens, cu_new, total_new: int,
                   max_new: int, max_ctx: int, num_q_heads: int, scale: float, workspace: torch.Tensor, stream=None):
    c = cache.c_struct()
    _check(lib().ag_attn_merged(C.byref(c), _ptr(q), _ptr(out), _i32(block_tables), block_tables.shape[1],
                                _i32(prefix_lens), _i32(new_lens), _i32(cu_new), new_lens.shape[0], total_new,
                                max_new, max_ctx, num_q_heads, scale, _ptr(workspace),
                                workspace.numel() * workspace.element_size(), _stream(stream)))


def ag_cumask_build(total_cus: int, n_xcd: int, first_cu_per_xcd: int, cus_per_xcd: int) -> list:
    n_words = (total_cus + 31) // 32
    words = (C.c_uint32 * n_words)()
    _check(lib().ag_cumask_build(words, n_words, total_cus, n_xcd, first_cu_per_xcd, cus_per_xcd))
    return list(words)


def ag_stream_create_cumask(words: Sequence[int]) -> int:
    arr = (C.c_uint32 * len(words))(*words)
    out = C.c_void_p()
    _check(lib().ag_stream_create_cumask(C.byref(out), arr, len(words)))
    return int(out.value)


def ag_stream_destroy(stream: int):
    _check(lib().ag_stream_destroy(stream))


def ag_probe_placement(ids_out: torch.Tensor, spin_cycles: int, stream=None):
    if ids_out.dtype != torch.int32:
        raise TypeError("ids_out is a 32-bit integer tensor")
    _check(lib().ag_probe_placement(_ptr(ids_out), ids_out.numel(), spin_cycles, _stream(stream)))


def ag_device_info() -> dict:
    cus, xcd, wave = C.c_int32(), C.c_int32(), C.c_int32()
    name = C.create_string_buffer(64)
    _check(lib().ag_device_info(C.byref(cus), C.byref(xcd), C.byref(wave), name, 64))
    return {"num_cus": cus.value, "num_xcd": xcd.value, "wavefront_size": wave.value, "arch": name.value.decode()}


def ag_debug_validate(cache: KVCache, block_tables, prefix_lens, new_lens, cu_new, stream=None):
    c = cache.c_struct()
    _check(lib().ag_debug_validate(C.byref(c), _i32(block_tables), block_tables.shape[1], _i32(prefix_lens),
                                   _i32(new_lens), _i32(cu_new), new_lens.shape[0], _stream(stream)))


def ag_prof_enable(max_launches: int):
    _check(lib().ag_prof_enable(max_launches))


def ag_prof_collect() -> dict:
    mean, lo, hi, n = C.c_double(), C.c_double(), C.c_double(), C.c_int32()
    _check(lib().ag_prof_collect(C.byref(mean), C.byref(lo), C.byref(hi), C.byref(n)))
    return {"mean_us": mean.value, "min_us": lo.value, "max_us": hi.value, "n": n.value}


def ag_prof_disable():
    _check(lib().ag_prof_disable())


def ag_version() -> str:
    return lib().ag_version().decode()


def ag_status_string(status: int) -> str:
    return lib().ag_status_string(status).decode()


# ---- ag_sched.h: controller (Algorithm 1) and the table of pre-established partitions ----

def _nonneg(v: int) -> int:
    if v < 0:
        raise AgError(v, lib().ag_last_error().decode())
    return v


class Controller:
    """Owns an ag_ctl.  Methods are the entry points of the same name without the prefix."""

    def __init__(self, **params):
        self._p = ag_ctl_params(**params)
        h = C.c_void_p()
        _check(lib().ag_ctl_create(C.byref(self._p), C.byref(h)))
        self._h = h

    def close(self):
        if self._h:
            _check(lib().ag_ctl_destroy(self._h))
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def record_decode(self, step_us: float):
        _check(lib().ag_ctl_record_decode(self._h, step_us))

    def _state(self, fn) -> dict:
        st = ag_ctl_state()
        _check(fn(self._h, C.byref(st)))
        return {k: getattr(st, k) for k, _ in ag_ctl_state._fields_}

    def tick(self) -> dict:
        return self._state(lib().ag_ctl_tick)

    def get(self) -> dict:
        return self._state(lib().ag_ctl_get)

    def classify(self, req_type: int, len_tokens: int) -> int:
        return _nonneg(lib().ag_ctl_classify(self._h, req_type, len_tokens))


def ag_partition_level_for(S: int, g: int, r_min: int) -> int:
    return _nonneg(lib().ag_partition_level_for(S, g, r_min))


class Slots:
    """Owns an ag_slots table (CU-masked stream pairs on the current device)."""

    def __init__(self, g_units: int):
        h = C.c_void_p()
        _check(lib().ag_slots_create(g_units, C.byref(h)))
        self._h = h

    def close(self):
        if self._h:
            _check(lib().ag_slots_destroy(self._h))
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def count(self) -> int:
        return _nonneg(lib().ag_slots_count(self._h))

    def units(self) -> int:
        return _nonneg(lib().ag_slots_units(self._h))

    def get(self, index: int) -> dict:
        u, d, p = C.c_int32(), C.c_void_p(), C.c_void_p()
        _check(lib().ag_slots_get(self._h, index, C.byref(u), C.byref(d), C.byref(p)))
        # the last entry reserves the whole device for decode and has NO prefill stream: None, never 0 - a 0 would
        # be taken for the default stream by every launch helper and run a prefill unmasked on all CUs
        return {"decode_units": u.value, "decode_stream": int(d.value or 0),
                "prefill_stream": int(p.value) if p.value else None}

    def bind(self, r_min: int) -> int:
        i = C.c_int32()
        _check(lib().ag_slots_bind(self._h, r_min, C.byref(i)))
        return i.value

    def current(self) -> int:
        return _nonneg(lib().ag_slots_current(self._h))


# ---- ag_pager.h: KV page manager ----

class Pager:
    """Owns an ag_pager.  Methods are the entry points of the same name without the prefix."""

    def __init__(self, num_pages: int, page_size: int, max_sessions: int, max_pages_per_seq: int):
        h = C.c_void_p()
        _check(lib().ag_pager_create(num_pages, page_size, max_sessions, max_pages_per_seq, C.byref(h)))
        self._h = h
        self.max_pages_per_seq = max_pages_per_seq

    def destroy(self):
        if self._h:
            _check(lib().ag_pager_destroy(self._h))
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def open(self) -> int:
        s = C.c_int32()
        _check(lib().ag_pager_open(self._h, C.byref(s)))
        return s.value

    def close(self, session: int):
        _check(lib().ag_pager_close(self._h, session))

    def reserve(self, session: int, new_tokens: int) -> int:
        start = C.c_int32()
        _check(lib().ag_pager_reserve(self._h, session, new_tokens, C.byref(start)))
        return start.value

    def seal(self, session: int):
        _check(lib().ag_pager_seal(self._h, session))

    def commit(self, session: int, stream=None):
        _check(lib().ag_pager_commit(self._h, session, _stream(stream)))

    def acquire(self, session: int, stream=None) -> int:
        n = C.c_int32()
        _check(lib().ag_pager_acquire(self._h, session, _stream(stream), C.byref(n)))
        return n.value

    def release(self, session: int, stream=None):
        _check(lib().ag_pager_release(self._h, session, _stream(stream)))

    def lengths(self, session: int) -> dict:
        r, s, p = C.c_int32(), C.c_int32(), C.c_int32()
        _check(lib().ag_pager_lengths(self._h, session, C.byref(r), C.byref(s), C.byref(p)))
        return {"reserved": r.value, "sealed": s.value, "pages": p.value}

    def export(self, sessions: Sequence[int]):
        """Block-table rows of the sessions as a host int32 array [n][max_pages_per_seq]."""
        import numpy as np
        n = len(sessions)
        ids = (C.c_int32 * n)(*sessions)
        rows = np.zeros((n, self.max_pages_per_seq), np.int32)
        _check(lib().ag_pager_export(self._h, ids, n, rows.ctypes.data_as(C.POINTER(C.c_int32))))
        return rows

    def page_state(self, page: int) -> int:
        return _nonneg(lib().ag_pager_page_state(self._h, page))

    def stats(self) -> dict:
        st = ag_pager_stats()
        _check(lib().ag_pager_get_stats(self._h, C.byref(st)))
        return {k: getattr(st, k) for k, _ in ag_pager_stats._fields_}
