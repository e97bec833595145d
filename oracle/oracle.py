"""ctypes front for the C oracle (oracle/ag_oracle.c).  TEST INFRASTRUCTURE ONLY.

Takes the same stored inputs the GPU library takes (numpy float32, or uint16
bf16 bit patterns), returns float64.  Every function is a direct call of the
C routine of the same name; there is no arithmetic in this file.
"""
from __future__ import annotations

import ctypes as C

import numpy as np

from . import build as _build

F32, BF16 = 0, 1


class _Cache(C.Structure):
    _fields_ = [("k_pool", C.c_void_p), ("v_pool", C.c_void_p),
                ("num_pages", C.c_int32), ("page_size", C.c_int32),
                ("num_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("dtype", C.c_int32)]


_lib = None


def lib(path: str | None = None):
    global _lib
    if path is not None:
        return _bind(C.CDLL(path))
    if _lib is None:
        _lib = _bind(C.CDLL(_build.build()))
    return _lib


def _bind(l):
    i32p, vp = C.POINTER(C.c_int32), C.c_void_p
    l.ago_num_threads.restype = C.c_int
    l.ago_kv_append.restype = C.c_int
    l.ago_kv_append.argtypes = [C.POINTER(_Cache), vp, vp, i32p, C.c_int32, i32p, i32p, i32p, C.c_int32]
    l.ago_attn_rows.restype = C.c_int
    l.ago_attn_rows.argtypes = [C.POINTER(_Cache), vp, i32p, C.c_int32, i32p, i32p, i32p, C.c_int32,
                                C.c_int32, C.c_double, i32p, i32p, C.c_int64, C.POINTER(C.c_double)]
    l.ago_attn.restype = C.c_int
    l.ago_attn.argtypes = [C.POINTER(_Cache), vp, i32p, C.c_int32, i32p, i32p, i32p, C.c_int32,
                           C.c_int32, C.c_double, C.POINTER(C.c_double)]
    return l


class OracleError(RuntimeError):
    pass


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(C.POINTER(C.c_int32))


def _check_storage(a: np.ndarray, dtype: int, name: str):
    want = np.float32 if dtype == F32 else np.uint16
    if a.dtype != want or not a.flags["C_CONTIGUOUS"]:
        raise TypeError(f"{name}: need contiguous {want.__name__}, got {a.dtype}")


def _cache(k_pool, v_pool, dtype):
    _check_storage(k_pool, dtype, "k_pool")
    _check_storage(v_pool, dtype, "v_pool")
    if k_pool.shape != v_pool.shape or k_pool.ndim != 4:
        raise ValueError("pools must both be [num_pages, Hkv, page_size, D]")
    p, h, ps, d = k_pool.shape
    return _Cache(k_pool.ctypes.data, v_pool.ctypes.data, p, ps, h, d, dtype)


def num_threads() -> int:
    return int(lib().ago_num_threads())


def kv_append(k_pool, v_pool, dtype, k_new, v_new, block_tables, prefix_lens, new_lens, cu_new, _lib=None):
    """Write the new tokens' K/V into the pools in place (host arrays)."""
    l = _lib or lib()
    c = _cache(k_pool, v_pool, dtype)
    _check_storage(k_new, dtype, "k_new")
    _check_storage(v_new, dtype, "v_new")
    bt, btp = _i32(block_tables)
    pl, plp = _i32(prefix_lens)
    nl, nlp = _i32(new_lens)
    cu, cup = _i32(cu_new)
    rc = l.ago_kv_append(C.byref(c), k_new.ctypes.data, v_new.ctypes.data, btp, bt.shape[1], plp, nlp, cup, len(nl))
    if rc:
        raise OracleError(f"ago_kv_append failed: {rc}")


def attn(k_pool, v_pool, dtype, q, block_tables, prefix_lens, new_lens, cu_new, num_q_heads, scale,
         rows=None, _lib=None) -> np.ndarray:
    """Softmax attention of the new rows over their paged contexts, in fp64.

    rows=None: every row, result [T, Hq, D].  rows=(sessions, indices): only
    those rows, result [len, Hq, D].
    """
    l = _lib or lib()
    c = _cache(k_pool, v_pool, dtype)
    _check_storage(q, dtype, "q")
    bt, btp = _i32(block_tables)
    pl, plp = _i32(prefix_lens)
    nl, nlp = _i32(new_lens)
    cu, cup = _i32(cu_new)
    d = k_pool.shape[3]
    if rows is None:
        out = np.empty((int(cu[-1]), num_q_heads, d), dtype=np.float64)
        rc = l.ago_attn(C.byref(c), q.ctypes.data, btp, bt.shape[1], plp, nlp, cup, len(nl), num_q_heads,
                        float(scale), out.ctypes.data_as(C.POINTER(C.c_double)))
    else:
        rs, rsp = _i32(rows[0])
        ri, rip = _i32(rows[1])
        out = np.empty((len(rs), num_q_heads, d), dtype=np.float64)
        rc = l.ago_attn_rows(C.byref(c), q.ctypes.data, btp, bt.shape[1], plp, nlp, cup, len(nl), num_q_heads,
                             float(scale), rsp, rip, len(rs), out.ctypes.data_as(C.POINTER(C.c_double)))
    if rc:
        raise OracleError(f"ago_attn failed: {rc}")
    return out


def decode(k_pool, v_pool, dtype, q, block_tables, ctx_lens, num_q_heads, scale, _lib=None) -> np.ndarray:
    """A decode step is the N = 1 case: one query per session at position ctx_len - 1
    (the step's own key/value are already in the cache).  q [B, Hq, D] -> [B, Hq, D]."""
    ctx = np.ascontiguousarray(ctx_lens, dtype=np.int32)
    b = len(ctx)
    if np.any(ctx < 1):
        raise ValueError("the oracle's decode needs ctx_len >= 1 (an empty context has no softmax)")
    return attn(k_pool, v_pool, dtype, q, block_tables, ctx - 1, np.ones(b, np.int32),
                np.arange(b + 1, dtype=np.int32), num_q_heads, scale, _lib=_lib)
