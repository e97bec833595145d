"""No GPU needed: the C-ABI library loads, exports every symbol the headers under include/
declare, and its host-side checks answer before any device work."""
import ctypes as C
import os
import re

import numpy as np

import pytest

from paper_2603_10342_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    inc = os.path.join(ROOT, "include")
    text = "".join(open(os.path.join(inc, f)).read() for f in sorted(os.listdir(inc)) if f.endswith(".h"))
    return sorted(set(re.findall(r"AG_API\s+[\w\s\*]+?\b(ag_\w+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert len(names) >= 14 and "ag_attn_decode" in names and "ag_stream_create_cumask" in names
    assert sorted(B.EXPORTS) == names
    l = B.lib()
    for n in names:
        assert hasattr(l, n), n


def test_status_strings_and_version():
    assert B.ag_status_string(0) == "AG_OK"
    assert B.ag_status_string(-3) == "AG_ERR_WORKSPACE"
    assert "gfx950" in B.ag_version()


def test_null_and_shape_errors_come_from_the_host_layer():
    l = B.lib()
    ok = B.ag_kv_cache(4096, 4096, 8, 16, 2, 128, B.AG_BF16)          # non-null fake pointers: never dereferenced here
    assert l.ag_kv_append(None, None, None, None, 1, None, None, None, 1, 1, None) == B.AG_ERR_INVALID_ARG
    assert l.ag_kv_append(C.byref(ok), None, None, None, 1, None, None, None, 1, 1, None) == B.AG_ERR_INVALID_ARG
    assert b"NULL" in l.ag_last_error()
    for field, val, want in [("dtype", 7, B.AG_ERR_UNSUPPORTED), ("head_dim", 100, B.AG_ERR_UNSUPPORTED),
                             ("head_dim", 512, B.AG_ERR_UNSUPPORTED), ("page_size", 24, B.AG_ERR_UNSUPPORTED),
                             ("num_pages", 0, B.AG_ERR_INVALID_ARG)]:
        c = B.ag_kv_cache(4096, 4096, 8, 16, 2, 128, B.AG_BF16)
        setattr(c, field, val)
        assert l.ag_attn_prefill(C.byref(c), 1, 1, 1, 4, 1, 1, 1, 16, 16, 4, 0.1, None) == want, field
    # heads not a multiple, contradictory bounds, bad scale
    assert l.ag_attn_prefill(C.byref(ok), 16, 16, 16, 4, 16, 16, 1, 16, 16, 3, 0.1, None) == B.AG_ERR_INVALID_ARG
    assert l.ag_attn_prefill(C.byref(ok), 16, 16, 16, 4, 16, 16, 1, 16, 32, 4, 0.1, None) == B.AG_ERR_INVALID_ARG
    assert l.ag_attn_prefill(C.byref(ok), 16, 16, 16, 4, 16, 16, 1, 16, 16, 4, 0.0, None) == B.AG_ERR_INVALID_ARG
    assert l.ag_attn_resume(C.byref(ok), 16, 16, 16, 4, 16, 16, 16, 1, 16, 16, 65, 4, 0.1, None) == B.AG_ERR_INVALID_ARG
    assert l.ag_attn_decode(C.byref(ok), 16, 16, 16, 4, 16, 1, 64, 4, 0.1, 16, 8, None) == B.AG_ERR_WORKSPACE
    assert l.ag_attn_decode(C.byref(ok), 16, 16, 16, 4, 16, 1, 65, 4, 0.1, 16, 1 << 20, None) == B.AG_ERR_INVALID_ARG
    # the static-scratch decode refuses, on the host, a step larger than its array (and checks its arguments first)
    assert l.ag_attn_decode_static(C.byref(ok), 16, 16, 16, 8192, 16, 512, 131072, 32, 0.1, None) == B.AG_ERR_WORKSPACE
    assert b"scratch" in l.ag_last_error()
    assert l.ag_attn_decode_static(C.byref(ok), 16, 16, 16, 4, 16, 1, 65, 4, 0.1, None) == B.AG_ERR_INVALID_ARG
    assert l.ag_attn_decode_static(C.byref(ok), None, 16, 16, 4, 16, 1, 64, 4, 0.1, None) == B.AG_ERR_INVALID_ARG
    # zero new tokens is a no-op that never reaches the device
    assert l.ag_kv_append(C.byref(ok), 16, 16, 16, 4, 16, 16, 16, 1, 0, None) == B.AG_OK
    assert l.ag_attn_prefill(C.byref(ok), 16, 16, 16, 4, 16, 16, 1, 0, 0, 4, 0.1, None) == B.AG_OK


def test_decode_workspace_size():
    # a header of 1 + batch int32 (rounded up to 16 bytes), then one (max, sum, D values) fp32 triple per
    # (session, query head, segment): shares are at least 256 tokens, and a context of n shares can straddle
    # one more boundary than it has shares
    assert B.ag_attn_decode_workspace_bytes(64, 32, 128, 4096) == 68 * 4 + 64 * 32 * 17 * 130 * 4
    assert B.ag_attn_decode_workspace_bytes(2, 4, 64, 1) == 4 * 4 + 2 * 4 * 2 * 66 * 4
    assert B.ag_attn_decode_workspace_bytes(0, 4, 64, 1) == 0


def test_cumask_builder_is_symmetric_over_xcds():
    w = B.ag_cumask_build(256, 8, 0, 4)                 # 4 CUs in each of 8 XCDs = 32 CUs
    assert w == [0xFFFFFFFF] + [0] * 7
    w = B.ag_cumask_build(256, 8, 4, 28)                # the complement
    assert w == [0] + [0xFFFFFFFF] * 7
    w = B.ag_cumask_build(256, 8, 0, 12)
    assert sum(bin(x).count("1") for x in w) == 96
    bits = [i for i in range(256) if (w[i // 32] >> (i % 32)) & 1]
    assert all(sum(1 for b in bits if b % 8 == x) == 12 for x in range(8))
    w = B.ag_cumask_build(64, 4, 1, 2)                  # other shapes: bit = cu * n_xcd + xcd
    assert [i for i in range(64) if (w[i // 32] >> (i % 32)) & 1] == [4, 5, 6, 7, 8, 9, 10, 11]
    with pytest.raises(B.AgError):
        B.ag_cumask_build(256, 8, 30, 4)
    with pytest.raises(B.AgError):
        B.ag_cumask_build(250, 8, 0, 4)


def test_empty_mask_is_rejected_without_touching_the_device():
    l = B.lib()
    words = (C.c_uint32 * 8)()
    out = C.c_void_p()
    assert l.ag_stream_create_cumask(C.byref(out), words, 8) == B.AG_ERR_INVALID_ARG
    assert l.ag_stream_create_cumask(None, words, 8) == B.AG_ERR_INVALID_ARG
    assert l.ag_stream_destroy(None) == B.AG_ERR_INVALID_ARG


def test_decode_workspace_covers_every_cut_of_a_context():
    """The decode kernel deals the batch's (session, KV head) contexts, laid end to end in steps of 32 tokens,
    in equal shares of q >= 8 steps; a context of n steps starting at flat step a is then cut into
    floor((a + n - 1) / q) - floor(a / q) + 1 partials.  The workspace must hold that many per (session, head)
    for any batch the bounds admit: checked here on the host against the size function."""
    rng = np.random.default_rng(7)
    for trial in range(200):
        batch = int(rng.integers(1, 40))
        hkv = int(rng.choice([1, 2, 4, 8]))
        hq = hkv * int(rng.choice([1, 2, 4]))
        max_ctx = int(rng.integers(1, 20000))
        ctx = rng.integers(0, max_ctx + 1, size=batch)
        ctx[rng.integers(0, batch)] = max_ctx
        nbytes = B.ag_attn_decode_workspace_bytes(batch, hq, 128, max_ctx)
        header = ((batch + 1 + 3) // 4) * 4 * 4
        slots = (nbytes - header) // (batch * hq * 130 * 4)
        assert header + batch * hq * slots * 130 * 4 == nbytes
        steps = (ctx + 31) // 32
        F = hkv * int(steps.sum())
        for W in (1024, 1, 37, max(1024, (hkv * batch * ((max_ctx + 31) // 32) + 127) // 128)):
            q = max(8, -(-F // W))
            a = 0
            for n in steps:
                for g in range(hkv):
                    if n:
                        assert (a + n - 1) // q - a // q + 1 <= slots, (batch, hkv, max_ctx, W, q, a, n, slots)
                    a += int(n)
