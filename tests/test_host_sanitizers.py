"""The library's host-side code and the C oracle under the CPU sanitizers (no GPU involved).

  - paper_2603_10342_amd/csrc/ag_api.hip (argument validation), ag_sched.hip (controller, partition table) and
    ag_pager.hip (page manager) are compiled as plain C++ against the stand-in HIP runtime of tests/hostbuild/
    and driven by tests/hostbuild/host_driver.cpp - bad and good arguments with exact-size buffers, the controller
    and the table from several threads, the page manager's close-versus-reader ordering and a four-thread random
    walk - once under AddressSanitizer + UndefinedBehaviorSanitizer and once under ThreadSanitizer;
  - oracle/ag_oracle.c is compiled with AddressSanitizer + UndefinedBehaviorSanitizer into a small program that
    runs append and attention on ragged, page-crossing inputs read from a file; its outputs must equal, bit for
    bit, what the ordinary build of the oracle gives for the same inputs.
"""
import os
import shutil
import subprocess
import sys

import numpy as np
import pytest

from helpers import fresh_pools, make_batch
from oracle import oracle as O
from paper_2603_10342_amd import inputs as I

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HB = os.path.join(ROOT, "tests", "hostbuild")
CSRC = os.path.join(ROOT, "paper_2603_10342_amd", "csrc")
BAD = ("ERROR: AddressSanitizer", "ERROR: LeakSanitizer", "runtime error:", "WARNING: ThreadSanitizer", "CHECK failed")

pytestmark = pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")


def run_checked(cmd, **kw):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               TSAN_OPTIONS="halt_on_error=1")
    r = subprocess.run(cmd, capture_output=True, text=True, env=env, timeout=600, **kw)
    text = r.stdout + r.stderr
    assert r.returncode == 0 and not any(b in text for b in BAD), text[-4000:]
    return text


@pytest.mark.parametrize("sanitizers", ["address,undefined", "thread"])
def test_host_side_of_the_library_under_sanitizers(tmp_path, sanitizers):
    exe = str(tmp_path / "host_driver")
    srcs = [os.path.join(CSRC, f) for f in ("ag_api.hip", "ag_sched.hip", "ag_pager.hip")] + [os.path.join(HB, "host_driver.cpp")]
    run_checked(["g++", "-std=c++17", "-g", "-O1", f"-fsanitize={sanitizers}", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
                 "-Wall", "-I" + HB, "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, "-x", "c++"] + srcs +
                ["-o", exe, "-pthread"])
    assert "host driver ok" in run_checked([exe])


def write_case(path, g, fill, chunk, rows):
    """One test case for the oracle program: a header of int32, the scale as float64, then the arrays."""
    hdr = np.array([g.dtype, g.num_pages, g.page_size, g.num_kv_heads, g.head_dim, g.num_q_heads, fill.batch,
                    fill.block_tables.shape[1], fill.total_new, chunk.total_new, len(rows[0])], np.int32)
    with open(path, "wb") as f:
        f.write(hdr.tobytes())
        f.write(np.float64(g.scale).tobytes())
        for b in (fill, chunk):
            for a in (b.block_tables, b.prefix_lens, b.new_lens, b.cu_new):
                f.write(np.ascontiguousarray(a, np.int32).tobytes())
            for a in (b.k_new, b.v_new, b.q):
                f.write(np.ascontiguousarray(a).tobytes())
        f.write(np.ascontiguousarray(rows[0], np.int32).tobytes())
        f.write(np.ascontiguousarray(rows[1], np.int32).tobytes())


@pytest.mark.parametrize("dtype", [I.F32, I.BF16])
def test_oracle_under_address_and_ub_sanitizers_equals_the_ordinary_build(tmp_path, dtype):
    exe = str(tmp_path / "oracle_san")
    run_checked(["gcc", "-std=c11", "-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                 "-fno-omit-frame-pointer", "-fopenmp", "-ffp-contract=off", "-Wall", "-Wextra",
                 os.path.join(ROOT, "oracle", "ag_oracle.c"), os.path.join(HB, "oracle_san_main.c"), "-o", exe, "-lm"])
    g = I.Geometry(6, 3, 24, 16, 40, dtype)
    prefix, new = [0, 5, 16, 33, 47], [1, 12, 17, 0, 30]              # page-crossing, mid-page starts, an empty session
    bt = I.deal_block_tables(I.rng_for(17, 0), [p + n for p, n in zip(prefix, new)], 16, g.num_pages)
    fill = make_batch(g, [0] * 5, prefix, seed=17, bt=bt)
    chunk = make_batch(g, prefix, new, seed=17, bt=bt, stream=2)
    rows = (np.array([0, 1, 1, 2, 4, 4], np.int32), np.array([0, 0, 11, 16, 0, 29], np.int32))
    case, res = str(tmp_path / "case.bin"), str(tmp_path / "out.bin")
    write_case(case, g, fill, chunk, rows)
    run_checked([exe, case, res])

    kp, vp = fresh_pools(g)
    for b in (fill, chunk):
        O.kv_append(kp, vp, g.dtype, b.k_new, b.v_new, b.block_tables, b.prefix_lens, b.new_lens, b.cu_new)
    full = O.attn(kp, vp, g.dtype, chunk.q, chunk.block_tables, chunk.prefix_lens, chunk.new_lens, chunk.cu_new,
                  g.num_q_heads, g.scale)
    some = O.attn(kp, vp, g.dtype, chunk.q, chunk.block_tables, chunk.prefix_lens, chunk.new_lens, chunk.cu_new,
                  g.num_q_heads, g.scale, rows=rows)
    raw = np.fromfile(res, dtype=np.uint8)
    pool_bytes = kp.nbytes
    got_k, got_v = raw[:pool_bytes], raw[pool_bytes:2 * pool_bytes]
    got_full = raw[2 * pool_bytes:2 * pool_bytes + full.nbytes].view(np.float64).reshape(full.shape)
    got_some = raw[2 * pool_bytes + full.nbytes:].view(np.float64).reshape(some.shape)
    assert np.array_equal(got_k, kp.view(np.uint8).ravel()) and np.array_equal(got_v, vp.view(np.uint8).ravel())
    assert np.array_equal(got_full.view(np.uint64), full.view(np.uint64))
    assert np.array_equal(got_some.view(np.uint64), some.view(np.uint64))
