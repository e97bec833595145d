"""Builds the HIP library in-tree: paper_2603_10342_amd/libagattn.so (gfx950 only)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libagattn.so")
SOURCES = ["ag_api.hip", "kv_append.hip", "attn_general.hip", "attn_decode_mfma.hip", "attn_prefill_mfma.hip", "attn_merged_mfma.hip",
           "ag_sched.hip", "ag_pager.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-strict-aliasing", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",      # no packed-fp32 instructions
         "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def build(extra=(), verbose: bool = False, lib: str = LIB, tag: str = "") -> str:
    """Compile every source and link `lib`.  `extra` are added hipcc flags; `tag` keeps the objects of a second
    build (another output path) apart."""
    global OBJ
    obj_dir = OBJ + tag
    os.makedirs(obj_dir, exist_ok=True)

    def comp(src):
        obj = os.path.join(obj_dir, src.replace(".hip", ".o"))
        cmd = [HIPCC] + FLAGS + list(extra) + ["-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
        if r.returncode:
            raise RuntimeError(f"hipcc failed on {src}:\n{err}")
        if err.strip():
            sys.stderr.write(err + "\n")
        return obj

    with ThreadPoolExecutor(len(SOURCES)) as ex:
        objs = list(ex.map(comp, SOURCES))
    LIBP = lib
    tmp = LIBP + f".tmp{os.getpid()}"
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode:
        raise RuntimeError("link failed:\n" + r.stderr)
    os.replace(tmp, LIBP)
    if verbose:
        print("built", LIBP)
    return LIBP


if __name__ == "__main__":
    build(extra=sys.argv[1:], verbose=True)
