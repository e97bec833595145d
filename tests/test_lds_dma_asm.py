"""The direct global-to-LDS loads (csrc/lds_dma.h) go through an asm statement that writes M0 itself and is not
modelled as an LDS write; their completion is waited for by hand.  This pins, in the code the compiler actually
generates for gfx950, what that relies on: M0 is written only by those statements, each write sits immediately
before its load, nothing else reads or writes M0, and every kernel that issues such loads also contains the
hand-placed vmcnt waits.  A compiler upgrade that breaks any of it fails here, on the CPU."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2603_10342_amd", "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

pytestmark = pytest.mark.skipif(not os.path.exists(HIPCC) and shutil.which("hipcc") is None, reason="needs hipcc")


def device_asm(src, tmp_path):
    out = str(tmp_path / (src + ".s"))
    from paper_2603_10342_amd import build as hip_build
    cmd = [HIPCC] + [f for f in hip_build.FLAGS if f != "-fPIC"] + ["--cuda-device-only", "-S", os.path.join(CSRC, src), "-o", out]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-3000:]
    return open(out).read()


@pytest.mark.parametrize("src", ["attn_prefill_mfma.hip", "attn_merged_mfma.hip"])
def test_m0_belongs_to_the_direct_loads_only(src, tmp_path):
    text = device_asm(src, tmp_path)
    # instruction lines only: no directives, labels, comments or metadata
    ins = []
    for line in text.splitlines():
        code = line.split(";")[0].strip()
        if not code or code.startswith(".") or code.endswith(":"):
            continue
        ins.append(code)
    loads = [i for i, c in enumerate(ins) if c.startswith("global_load_lds_dword")]     # the 16-byte and the 4-byte form
    assert len(loads) >= 8, "the direct loads are gone from the generated code?"
    for i in loads:
        assert re.match(r"s_mov_b32 m0, ", ins[i - 1]), (ins[i - 2:i + 1])
    m0_lines = [i for i, c in enumerate(ins) if re.search(r"\bm0\b", c)]
    assert m0_lines == [i - 1 for i in loads], [ins[i] for i in m0_lines if i + 1 not in loads][:5]
    # the waits that stand in for the compiler's own bookkeeping are present as written
    assert any(re.match(r"s_waitcnt vmcnt\(0\)", c) for c in ins)
    if src == "attn_prefill_mfma.hip":
        assert any(re.match(r"s_waitcnt vmcnt\([24]\)$", c) for c in ins), "the partial wait of the tile loop"
