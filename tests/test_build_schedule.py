"""Host-side guard on the compiled row loops (no GPU needed): every kernel that streams weight
rows must keep its batch of row loads in flight together.  The instruction scheduler has, for
some template instantiations, paired each load with a full wait of its own (one row in flight
instead of eight), which costs a third of the streaming rate and no test of results can see it.
The check compiles the kernel sources to assembly with the library's own flags and looks at what
follows every non-temporal row load."""
import os
import re
import subprocess
from concurrent.futures import ThreadPoolExecutor

import pytest

from paper_2504_08378_amd import build

SOURCES = ["gemv_f16.hip", "gemv_q4.hip", "union.hip", "layer.hip"]


def _assembly(src, tmp):
    out = os.path.join(tmp, src.replace(".hip", ".s"))
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in build.HIPCC_FLAGS if f != "-fPIC"]
    cmd = [hipcc, *flags, "-I", os.path.join(build.ROOT, "include"), "-I", build.CSRC,
           "--cuda-device-only", "-S", os.path.join(build.CSRC, src), "-o", out]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout[-2000:]
    return open(out).read().split("\n")


def _serialized_row_loads(lines):
    """{kernel: (row loads, row loads directly followed by s_waitcnt vmcnt(0))}"""
    res, cur = {}, None
    for i, l in enumerate(lines):
        m = re.match(r"^(_Z\w+):", l)
        if m:
            cur = m.group(1)
            res[cur] = [0, 0]
        if cur and "global_load_dword" in l and l.rstrip().endswith(" nt"):
            res[cur][0] += 1
            j = i + 1
            while j < len(lines) and (not lines[j].strip() or lines[j].strip().startswith(";")):
                j += 1
            if j < len(lines) and "s_waitcnt vmcnt(0)" in lines[j]:
                res[cur][1] += 1
    return {k: tuple(v) for k, v in res.items() if v[0]}


@pytest.mark.skipif(not os.path.exists(os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")), reason="no hipcc")
def test_row_loads_stay_in_flight_together(tmp_path):
    with ThreadPoolExecutor(4) as ex:
        asm = list(ex.map(lambda s: _assembly(s, str(tmp_path)), SOURCES))
    seen = 0
    for src, lines in zip(SOURCES, asm):
        stats = _serialized_row_loads(lines)
        assert stats, f"{src}: no row loads found (did the load marker change?)"
        for kernel, (n, bad) in stats.items():
            seen += 1
            # a masked tail batch may end in one such pair; a serialized loop has one per row
            assert bad <= 2, f"{src}: {kernel} waits after {bad} of its {n} row loads"
    assert seen >= 40
