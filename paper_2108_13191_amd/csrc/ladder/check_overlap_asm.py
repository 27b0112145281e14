"""Build-time check of the generated code of gemm_overlap.hip (beside this file).

That kernel requests slabs of C with inline-assembly loads whose results are
used two k steps later, after a wait that the pipeline implies; the compiler is
told nothing about the latency.  This is only sound if no instruction touches a
destination register between the load ("; C slab load") and the marker the
kernel emits where the slab is known to have arrived ("; C slab arrived
<registers>").  `hazards()` scans the assembly hipcc produces for exactly that;
tests/test_abi_host.py runs it on every build of the test suite.

    python paper_2108_13191_amd/csrc/ladder/check_overlap_asm.py        # compiles to assembly and checks
"""
from __future__ import annotations

import os
import re
import subprocess
import sys
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
SOURCE = os.path.join(HERE, "gemm_overlap.hip")
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument", "-S", "--cuda-device-only"]


def _regs(text: str) -> set:
    out = set()
    for m in re.finditer(r"\bv\[(\d+):(\d+)\]|\bv(\d+)\b", text):
        if m.group(1):
            out |= set(range(int(m.group(1)), int(m.group(2)) + 1))
        else:
            out.add(int(m.group(3)))
    return out


def hazards(asm_text: str):
    """Return (number of marked C loads, list of offending lines).  Linear scan in
    program order: both sides of a branch are covered, a loop back edge is not
    (the kernel issues and consumes a slab in straight-line code)."""
    pending = {}                      # register -> line number of the load that targets it
    loads, bad = 0, []
    for no, line in enumerate(asm_text.split("\n"), 1):
        t = line.strip()
        if t.endswith(":") and t.startswith("_Z"):
            pending = {}              # next kernel
        if "C slab arrived" in t:
            for r in _regs(t):
                pending.pop(r, None)
            continue
        if not t or t.startswith(";") or t.startswith("."):
            continue
        if re.match(r"global_load_dwordx[24] ", t) and "C slab load" in t:
            loads += 1
            for r in _regs(t.split(",")[0]):
                pending[r] = no
            continue
        if t.startswith("s_waitcnt") and "vmcnt(0)" in t:
            pending = {}
            continue
        if pending:
            used = _regs(t.split(";")[0]) & set(pending)
            if used:
                bad.append((no, t, sorted(used)))
    return loads, bad


def compile_to_asm() -> str:
    with tempfile.TemporaryDirectory() as d:
        out = os.path.join(d, "gemm_overlap.s")
        subprocess.run(["hipcc", *FLAGS, "-o", out, SOURCE], check=True, capture_output=True)
        with open(out) as f:
            return f.read()


def main() -> int:
    loads, bad = hazards(compile_to_asm())
    for no, t, used in bad:
        print(f"line {no}: {t}   touches in-flight registers {used}")
    print(f"{loads} marked C loads, {len(bad)} hazards")
    return 1 if bad or loads == 0 else 0


if __name__ == "__main__":
    sys.exit(main())
