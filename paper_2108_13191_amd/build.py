"""Build the HIP library (libgemm_f16.so) in-tree for gfx950 with hipcc."""
from __future__ import annotations

import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libgemm_f16.so")
SOURCES = ["gemm_api.hip", "gemm_generic.hip", "gemm_tiled.hip", "gemm_pingpong.hip", "gemm_overlap.hip", "gemm_w4.hip"]
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
         # packed-f32 VALU forms are kept off for every HIP file of this library
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def build(verbose: bool = False, extra=()) -> str:
    cmd = ["hipcc", *FLAGS, *extra, "-o", LIB, *[os.path.join(CSRC, s) for s in SOURCES]]
    if verbose:
        cmd.insert(1, "-Rpass-analysis=kernel-resource-usage")
    res = subprocess.run(cmd, capture_output=True, text=True)
    out = res.stdout + res.stderr
    if res.returncode != 0:
        sys.stderr.write(out)
        raise RuntimeError("hipcc failed")
    if verbose:
        print(resource_table(out))
    # measurement aid (MFMA-only throughput versus operand data), a stand-alone program
    probe = os.path.join(HERE, "probe_mfma_ceiling")
    subprocess.run(["hipcc", "-O3", "--offload-arch=gfx950", "-Wno-unused-command-line-argument",
                    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                    "-o", probe, os.path.join(CSRC, "probe_mfma_ceiling.hip")], check=True, capture_output=True)
    return LIB


def resource_table(text: str) -> str:
    rows, cur = [], {}
    for line in text.splitlines():
        m = re.search(r"remark:\s+(.+?) \[-Rpass", line)
        if not m:
            continue
        body = m.group(1).strip()
        if body.startswith("Function Name:"):
            if cur:
                rows.append(cur)
            cur = {"name": body.split(":", 1)[1].strip()}
        elif ":" in body:
            k, v = body.split(":", 1)
            cur[k.strip()] = v.strip()
    if cur:
        rows.append(cur)
    keys = ["VGPRs", "AGPRs", "TotalSGPRs", "ScratchSize [bytes/lane]", "Occupancy [waves/SIMD]",
            "SGPRs Spill", "VGPRs Spill", "LDS Size [bytes/block]"]
    lines = ["kernel | " + " | ".join(k.split(" [")[0] for k in keys)]
    for r in rows:
        name = subprocess.run(["c++filt", r["name"]], capture_output=True, text=True).stdout.strip() or r["name"]
        name = re.sub(r"\(anonymous namespace\)::", "", name)[:70]
        lines.append(name + " | " + " | ".join(r.get(k, "?") for k in keys))
    return "\n".join(lines)


if __name__ == "__main__":
    build(verbose=True)
    print("built", LIB)
