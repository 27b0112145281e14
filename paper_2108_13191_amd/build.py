"""Build the HIP libraries in-tree for gfx950 with hipcc.

libgemm_f16.so         the product: the C ABI of include/gemm_f16.h and the kernels it selects
libgemm_f16_ladder.so  the same sources compiled with -DGEMM_F16_LADDER plus csrc/ladder/*.hip: the
                       comparison kernels and ablation rows appended to the configuration table
                       (never selected; tests and profiles reach them by forcing their ids)
"""
from __future__ import annotations

import concurrent.futures
import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libgemm_f16.so")
LADDER_LIB = os.path.join(HERE, "libgemm_f16_ladder.so")
SOURCES = ["gemm_api.hip", "gemm_generic.hip", "gemm_tiled.hip", "gemm_pingpong.hip", "gemm_w4a.hip", "gemm_w4a128.hip", "gemm_splitk_f16.hip"]
LADDER_SOURCES = ["ladder/gemm_w4.hip", "ladder/gemm_overlap.hip", "ladder/gemm_interleaved.hip"]
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
         # packed-f32 VALU forms are kept off for every HIP file of this library
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def _compile(src: str, obj: str, extra, verbose: bool) -> str:
    cmd = ["hipcc", *FLAGS, *extra, "-c", "-o", obj, os.path.join(CSRC, src)]
    if verbose:
        cmd.insert(1, "-Rpass-analysis=kernel-resource-usage")
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stdout + res.stderr)
        raise RuntimeError(f"hipcc failed on {src}")
    return res.stdout + res.stderr


def build(verbose: bool = False, ladder: bool = True, extra=()) -> str:
    """Compile every source (in parallel) and link the product library and, with `ladder`,
    the ladder library.  Returns the product library's path."""
    os.makedirs(OBJ, exist_ok=True)
    jobs = [(s, os.path.join(OBJ, s.replace("/", "_") + ".o"), list(extra)) for s in SOURCES]
    if ladder:
        jobs += [(s, os.path.join(OBJ, s.replace("/", "_") + ".ladder.o"), ["-DGEMM_F16_LADDER", *extra])
                 for s in SOURCES + LADDER_SOURCES]
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
        logs = list(pool.map(lambda j: _compile(j[0], j[1], j[2], verbose), jobs))
    link = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-Wno-unused-command-line-argument"]
    subprocess.run([*link, "-o", LIB, *[j[1] for j in jobs[:len(SOURCES)]]], check=True)
    if ladder:
        subprocess.run([*link, "-o", LADDER_LIB, *[j[1] for j in jobs[len(SOURCES):]]], check=True)
    if verbose:
        print(resource_table("".join(logs[:len(SOURCES)])))
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
    print("built", LIB, "and", LADDER_LIB)
