#!/usr/bin/env python3
"""Benchmark of the f16 GEMM hot path on one MI355X.

A step is one call of gemm_f16_f32acc on the headline workload (M = N = K =
8192, A and B ~ N(0,1)/sqrt(K) in f16, C f32 starting at zero and accumulating
over the steps): C tile -> accumulators, global -> LDS staging, MFMA main loop,
store.  Inputs are resident in HBM before the timed region.  Prints ONE JSON
line: TFLOP/s = 2 M N K / time, the roofline of the kernel measured with HIP
events on the launch stream, and the CPU oracle timed on a bounded row sample.

Order of the legs of a default run, all on one stream and without a pause between
the first three: (1) an MFMA-only loop on operands drawn from the workload's own
distribution, about 45 ms -- the throughput the matrix units sustain on that data
before a single byte moves (`mfma_only_ceiling`); (2) the headline: W untimed and
exactly K timed f32-accumulate calls (`value`); (3) the same for the
f16-accumulate mode (`f16acc`); (4) the CPU oracle; (5) the headline protocol once
more right after the GPU has sat idle under (4) (`after_idle`): the part's power
management answers a load step with a transient of about 25 launches (two fast
ones, five about 30 % slow, a slow recovery), which is all a 5 + 20 launch run
sees when it starts cold.  `value` is the steady state; `after_idle` and the
quarter means of the timed series (`series`) show the transient and any drift.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]
                    [--mode f32|f16] [--no-cpu] [--sweep] [--cold]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_F16_MFMA_TFLOPS = 2516.6      # 256 CU x 4096 flop/clk/CU x 2.4 GHz, dense
ROTATE_BELOW_BYTES = 512 << 20   # operands + C of one call; the last-level cache holds 256 MB
PEAK_HBM_GBS = 8000.0


def algorithmic_bytes(M, N, K, c_bytes):
    """A and B read once (f16), C read once and written once."""
    return 2 * (M * K + K * N) + 2 * M * N * c_bytes


def kernel_symbol(tile_name, mode, K=0):
    """Name of the kernel as it shows in a rocprofv3 kernel trace."""
    ct = "float" if mode == "f32" else "_Float16"
    if tile_name.startswith("pp"):
        mi = 16 if "mi16" in tile_name else 32
        bm, bn = int(tile_name[2:5]), int(tile_name[6:9])
        tail = "true" if K % 64 else "false"
        if tile_name.endswith("_chain"):
            return f"gemm_pp256_persistent_kernel<{ct}, {mi}, {tail}>"
        if tile_name.endswith("_stag"):
            return f"gemm_pp_mixed_kernel<{ct}, {mi}, {tail}>"
        return f"gemm_pp256_kernel<{ct}, {mi}, {'true' if K % 64 else 'false'}, {bm}, {bn}>"
    if tile_name.startswith("ov"):
        return f"gemm_pp_overlap_kernel<{ct}>"
    if tile_name.startswith("w4a_128"):
        return f"gemm_w4a128_kernel<{ct}>"
    if tile_name.startswith("w4a_"):
        return f"gemm_w4a_kernel<{ct}>"
    if tile_name.startswith("w4_"):
        return f"gemm_w4_kernel<{ct}>"
    if tile_name.startswith("il"):
        return f"gemm_il256_kernel<{ct}>"
    if tile_name.startswith("generic"):
        return f"gemm_generic_kernel<{ct}, {'true' if tile_name.endswith('_c_in_loop') else 'false'}>"
    # t<BM>x<BN>x64_w<WM>x<WN>: template arguments BM, BN, waves along m, along n, LDS stages, C type
    import re
    bm, bn, wm, wn = (int(x) for x in re.match(r"t(\d+)x(\d+)x\d+_w(\d+)x(\d+)", tile_name).groups())
    return f"gemm_tiled_kernel<{bm}, {bn}, {wm}, {wn}, {4 if bm == 64 else 2}, {ct}, {'false' if tile_name.endswith('_noswz') else 'true'}>"


def measured_traffic(tile_name, workload, mode):
    """HBM bytes per launch (FETCH_SIZE + WRITE_SIZE from rocprofv3 --pmc runs,
    scaled by a copy kernel of known size) if a committed profile summary under
    profiles/ records them for this kernel and workload, and where the figure comes
    from; (None, reason) otherwise.  Counters cannot be read from inside this
    program: the figure is the committed one, not one of this run."""
    rel = os.path.join("profiles", f"hbm_traffic_{tile_name}_{workload}_{mode}.md")
    try:
        for line in open(os.path.join(ROOT, rel)):
            if line.startswith("traffic_bytes_per_launch:"):
                return int(float(line.split(":", 1)[1].strip())), f"{rel} (rocprofv3 --pmc runs of this command, committed; not measured in this run)"
    except OSError:
        pass
    return None, "no committed counter run for this kernel and workload"


PROBE_LIB = os.path.join(ROOT, "libbench_probe.so")


def build_probe():
    """Compile bench_probe.hip (the MFMA-only loop) next to this file."""
    import subprocess
    subprocess.run(["hipcc", "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
                    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
                    "-o", PROBE_LIB, os.path.join(ROOT, "bench_probe.hip")], check=True, capture_output=True)
    return PROBE_LIB


def mfma_only_ceiling(torch, np, wl, dist, K, seconds=0.045):
    """TFLOP/s of a loop of nothing but v_mfma_f32_16x16x32_f16 (two wavefronts per SIMD, the
    library's register blocking, operands in registers) on f16 operands drawn from `dist`,
    the workload's distribution: the data-dependent, power-limited ceiling of the matrix
    units.  Runs about `seconds` in three launches; the figure is the last launch's."""
    import ctypes
    if not os.path.exists(PROBE_LIB):
        build_probe()
    lib = ctypes.CDLL(PROBE_LIB)
    lib.bench_mfma_only.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
    lib.bench_mfma_only.restype = ctypes.c_int
    rng = np.random.default_rng(0)
    frags = torch.from_numpy(wl.draw(rng, (12 * 256, 8), dist, K).astype(np.float16)).cuda()
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    stream = torch.cuda.current_stream()

    def run(iters):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        rc = lib.bench_mfma_only(frags.data_ptr(), sink.data_ptr(), iters, cus, stream.cuda_stream)
        e1.record(stream)
        if rc != 0:
            raise RuntimeError(f"bench_mfma_only returned {rc}")
        return e0, e1, iters

    e0, e1, it = run(2000)
    torch.cuda.synchronize()
    per_iter_ms = max(e0.elapsed_time(e1) / it, 1e-7)
    iters = int(max(1000, seconds / 3 * 1e3 / per_iter_ms))
    launches = [run(iters) for _ in range(3)]          # queued back to back; the caller's next leg follows without a pause
    return launches, cus


def loop_budget(torch, np, wl, dist, K, seconds=0.03):
    """bench_probe.hip's three hand-scheduled loops (MFMAs only; + the LDS fragment reads of the
    library's main loop; + its global -> LDS copies from L2) on operands drawn from `dist`: TFLOP/s
    of each, the second of two launches of about `seconds`."""
    import ctypes
    if not os.path.exists(PROBE_LIB):
        build_probe()
    lib = ctypes.CDLL(PROBE_LIB)
    lib.bench_loop_budget.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
    lib.bench_loop_budget.restype = ctypes.c_int
    rng = np.random.default_rng(0)
    data = torch.from_numpy(wl.draw(rng, (32768,), dist, K).astype(np.float16)).cuda()      # 64 KB
    sink = torch.zeros(1, dtype=torch.float32, device="cuda")
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    stream = torch.cuda.current_stream()
    out = {}
    for variant, name in ((0, "mfma_only"), (1, "with_lds_reads"), (2, "with_lds_reads_and_copies")):
        iters = 2000
        for rep in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            rc = lib.bench_loop_budget(data.data_ptr(), sink.data_ptr(), variant, iters, cus, stream.cuda_stream)
            e1.record(stream)
            torch.cuda.synchronize()
            if rc != 0:
                raise RuntimeError(f"bench_loop_budget returned {rc}")
            ms = e0.elapsed_time(e1)
            if rep == 0:
                iters = int(max(2000, seconds * 1e3 / max(ms / iters, 1e-7)))
        out[name] = round(float(cus) * 8 * iters * 32 * 16384 / (ms * 1e-3) / 1e12, 1)
    return out


def ceiling_result(launches, cus):
    e0, e1, iters = launches[-1]
    ms = e0.elapsed_time(e1)
    flops = float(cus) * 8 * iters * 32 * 16384
    return {"value": round(flops / (ms * 1e-3) / 1e12, 1), "unit": "TFLOP/s", "ms": round(ms, 3),
            "frac_of_peak": round(flops / (ms * 1e-3) / 1e12 / PEAK_F16_MFMA_TFLOPS, 4),
            "what": "v_mfma_f32_16x16x32_f16 only, two wavefronts per SIMD, 8 x 4 accumulator blocks per wavefront "
                    "walked in the library's order (one operand changes per MFMA), "
                    "operands in registers drawn from the workload's distribution; last of three back-to-back launches"}


def time_gemm(binding, torch, mode, M, N, K, sets, steps, warmup):
    """Time `steps` launches; launch i works on sets[i % len(sets)] (one set: every
    launch re-reads the same operands, which the 256 MB last-level cache may still
    hold; several sets larger than that cache in total: every launch finds its
    operands in HBM only).  Return (ms per step, mean launch ms of each quarter of the
    timed series, host ms per step)."""
    fn = binding.gemm_f16_f32acc if mode == "f32" else binding.gemm_f16_f16acc
    stream = torch.cuda.current_stream()
    sp = stream.cuda_stream
    if mode == "f16ws":         # the f16 mode with M x N floats of lent scratch memory (skinny problems: split k)
        ws_bytes = max(binding.gemm_f16_f16acc_workspace_bytes(M, N, K), 16)
        ws = torch.empty(ws_bytes // 4, dtype=torch.float32, device=sets[0][0].device)

        def fn(M, N, K, a, lda, b, ldb, c, ldc, sp):
            return binding.gemm_f16_f16acc_workspace(M, N, K, a, lda, b, ldb, c, ldc, ws, ws_bytes, sp)
    dA, dB, dC = sets[0]
    lda, ldb, ldc = dA.stride(0), dB.stride(0), dC.stride(0)
    R = len(sets)
    for i in range(warmup):
        a, b, c = sets[i % R]
        binding.check(fn(M, N, K, a, lda, b, ldb, c, ldc, sp))
    # events at the quarter points only: an event between two launches costs a few microseconds,
    # which is nothing for the headline and a third of the time of the smallest problems
    marks = sorted({(steps * q) // 4 for q in range(5)})
    evs = {m: torch.cuda.Event(enable_timing=True) for m in marks}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    evs[0].record(stream)
    for i in range(steps):
        a, b, c = sets[(warmup + i) % R]
        binding.check(fn(M, N, K, a, lda, b, ldb, c, ldc, sp))
        if i + 1 in evs:
            evs[i + 1].record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    per = [evs[a].elapsed_time(evs[b]) / (b - a) for a, b in zip(marks[:-1], marks[1:])]     # mean launch time per quarter
    total = evs[0].elapsed_time(evs[steps])
    return total / steps, per, wall_ms / steps


def rotation_sets(nbytes):
    """Number of operand sets to rotate through so that a set has left the 256 MB
    last-level cache before its turn comes again: at least 3, at least 1 GiB in
    total, at most 64."""
    return int(min(64, max(3, -(-(1 << 30) // max(nbytes, 1)))))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10, help="untimed launches in front of the timed ones")
    ap.add_argument("--cold", action="store_true",
                    help="leave out the MFMA-only leg in front of the timed region (the timed launches then "
                         "start on an idle GPU and show the transient of its power management)")
    ap.add_argument("--workload", default="sq8192_normal")
    ap.add_argument("--shape", default=None, metavar="M,N,K",
                    help="instead of a named workload: this shape with A, B ~ U[-1,1] and C zero (as the square sweep's points)")
    ap.add_argument("--mode", default="f32", choices=["f32", "f16"])
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--cpu-rows", type=int, default=4096, help="rows of C the oracle is timed on")
    ap.add_argument("--copy-probe", type=int, default=0, metavar="MiB",
                    help="instead of the GEMM, run plain device-to-device copies of this many MiB "
                         "(calibration of the FETCH_SIZE / WRITE_SIZE counters under rocprofv3)")
    ap.add_argument("--loop-budget", action="store_true",
                    help="instead of the GEMM, run bench_probe.hip's three hand-scheduled loops (MFMAs only; + LDS "
                         "fragment reads; + global -> LDS copies) on the workload's operand distribution")
    ap.add_argument("--sweep", action="store_true", help="also time every workload and the square sweep (extra lines on stderr)")
    ap.add_argument("--force-config", default="-1", metavar="ID|NAME",
                    help="run this configuration of the library's table instead of the selected one")
    ap.add_argument("--no-idle-leg", action="store_true", help="leave out the repeat of the protocol after an idle gap")
    ap.add_argument("--ladder", action="store_true", help="use libgemm_f16_ladder.so (for --force-config on a comparison kernel)")
    ap.add_argument("--rotate", default="auto", choices=["auto", "on", "off"],
                    help="launch i works on operand set i mod R (R sets, 1 GiB or more in total), so that no launch finds "
                         "its operands in the last-level cache; auto: for problems under 512 MiB, and the same-set "
                         "figure is reported beside it")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1")

    import numpy as np
    import torch
    from paper_2108_13191_amd import binding, workloads as wl

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    if args.copy_probe:
        n = args.copy_probe << 20
        src = torch.empty(n, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(args.warmup + args.steps):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe_bytes_read_per_copy": n, "copy_probe_bytes_written_per_copy": n,
                          "copies": args.warmup + args.steps}))
        return
    if args.loop_budget:
        dist, k = wl.WORKLOADS[args.workload][3], wl.WORKLOADS[args.workload][2]
        res = loop_budget(torch, np, wl, dist, k)
        print(json.dumps({"loop_budget": res, "unit": "TFLOP/s", "workload": args.workload, "operands": dist,
                          "what": "32 v_mfma_f32_16x16x32_f16 per wavefront and iteration, two wavefronts per SIMD, "
                                  "hand-scheduled: alone; + 8 ds_read_b128 and 8 ds_read_b64_tr_b16; + 4 global_load_lds_dwordx4 from L2"}))
        return
    if args.ladder:
        binding._active = "ladder"          # the library that also holds the comparison kernels (same selection)
    binding.load()
    forced = args.force_config
    if not forced.lstrip("-").isdigit():
        names = [binding.describe_config(i)["name"] for i in range(binding.num_configs())]
        if forced not in names:
            sys.exit(f"bench.py: no configuration named {forced!r}; the table holds {names}")
        forced = names.index(forced)
    binding.force_config(int(forced))
    dev = torch.device("cuda:0")

    def prepare(name, mode, shape=None, rotate=False, host=None):
        """Operands of a workload on the device (R rotating sets if `rotate`); `host` reuses
        the A and B another mode's call has drawn."""
        if shape is None:
            M, N, K, dab, dc, _ = wl.WORKLOADS[name]
        else:
            M, N, K, dab, dc = (*shape, "uniform", "zeros")
        cdt = np.float32 if mode == "f32" else np.float16
        if host is None:
            A, B, C0 = wl.make_inputs(M, N, K, dab, dc, seed=0, c_dtype=cdt)
        else:
            A, B, C0 = host[0], host[1], host[2].astype(cdt)
        dA, dB, dC = (torch.from_numpy(x).to(dev) for x in (A, B, C0))
        sets = [(dA, dB, dC)]
        if rotate:
            for _ in range(rotation_sets(algorithmic_bytes(M, N, K, 4 if mode == "f32" else 2)) - 1):
                sets.append((dA.clone(), dB.clone(), dC.clone()))
        return dict(M=M, N=N, K=K, mode=mode, sets=sets, host=(A, B, C0), dist=dab)

    def timed(prep, steps, warmup):
        M, N, K, mode, sets = prep["M"], prep["N"], prep["K"], prep["mode"], prep["sets"]
        ms, per, wall = time_gemm(binding, torch, mode, M, N, K, sets, steps, warmup)
        dA, dB, dC = sets[0]
        cfg = binding.query_config(mode != "f32", M, N, K, dA, dA.stride(0), dB, dB.stride(0), dC, dC.stride(0))
        if mode == "f16ws" and binding.gemm_f16_f16acc_workspace_bytes(M, N, K) > 0:
            cfg["name"] = "w4a_128x128x64, k loop in parts through a workspace of M x N floats"
        flops = 2.0 * M * N * K
        if cfg.get("split_rows"):
            cfg["plan"] = f"{cfg['name']} on rows 0..{cfg['split_rows'] - 1} + {binding.describe_config(cfg['id2'])['name']} on the rest"
        else:
            cfg["plan"] = cfg["name"]
        return dict(M=M, N=N, K=K, ms=ms, per=per, wall_ms=wall, tflops=flops / (ms * 1e-3) / 1e12, cfg=cfg, sets=len(sets),
                    bytes=algorithmic_bytes(M, N, K, 4 if mode == "f32" else 2))

    def quarters(per):
        """Mean launch time of the first and of the last quarter of the timed series (as launched)."""
        return {"first_quarter_ms": round(per[0], 5), "last_quarter_ms": round(per[-1], 5),
                "quarter_means_ms": [round(x, 5) for x in per]}

    # A problem whose operands fit the 256 MB last-level cache a few times over is
    # timed on rotating operand sets (every launch reads from HBM); the figure with
    # one set, re-read from the cache, is reported beside it.
    def small(m, n, k, mode):
        return algorithmic_bytes(m, n, k, 4 if mode == "f32" else 2) < ROTATE_BELOW_BYTES

    shape = tuple(int(x) for x in args.shape.split(",")) if args.shape else None
    if shape:
        args.workload = "shape" + "x".join(str(x) for x in shape)
        wl.WORKLOADS[args.workload] = (*shape, "uniform", "zeros", ("f32", "f16"))
    m0, n0, k0 = wl.WORKLOADS[args.workload][:3]
    modes = wl.WORKLOADS[args.workload][5]
    other = {"f32": "f16", "f16": "f32"}[args.mode]
    rot = small(m0, n0, k0, args.mode) if args.rotate == "auto" else args.rotate == "on"
    # everything on the device before the first timed leg, so that the legs follow each other without a pause
    prep = prepare(args.workload, args.mode, rotate=rot)
    prep_other = prepare(args.workload, other, rotate=rot, host=prep["host"]) if other in modes else None
    prep_same = prepare(args.workload, args.mode, host=prep["host"]) if rot and args.rotate == "auto" else None
    A, B, C0 = prep["host"]
    launches = None if args.cold else mfma_only_ceiling(torch, np, wl, prep["dist"], k0)
    r = timed(prep, args.steps, args.warmup)
    r_other = timed(prep_other, args.steps, args.warmup) if prep_other else None
    same_set = timed(prep_same, args.steps, args.warmup) if prep_same else None
    M, N, K = r["M"], r["N"], r["K"]
    avg_launch_ms = r["ms"]             # HIP events around the timed launches on the launch stream / launches
    achieved = 2.0 * M * N * K / (avg_launch_ms * 1e-3) / 1e12
    t_mfma = 2.0 * M * N * K / (PEAK_F16_MFMA_TFLOPS * 1e12)
    t_hbm = r["bytes"] / (PEAK_HBM_GBS * 1e9)
    if t_mfma >= t_hbm:
        roofline = {"bound": "mfma", "achieved": round(achieved, 2), "peak": PEAK_F16_MFMA_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(achieved / PEAK_F16_MFMA_TFLOPS, 4), "traffic": None}
    else:
        gbs = r["bytes"] / (avg_launch_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": round(gbs / PEAK_HBM_GBS, 4), "traffic": None}
    roofline["traffic"], roofline["traffic_source"] = measured_traffic(r["cfg"]["name"], args.workload, args.mode)
    kernels = kernel_symbol(r["cfg"]["name"], args.mode, K)
    if r["cfg"].get("split_rows"):          # two launches: the time below is that of the pair
        kernels += " + " + kernel_symbol(binding.describe_config(r["cfg"]["id2"])["name"], args.mode, K)
    roofline.update({"kernel": kernels, "avg_launch_ms": round(avg_launch_ms, 5),
                     "algorithmic_bytes": r["bytes"], "flops": 2 * M * N * K})

    cpu = None
    if not args.no_cpu:
        import oracle
        nrows = min(args.cpu_rows, M)
        rows = np.arange(nrows, dtype=np.int64)
        t0 = time.perf_counter()
        oracle.gemm_f16(A, B, C0, rows=rows)
        dt = time.perf_counter() - t0
        cpu = {"value": round(2.0 * nrows * N * K / dt / 1e12, 6), "unit": "TFLOP/s", "cores": oracle.num_threads(),
               "kind": "oracle", "seconds": round(dt, 2),
               "sample": f"first {nrows} of {M} rows of C (all {N} columns, full K={K}) of the same workload, "
                         f"binary64 triple loop incl. decoding B; host has {os.cpu_count()} logical CPUs"}
    # the same protocol once more after the GPU has been idle (under the CPU leg, or for a second)
    idle = None
    if not args.no_idle_leg:
        if args.no_cpu:
            time.sleep(1.0)
        idle = timed(prep, args.steps, args.warmup)

    out = {
        "metric": "TFLOP/s (2MNK/time), f16 GEMM " + ("f32" if args.mode == "f32" else "f16") + "-accumulate, M=N=K=8192"
                  if args.workload == "sq8192_normal" else f"TFLOP/s (2MNK/time), f16 GEMM {args.mode}-accumulate",
        "value": round(r["tflops"], 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(r["ms"], 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16 inputs, f32 accumulate" + ("" if args.mode == "f32" else ", f16 store"),
        "data": "synthetic", "pct_of_f16_mfma_peak": round(100 * r["tflops"] / PEAK_F16_MFMA_TFLOPS, 2),
        "config": {"workload": f"{args.workload}: M={M} N={N} K={K}, mode {args.mode}", "tile": r["cfg"]["plan"],
                   "grid": r["cfg"]["grid"], "host_wall_ms_per_step": round(r["wall_ms"], 5),
                   "operand_sets": r["sets"],
                   "timed_region": ("starts cold (--cold)" if args.cold else
                                    "follows the MFMA-only leg and the warm-up launches without a pause (steady state)")},
        "roofline": roofline, "cpu_baseline": cpu,
        "series": quarters(r["per"]),
    }
    if idle is not None:
        out["after_idle"] = {"value": round(idle["tflops"], 2), "ms_per_step": round(idle["ms"], 5), **quarters(idle["per"]),
                             "what": "the same W + K launches started right after the GPU sat idle (under the CPU leg, or "
                                     "for a second): the transient of the part's power management, not the kernel"}
    if launches is not None:
        ceil = ceiling_result(*launches)
        ceil["value_over_ceiling"] = round(r["tflops"] / ceil["value"], 4)
        out["mfma_only_ceiling"] = ceil
    if r_other is not None:
        out[other + "acc"] = {"value": round(r_other["tflops"], 2), "ms_per_step": round(r_other["ms"], 5),
                              "frac": round(r_other["tflops"] / PEAK_F16_MFMA_TFLOPS, 4), "tile": r_other["cfg"]["plan"],
                              **quarters(r_other["per"])}

    if same_set is not None:
        out["same_operands_every_launch"] = {"value": round(same_set["tflops"], 2), "ms_per_step": round(same_set["ms"], 5)}

    if args.sweep:
        # every point gets the same treatment as the headline: about 25 ms of
        # untimed launches first (the first launches after a pause run at a lower
        # clock), then about 40 ms of timed ones
        def warm_run(name, mode, shape=None, rotate=False):
            pr = prepare(name, mode, shape, rotate)
            est = max(timed(pr, 3, 2)["ms"], 1e-3)
            return timed(pr, int(min(400, max(10, 40.0 / est))), int(min(400, max(3, 25.0 / est))))

        extra = []

        def point(label, name, mode, m, n, k, shape=None):
            rr = warm_run(name, mode, shape)
            row = {"workload": label, "mode": mode, "M": m, "N": n, "K": k, "ms": round(rr["ms"], 5),
                   "tflops": round(rr["tflops"], 1), "pct_peak": round(100 * rr["tflops"] / PEAK_F16_MFMA_TFLOPS, 1),
                   "gbs": round(rr["bytes"] / (rr["ms"] * 1e-3) / 1e9, 1), "tile": rr["cfg"]["plan"]}
            # fraction of the roofline time max(flops / MFMA peak, algorithmic bytes / HBM peak)
            t_roof = max(2.0 * m * n * k / (PEAK_F16_MFMA_TFLOPS * 1e12), rr["bytes"] / (PEAK_HBM_GBS * 1e9))
            row["roofline_frac"] = round(t_roof / (rr["ms"] * 1e-3), 4)
            if small(m, n, k, mode):            # the same point with every launch reading from HBM
                rc = warm_run(name, mode, shape, rotate=True)
                row.update({"rotated_sets": rc["sets"], "rotated_ms": round(rc["ms"], 5), "rotated_tflops": round(rc["tflops"], 1),
                            "rotated_roofline_frac": round(t_roof / (rc["ms"] * 1e-3), 4),
                            "rotated_gbs": round(rc["bytes"] / (rc["ms"] * 1e-3) / 1e9, 1)})
            extra.append(row)
            print(json.dumps(row), file=sys.stderr, flush=True)

        for name, (m, n, k, _, _, modes) in wl.WORKLOADS.items():
            for mode in modes:
                point(name, name, mode, m, n, k)
                if mode == "f16" and binding.gemm_f16_f16acc_workspace_bytes(m, n, k) > 0:
                    point(name, name, "f16ws", m, n, k)           # gemm_f16_f16acc_workspace on the same problem
        for n in wl.SQUARE_SWEEP:
            for mode in ("f32", "f16"):
                point(f"square{n}", None, mode, n, n, n, shape=(n, n, n))
        out["sweep"] = extra

    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
