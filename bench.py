#!/usr/bin/env python3
"""Benchmark of the f16 GEMM hot path on one MI355X.

A step is one call of gemm_f16_f32acc on the headline workload (M = N = K =
8192, A and B ~ N(0,1)/sqrt(K) in f16, C f32 starting at zero and accumulating
over the steps): C tile -> accumulators, global -> LDS staging, MFMA main loop,
store.  Inputs are resident in HBM before the timed region.  Prints ONE JSON
line: TFLOP/s = 2 M N K / time, the roofline of the kernel measured with HIP
events on the launch stream, and the CPU oracle timed on a bounded row sample.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]
                    [--mode f32|f16] [--no-cpu] [--sweep]
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
    if tile_name.startswith("w4_"):
        return f"gemm_w4_kernel<{ct}>"
    if tile_name.startswith("generic"):
        return f"gemm_generic_kernel<{ct}>"
    # t<BM>x<BN>x64_w<WM>x<WN>: template arguments BM, BN, waves along m, along n, LDS stages, C type
    import re
    bm, bn, wm, wn = (int(x) for x in re.match(r"t(\d+)x(\d+)x\d+_w(\d+)x(\d+)", tile_name).groups())
    return f"gemm_tiled_kernel<{bm}, {bn}, {wm}, {wn}, {4 if bm == 64 else 2}, {ct}>"


def measured_traffic(tile_name, workload, mode):
    """HBM bytes per launch (FETCH_SIZE + WRITE_SIZE from rocprofv3 --pmc runs,
    scaled by a copy kernel of known size) if a committed profile summary under
    profiles/ records them for this kernel and workload; otherwise None."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{tile_name}_{workload}_{mode}.md")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return int(float(line.split(":", 1)[1].strip()))
    except OSError:
        pass
    return None


def time_gemm(binding, torch, mode, M, N, K, sets, steps, warmup):
    """Time `steps` launches; launch i works on sets[i % len(sets)] (one set: every
    launch re-reads the same operands, which the 256 MB last-level cache may still
    hold; several sets larger than that cache in total: every launch finds its
    operands in HBM only).  Return (ms per step, list of per-launch ms, host ms)."""
    fn = binding.gemm_f16_f32acc if mode == "f32" else binding.gemm_f16_f16acc
    stream = torch.cuda.current_stream()
    sp = stream.cuda_stream
    dA, dB, dC = sets[0]
    lda, ldb, ldc = dA.stride(0), dB.stride(0), dC.stride(0)
    R = len(sets)
    for i in range(warmup):
        a, b, c = sets[i % R]
        binding.check(fn(M, N, K, a, lda, b, ldb, c, ldc, sp))
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    evs[0].record(stream)
    for i in range(steps):
        a, b, c = sets[(warmup + i) % R]
        binding.check(fn(M, N, K, a, lda, b, ldb, c, ldc, sp))
        evs[i + 1].record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    per = [evs[i].elapsed_time(evs[i + 1]) for i in range(steps)]
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
    ap.add_argument("--warmup", type=int, default=40,
                    help="untimed launches first; the shader clock needs about 25 ms of work to settle after a pause")
    ap.add_argument("--workload", default="sq8192_normal")
    ap.add_argument("--mode", default="f32", choices=["f32", "f16"])
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--cpu-rows", type=int, default=4096, help="rows of C the oracle is timed on")
    ap.add_argument("--copy-probe", type=int, default=0, metavar="MiB",
                    help="instead of the GEMM, run plain device-to-device copies of this many MiB "
                         "(calibration of the FETCH_SIZE / WRITE_SIZE counters under rocprofv3)")
    ap.add_argument("--sweep", action="store_true", help="also time every workload and the square sweep (extra lines on stderr)")
    ap.add_argument("--force-config", type=int, default=-1)
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
    binding.load()
    binding.force_config(args.force_config)
    dev = torch.device("cuda:0")

    def run_workload(name, mode, steps, warmup, shape=None, rotate=False):
        if shape is None:
            M, N, K, dab, dc, _ = wl.WORKLOADS[name]
        else:
            M, N, K, dab, dc = (*shape, "uniform", "zeros")
        cdt = np.float32 if mode == "f32" else np.float16
        A, B, C0 = wl.make_inputs(M, N, K, dab, dc, seed=0, c_dtype=cdt)
        dA, dB, dC = (torch.from_numpy(x).to(dev) for x in (A, B, C0))
        sets = [(dA, dB, dC)]
        if rotate:
            for _ in range(rotation_sets(algorithmic_bytes(M, N, K, 4 if mode == "f32" else 2)) - 1):
                sets.append((dA.clone(), dB.clone(), dC.clone()))
        ms, per, wall = time_gemm(binding, torch, mode, M, N, K, sets, steps, warmup)
        cfg = binding.query_config(mode == "f16", M, N, K, dA, dA.stride(0), dB, dB.stride(0), dC, dC.stride(0))
        flops = 2.0 * M * N * K
        if cfg.get("split_rows"):
            cfg["plan"] = f"{cfg['name']} on rows 0..{cfg['split_rows'] - 1} + {binding.describe_config(cfg['id2'])['name']} on the rest"
        else:
            cfg["plan"] = cfg["name"]
        return dict(M=M, N=N, K=K, ms=ms, per=per, wall_ms=wall, tflops=flops / (ms * 1e-3) / 1e12, cfg=cfg, sets=len(sets),
                    bytes=algorithmic_bytes(M, N, K, 4 if mode == "f32" else 2)), (A, B, C0)

    # A problem whose operands fit the 256 MB last-level cache a few times over is
    # timed on rotating operand sets (every launch reads from HBM); the figure with
    # one set, re-read from the cache, is reported beside it.
    def small(m, n, k, mode):
        return algorithmic_bytes(m, n, k, 4 if mode == "f32" else 2) < ROTATE_BELOW_BYTES

    m0, n0, k0 = wl.WORKLOADS[args.workload][:3]
    rot = small(m0, n0, k0, args.mode) if args.rotate == "auto" else args.rotate == "on"
    r, (A, B, C0) = run_workload(args.workload, args.mode, args.steps, args.warmup, rotate=rot)
    same_set = run_workload(args.workload, args.mode, args.steps, args.warmup)[0] if rot and args.rotate == "auto" else None
    M, N, K = r["M"], r["N"], r["K"]
    per = sorted(r["per"])
    avg_launch_ms = sum(per) / len(per)
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
    roofline["traffic"] = measured_traffic(r["cfg"]["name"], args.workload, args.mode)
    kernels = kernel_symbol(r["cfg"]["name"], args.mode, K)
    if r["cfg"].get("split_rows"):          # two launches: the time below is that of the pair
        kernels += " + " + kernel_symbol(binding.describe_config(r["cfg"]["id2"])["name"], args.mode, K)
    roofline.update({"kernel": kernels, "avg_launch_ms": round(avg_launch_ms, 5),
                     "median_launch_ms": round(per[len(per) // 2], 5), "min_launch_ms": round(per[0], 5),
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

    out = {
        "metric": "TFLOP/s (2MNK/time), f16 GEMM " + ("f32" if args.mode == "f32" else "f16") + "-accumulate, M=N=K=8192"
                  if args.workload == "sq8192_normal" else f"TFLOP/s (2MNK/time), f16 GEMM {args.mode}-accumulate",
        "value": round(r["tflops"], 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(r["ms"], 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16 inputs, f32 accumulate" + ("" if args.mode == "f32" else ", f16 store"),
        "data": "synthetic", "pct_of_f16_mfma_peak": round(100 * r["tflops"] / PEAK_F16_MFMA_TFLOPS, 2),
        "config": {"workload": f"{args.workload}: M={M} N={N} K={K}, mode {args.mode}", "tile": r["cfg"]["plan"],
                   "grid": r["cfg"]["grid"], "host_wall_ms_per_step": round(r["wall_ms"], 5),
                   "operand_sets": r["sets"]},
        "roofline": roofline, "cpu_baseline": cpu,
    }

    if same_set is not None:
        out["same_operands_every_launch"] = {"value": round(same_set["tflops"], 2), "ms_per_step": round(same_set["ms"], 5)}

    if args.sweep:
        # every point gets the same treatment as the headline: about 25 ms of
        # untimed launches first (the first launches after a pause run at a lower
        # clock), then about 40 ms of timed ones
        def warm_run(name, mode, shape=None, rotate=False):
            probe, _ = run_workload(name, mode, 3, 2, shape)
            est = max(probe["ms"], 1e-3)
            return run_workload(name, mode, int(min(400, max(10, 40.0 / est))), int(min(400, max(3, 25.0 / est))), shape,
                                rotate=rotate)[0]

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
        for n in wl.SQUARE_SWEEP:
            for mode in ("f32", "f16"):
                point(f"square{n}", None, mode, n, n, n, shape=(n, n, n))
        out["sweep"] = extra

    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
