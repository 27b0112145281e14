"""bench.py's command-line contract: one GPU only; on a GPU, ONE JSON line on stdout with
the metric, the roofline object (algorithmic flops / measured launch time against the
published peak), the CPU-oracle baseline, and this build's additions (MFMA-only ceiling
on the workload's operand data, the other accumulate mode, the quarter means of the timed
series, the same protocol after an idle gap)."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode != 0 and "one GPU" in (res.stderr + res.stdout)


@pytest.mark.gpu
def test_one_json_line_with_roofline_and_cpu_baseline():
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "1", "--steps", "4", "--warmup", "2",
                          "--cpu-rows", "64"], capture_output=True, text=True, timeout=600)
    assert res.returncode == 0, res.stderr[-2000:]
    lines = [l for l in res.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    j = json.loads(lines[0])
    assert j["unit"] == "TFLOP/s" and j["n_gpus"] == 1 and j["steps"] == 4 and j["warmup"] == 2
    assert j["higher_is_better"] is True and j["data"] == "synthetic" and j["vs_baseline"] is None
    assert "8192" in j["metric"] and "sq8192_normal" in j["config"]["workload"]
    flops = 2 * 8192 ** 3
    assert abs(j["value"] - flops / (j["ms_per_step"] * 1e-3) / 1e12) <= 0.01 * j["value"]
    r = j["roofline"]
    assert r["bound"] == "mfma" and r["unit"] == "TFLOP/s" and r["peak"] == 2516.6 and r["flops"] == flops
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-3 and 0.05 < r["frac"] < 1.0
    assert abs(r["achieved"] - flops / (r["avg_launch_ms"] * 1e-3) / 1e12) <= 0.01 * r["achieved"]
    assert r["algorithmic_bytes"] == 2 * 2 * 8192 * 8192 + 2 * 4 * 8192 * 8192 and "kernel" in r and "traffic_source" in r
    c = j["cpu_baseline"]
    assert c["kind"] == "oracle" and c["unit"] == "TFLOP/s" and c["cores"] >= 1 and 0 < c["value"] < 1 and "rows" in c["sample"]
    ceil = j["mfma_only_ceiling"]
    assert j["value"] < ceil["value"] < 2516.6 and abs(ceil["value_over_ceiling"] - j["value"] / ceil["value"]) < 1e-3
    assert j["f16acc"]["value"] > 0 and len(j["series"]["quarter_means_ms"]) == 4 and j["after_idle"]["value"] > 0
