"""The bench line is what the measurements are read from: one JSON object on stdout with the
agreed keys, the roofline and the CPU baseline beside the value.  Runs bench.py as a program (a
short run of the headline leg and the per-config table) and checks the shape of what it prints."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_prints_one_json_line_with_roofline_and_cpu_baseline():
    cmd = [sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "50", "--warmup", "10", "--cpu-seconds", "3",
           "--no-trace", "--no-cache-ops", "--no-mask-select", "--no-joint", "--no-mfma-probe"]
    res = subprocess.run(cmd, capture_output=True, text=True, timeout=280, cwd=ROOT)
    assert res.returncode == 0, res.stderr[-2000:]
    lines = [l for l in res.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, lines
    d = json.loads(lines[0])
    for key, typ in (("metric", str), ("value", float), ("unit", str), ("n_gpus", int), ("steps", int), ("warmup", int),
                     ("ms_per_step", float), ("higher_is_better", bool), ("scaling", str), ("dtype", str), ("data", str),
                     ("config", dict), ("roofline", dict), ("cpu_baseline", dict), ("configs", list)):
        assert isinstance(d[key], typ), (key, d[key])
    assert d["n_gpus"] == 1 and d["steps"] == 50 and d["warmup"] == 10 and d["higher_is_better"] is True
    assert d["vs_baseline"] is None and d["dtype"] == "bf16" and "workload" in d["config"] and "model" not in d["config"]
    r = d["roofline"]
    assert r["bound"] == "mfma" and r["unit"] == "TFLOP/s" and r["peak"] == 2500.0
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-3 and 0.2 < r["frac"] < 1.0
    assert abs(d["value"] - r["achieved"]) / d["value"] < 0.15          # same region, two clocks
    assert r["traffic"] is None or r["traffic"] >= r["algorithmic_bytes"] * 0.9
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["cores"] >= 1 and c["value"] > 0 and isinstance(c["sample"], str)
    names = [w["workload"] for w in d["configs"]]
    assert names == ["tiny", "sd3_1024", "flux_1024", "grpo_sd3", "flux_2048"]
    for w in d["configs"]:
        assert w["dense"]["ms"] > 0 and all(s["ms"] > 0 and s["time_over_density_x_dense"] > 0.5 for s in w["sparse"])

