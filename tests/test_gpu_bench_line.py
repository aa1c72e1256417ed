"""The line bench.py prints: one JSON object with the fields the measurement contract names, on the smallest
workload (the 512x512 layer), through the same code path as the default run."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

pytestmark = pytest.mark.gpu


def test_bench_line_of_the_small_workload():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "1", "--workload", "toy",
                          "--steps", "3", "--warmup", "1"], capture_output=True, text=True, cwd=ROOT, timeout=140)
    assert res.returncode == 0, res.stderr[-2000:]
    lines = [ln for ln in res.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1, res.stdout[-2000:]
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1 and d["higher_is_better"] is True
    assert d["data"] == "synthetic" and d["vs_baseline"] is None and "workload" in d["config"]
    assert d["value"] > 0 and d["ms_per_step"] > 0
    r = d["roofline"]
    assert r["bound"] in ("mfma", "hbm", "alu") and r["unit"] in ("TFLOP/s", "GB/s")
    assert r["frac"] == pytest.approx(r["achieved"] / r["peak"], rel=1e-6) and 0 < r["frac"] < 1
    assert 0 < r["min_us"] <= r["median_us"] <= r["max_us"]
    loop = r["chip_mfma_loop"]
    assert 0.3 < loop["frac_of_peak"] < 1.0 and 500 < loop["clock_mhz"] < 2600   # the chip's own loop under its power limit
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["value"] > 0 and c["cores"] >= 1 and c["sample"]
