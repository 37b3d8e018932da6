"""bench.py's command-line contract: more than one GPU is refused with a message (CPU); the
default-mode output is one JSON line with the agreed keys (GPU, short run)."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


@pytest.mark.gpu
def test_default_mode_prints_one_json_line():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "1", "--steps", "4",
                        "--warmup", "1", "--no-cpu-baseline"],
                       capture_output=True, text=True, timeout=280, cwd=ROOT)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better",
              "scaling", "vs_baseline", "dtype", "data", "config", "roofline"):
        assert k in d, k
    assert d["n_gpus"] == 1 and d["steps"] == 4 and d["warmup"] == 1 and d["unit"] == "GB/s"
    assert d["dtype"] == "u8" and d["data"] == "synthetic" and d["vs_baseline"] is None
    assert "workload" in d["config"] and "model" not in d["config"]
    rf = d["roofline"]
    assert rf["bound"] == "hbm" and rf["peak"] == 8000.0 and rf["unit"] == "GB/s"
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-3
    assert 0.3 < rf["frac"] < 1.0            # a copy cannot beat the HBM roofline
    assert d["value"] > 0 and d["ms_per_step"] > 0
    assert 0 < d["min_ms"] <= d["median_ms"] <= d["max_ms"]
    rh = d["roofline_hash"]
    assert rh["bound"] == "latency" and 0 < rh["frac"] <= 1.0 and rh["peak"] <= rh["achieved"]
    pr = d["per_request"]
    for path in ("staged", "direct"):                  # (A) one call per request, from C and from Python
        assert pr["c_abi"][path].get("us_per_request", 0) > 0, pr["c_abi"][path]
        assert pr["python_binding"][path]["us_per_request"] > 0
    assert d["fused"]["value"] > d["value"]            # half the traffic per block
