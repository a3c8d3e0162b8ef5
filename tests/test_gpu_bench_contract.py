"""bench.py's output contract on a real GPU: one JSON line on stdout with the
agreed keys, the roofline object measured live and the oracle timed beside it."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_bench(*args):
    cmd = [sys.executable, os.path.join(ROOT, "bench.py"), *[str(a) for a in args]]
    print(" ".join(cmd), flush=True)
    p = subprocess.run(cmd, capture_output=True, text=True, timeout=110, cwd=ROOT)
    assert p.returncode == 0, p.stderr[-2000:]
    lines = [ln for ln in p.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1, lines
    return json.loads(lines[0])


def test_default_workload_line():
    out = run_bench("--gpus", 1, "--steps", 12, "--warmup", 3, "--cpu-seconds", 1)
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step",
                "higher_is_better", "scaling", "vs_baseline", "dtype", "data", "config",
                "roofline", "cpu_baseline"):
        assert key in out, key
    assert out["n_gpus"] == 1 and out["steps"] == 12 and out["warmup"] == 3
    assert out["higher_is_better"] is True and out["vs_baseline"] is None and out["data"] == "synthetic"
    assert out["config"]["workload"].startswith("cfg2") and "model" not in out["config"]
    assert abs(out["value"] - out["config"]["d"] * 12 / (out["ms_per_step"] * 12e-3)) < 1e-6 * out["value"]
    r = out["roofline"]
    assert r["bound"] == "hbm" and r["unit"] == "GB/s" and r["peak"] == 8000.0
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-12
    assert 0.5 < r["frac"] < 1.0, r                      # a streaming kernel on HBM3E
    assert r["launches_timed"] == 12 and r["timed_by"].startswith("HIP ")
    assert r["traffic"] is None or 0.9 < r["traffic"] / r["algorithmic_bytes_per_launch"] < 1.1
    c = out["cpu_baseline"]
    assert c["kind"] == "oracle" and c["cores"] >= 1 and c["value"] > 0 and "sample" in c
    assert out["value"] > 20 * c["value"]                # the GPU path is not the oracle in disguise


def test_more_than_one_gpu_is_refused_on_the_box_too():
    cmd = [sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"]
    p = subprocess.run(cmd, capture_output=True, text=True, timeout=100, cwd=ROOT)
    assert p.returncode != 0 and "ONE GPU" in p.stderr and p.stdout.strip() == ""
