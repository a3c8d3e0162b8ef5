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
    p = subprocess.run(cmd, capture_output=True, text=True, timeout=170, cwd=ROOT)
    assert p.returncode == 0, p.stderr[-2000:]
    lines = [ln for ln in p.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1, lines
    return json.loads(lines[0])


def test_default_workload_line():
    out = run_bench("--gpus", 1, "--steps", 12, "--warmup", 3, "--cpu-seconds", 1, "--legs", "none")
    assert "all_configs" not in out
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


def test_default_run_reports_every_configuration_and_the_cache_unassisted_fraction():
    """What the driver runs: after the headline region, a leg of the same workload with
    nothing left in the last-level cache, and a short leg per other configuration."""
    out = run_bench("--gpus", 1, "--steps", 12, "--warmup", 3, "--cpu-seconds", 1)
    assert out["steps"] == 12 and out["config"]["workload"].startswith("cfg2")
    r = out["roofline"]
    assert r["bound"] == "hbm" and r["launches_timed"] == 12
    assert 0.5 < r["frac_nothing_cached"] <= r["frac"] * 1.03 < 1.03
    assert r["practical_ceiling_GBs"] is None or 0.8 < r["frac_of_practical"] < 1.25
    assert "traffic_source" in r and "which_is_hbm_only" in r
    legs = out["all_configs"]
    assert sorted(legs) == ["cfg0", "cfg1", "cfg2", "cfg2_bf16_snapshots", "cfg2_fused_worker",
                            "cfg2_variant_c", "cfg3", "cfg3iid", "cfg4", "fold", "fold_ordered"]
    for name, leg in legs.items():
        assert leg["value"] > 0 and leg["workload"].startswith(name[:4]), name
        assert leg["avg_launch_ms"] > 0 and leg["bytes_per_element_update"] > 0, name
    assert legs["cfg3"]["bytes_per_element_update"] == 13 and legs["cfg4"]["bytes_per_element_update"] == 26
    assert legs["fold"]["bytes_per_element_update"] == 5
    for name in ("cfg2", "cfg3", "cfg4"):
        assert legs[name]["bound"] == "hbm" and 0.5 < legs[name]["frac"] < 1.0, (name, legs[name])
    assert 1.0 < legs["cfg3iid"]["launches_per_queue"] <= 16
    assert legs["cfg3iid"]["value"] < legs["cfg3"]["value"]
    for name in ("cfg0", "cfg1"):
        assert legs[name]["native_loop_path"]["value"] > legs[name]["value"], name
        # launch-bound eagerly: replayed from a graph faster, the block kernel faster still
        assert legs[name]["value"] < legs[name]["graph_replay_path"]["value"] \
            < legs[name]["native_loop_path"]["value"], name
    assert legs["cfg2_variant_c"]["variant"] == "DC-ASGD-c" and legs["cfg2_variant_c"]["bytes_per_element_update"] == 20
    assert legs["cfg2_bf16_snapshots"]["snapshots"] == "bf16" and legs["cfg2_bf16_snapshots"]["bytes_per_element_update"] == 24
    assert legs["cfg2_fused_worker"]["fused_worker_path"]["value"] > legs["cfg2"]["value"]
    assert legs["cfg2_fused_worker"]["native_loop_path"]["value"] \
        > legs["cfg2_fused_worker"]["fused_worker_path"]["value"]
    assert legs["fold_ordered"]["ordered_fold_path"]["value"] < legs["fold"]["value"]


def test_more_than_one_gpu_is_refused_on_the_box_too():
    cmd = [sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"]
    p = subprocess.run(cmd, capture_output=True, text=True, timeout=100, cwd=ROOT)
    assert p.returncode != 0 and "ONE GPU" in p.stderr and p.stdout.strip() == ""
