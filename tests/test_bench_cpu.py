"""Host-side pieces of bench.py that need no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def test_algorithmic_bytes_per_update():
    import bench
    from paper_1609_08326_amd import workloads as W
    c = W.CONFIGS
    assert bench.algorithmic_bytes_per_update(c[0]) == 20      # c: w, bak, g in; w, bak out
    assert bench.algorithmic_bytes_per_update(c[1]) == 28      # a: + MeanSquare in and out
    assert bench.algorithmic_bytes_per_update(c[2]) == 28
    assert bench.algorithmic_bytes_per_update(c[3]) == 13      # (16 + 16*12) / 16
    assert bench.algorithmic_bytes_per_update(c[4]) == 26      # bf16 gradient
    assert bench.algorithmic_bytes_per_update(W.get("fold")) == 5
    assert bench.algorithmic_bytes_per_update(c[2], bak_bf16=True) == 24   # backup 2 B in, 2 B out
    assert bench.algorithmic_bytes_per_update(c[4], bak_bf16=True) == 22
    assert bench.algorithmic_bytes_per_update(c[3], bak_bf16=True) == 9    # (16 + 16*8) / 16


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in r.stderr


def test_profile_figures_are_read_from_the_committed_summaries():
    import bench
    assert bench.read_profile("push_fused_cfg2") > 7.0e8
    assert bench.read_profile("sync_fold_J16_fold", "valu_instr_per_launch") > 1e8
    # the event loop's kernel: per launch of 64 arrivals, about 90 instructions per update
    # (about 105 at the 1 MB size, where two lanes share a group and both draw its Philox words)
    for cfg, d in (("cfg1", 272_474), ("cfg2", 25_557_032), ("cfg4", 138_357_544)):
        valu = bench.read_profile("run_synth_blocks_%s" % cfg, "valu_instr_per_launch")
        assert 80.0 < valu * 64 / (d * 64.0) < 115.0, cfg
    assert bench.read_profile("no_such_kernel") is None


def test_practical_ceilings_are_read_from_the_probe_summary():
    import bench
    for size in ("25m", "138m"):
        v = bench.read_probe("practical_ceiling_4r3w_GBs", size)
        assert v is not None and 5000.0 < v < 8000.0, (size, v)
    assert bench.read_probe("no_such_key", "25m") is None
