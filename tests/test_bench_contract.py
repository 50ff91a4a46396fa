"""Host-side checks of bench.py's contract (no GPU): one GPU only, default flags, and the CPU-baseline leg."""
import json
import os
import subprocess
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_bench(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True, cwd=ROOT)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = run_bench("--gpus", "2")
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr + r.stdout
    r8 = run_bench("--gpus", "8", "--steps", "1", "--warmup", "0")
    assert r8.returncode != 0


def test_defaults_are_one_gpu_and_a_short_run():
    sys.path.insert(0, ROOT)
    import bench
    src = open(os.path.join(ROOT, "bench.py")).read()
    assert 'add_argument("--gpus", type=int, default=1)' in src
    assert 'add_argument("--workload", default="lidar8"' in src        # the largest of the five configurations
    assert hasattr(bench, "cpu_baseline") and hasattr(bench, "PEAK_BF16_TFLOPS") and hasattr(bench, "PEAK_HBM_GBPS")
    assert bench.PEAK_BF16_TFLOPS == 2500.0 and bench.PEAK_HBM_GBPS == 8000.0


def test_cpu_baseline_leg_reports_the_oracle_on_a_bounded_sample():
    sys.path.insert(0, ROOT)
    import bench
    from paper_2412_16481_amd import workloads as wl
    w = wl.make_workload("tiny")
    b = bench.cpu_baseline(w, 256)
    assert b["kind"] == "oracle" and b["unit"] == "points/s" and b["cores"] >= 1
    assert b["value"] > 0 and np.isfinite(b["value"]) and "sampled query rows" in b["sample"]
    json.dumps(b)                                                       # plain data, goes into the JSON line as is
