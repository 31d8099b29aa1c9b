"""bench.py's contract, the parts that need no GPU: more than one GPU is refused with a message, and the HBM traffic
figures come out of the committed rocprofv3 summaries.  With a GPU: one small workload end to end, the JSON line's keys."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, cwd=ROOT)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
    env = dict(os.environ, WORLD_SIZE="4")
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")], capture_output=True, text=True, cwd=ROOT, env=env)
    assert r.returncode == 2 and "ONE GPU" in r.stderr


def test_traffic_is_read_from_the_committed_summaries():
    sys.path.insert(0, ROOT)
    try:
        import bench
    finally:
        sys.path.pop(0)
    prune = bench.read_traffic("c5_decoder_mlp_2of4", "prune")
    gemm = bench.read_traffic("c5_decoder_mlp_2of4", "gemm")
    algorithmic = 32768 * 28672 * 25 // 8                       # read g, write T/2 values and T/16 index words per column
    assert abs(prune - algorithmic) < 0.01 * algorithmic         # the prune re-reads nothing
    assert 1.0e10 < gemm < 2.5e10
    assert bench.read_traffic("no_such_workload", "prune") is None


@pytest.mark.gpu
def test_json_line_of_a_small_workload():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "c4_vit_proj_2of4", "--steps", "5", "--warmup", "2",
                        "--no-cpu-baseline"], capture_output=True, text=True, cwd=ROOT, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling", "vs_baseline",
              "dtype", "data", "config", "roofline", "roofline_prune", "cache"):
        assert k in d, k
    assert d["n_gpus"] == 1 and d["steps"] == 5 and d["vs_baseline"] is None and d["data"] == "synthetic"
    assert "workload" in d["config"] and "model" not in d["config"]
    for k in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert k in d["roofline"], k
    assert abs(d["roofline"]["frac"] - d["roofline"]["achieved"] / d["roofline"]["peak"]) < 1e-9
    assert d["cache"].startswith("cold")
