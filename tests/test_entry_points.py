"""The two entry points a harness calls: bench.py's one JSON line and __graft_entry__.smoke()."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


@pytest.mark.gpu
@pytest.mark.parametrize("workload,layout", [("tiny_fc", "nchw"), ("resnet_conv3x3_7", "nhwc")])
def test_bench_prints_one_json_line_with_the_contract_keys(workload, layout):
    print("bench", workload, layout, flush=True)
    cmd = [sys.executable, os.path.join(ROOT, "bench.py"), "--workload", workload, "--layout", layout,
           "--steps", "5", "--warmup", "2", "--no-cpu-baseline"]
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=170)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.startswith("{")]
    assert len(lines) == 1
    out = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline"):
        assert key in out, key
    assert out["n_gpus"] == 1 and out["steps"] == 5 and out["warmup"] == 2 and out["vs_baseline"] is None
    assert out["data"] == "synthetic" and "workload" in out["config"] and out["value"] > 0
    roof = out["roofline"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert key in roof, key
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-9


@pytest.mark.gpu
def test_smoke_runs():
    sys.path.insert(0, ROOT)
    import __graft_entry__
    __graft_entry__.smoke()
