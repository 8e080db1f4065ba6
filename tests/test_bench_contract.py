"""The benchmark's command-line contract: one JSON line with the agreed fields on one GPU, a clear
refusal for more than one."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BENCH = os.path.join(ROOT, "bench.py")


def test_more_than_one_gpu_is_refused_before_anything_touches_a_device():
    res = subprocess.run([sys.executable, BENCH, "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert res.returncode != 0 and res.stdout.strip() == ""
    assert "one GPU only" in res.stderr
    env = dict(os.environ, WORLD_SIZE="4", RANK="1")
    res = subprocess.run([sys.executable, BENCH], capture_output=True, text=True, timeout=120, env=env)
    assert res.returncode != 0 and "one GPU only" in res.stderr


@pytest.mark.gpu
@pytest.mark.parametrize("workload", ["tiny", "100m"])
def test_one_json_line_with_roofline_and_cpu_baseline(workload):
    res = subprocess.run([sys.executable, BENCH, "--workload", workload, "--steps", "3", "--warmup", "1"],
                         capture_output=True, text=True, timeout=600)
    assert res.returncode == 0, res.stderr[-2000:]
    lines = [l for l in res.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    assert d["metric"] == "fragment_outer_step_params_per_s" and d["unit"] == "params/s"
    assert d["n_gpus"] == 1 and d["steps"] == 3 and d["warmup"] == 1
    assert d["higher_is_better"] is True and d["vs_baseline"] is None and d["data"] == "synthetic"
    assert d["dtype"] == "f32" and "model" not in d["config"] and workload in d["config"]["workload"]
    assert abs(d["value"] - d["config"]["fragment_params"] / (d["ms_per_step"] * 1e-3)) <= 1e-6 * d["value"]
    r = d["roofline"]
    assert r["bound"] == "hbm" and r["unit"] == "GB/s" and r["peak"] == 8000.0
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-12 and 0 < r["frac"] < 1
    assert abs(r["achieved"] - r["bytes_per_launch"] / (r["launch_ms"] * 1e-3) / 1e9) <= 1e-6 * r["achieved"]
    assert r["traffic"] is None or abs(r["traffic"] / r["bytes_per_launch"] - 1) < 0.05
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["unit"] == "params/s" and c["value"] > 0 and 1 <= c["cores"] <= 16
    assert isinstance(c["sample"], str) and c["single_thread"]["cores"] == 1


@pytest.mark.gpu
def test_smoke_entry_point():
    if ROOT not in sys.path:
        sys.path.insert(0, ROOT)
    import __graft_entry__
    __graft_entry__.smoke()
