"""bench.py: its command line without a GPU, and (GPU) the one JSON line it prints."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout == ""


@pytest.mark.gpu
def test_one_json_line_with_the_fields_of_the_contract():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "20", "--warmup", "3", "--workload",
                        "tiny2d", "--no-probes", "--other-workloads", "image2d"], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1
    j = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in j, key
    assert j["n_gpus"] == 1 and j["steps"] == 20 and j["warmup"] == 3 and j["data"] == "synthetic"
    assert j["vs_baseline"] is None and j["higher_is_better"] is True and j["unit"] == "Mpoints/s"
    assert "workload" in j["config"] and j["config"]["workload"].startswith("tiny2d")
    assert j["value"] > 0 and abs(j["value"] - 4096 / (j["ms_per_step"] * 1e-3) / 1e6) < 1e-6 * j["value"]
    roof = j["roofline"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert key in roof, key
    assert roof["bound"] == "hbm" and roof["peak"] == 8000.0 and abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-12
    assert roof["pass"] in ("fwd", "bwd") and set(roof["passes"]) == {"fwd", "bwd", "step"}
    (other,) = j["workloads"]  # the other workloads asked for: the same step, GPU side only
    assert other["name"] == "image2d" and other["B"] == 1 << 18 and other["sorted_backward"] is True
    for key in ("ms_step", "mpoints_s", "ms_fwd", "ms_bwd", "frac"):
        assert other[key] > 0, key
    assert abs(other["mpoints_s"] - other["B"] / (other["ms_step"] * 1e-3) / 1e6) < 1e-6 * other["mpoints_s"]
    cpu = j["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["cores"] >= 1 and cpu["value"] > 0 and cpu["sample"]
