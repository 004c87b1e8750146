"""bench.py's output contract: one JSON line with the agreed keys, a roofline object for the
forward kernel and a cpu_baseline object from the oracle; more than one GPU is refused."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BENCH = os.path.join(ROOT, "bench.py")


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, BENCH, "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


@pytest.mark.gpu
@pytest.mark.parametrize("launch", ["direct", "graph"])
def test_one_json_line_with_roofline_and_cpu_baseline(launch):
    cmd = [sys.executable, BENCH, "--config", "0", "--steps", "5", "--warmup", "2", "--prewarm-s", "0",
           "--kernel-warm-s", "0", "--kernel-rounds", "1", "--cpu-sample", "65536", "--launch", launch]
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    out = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better",
                "scaling", "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in out, key
    assert out["n_gpus"] == 1 and out["steps"] == 5 and out["warmup"] == 2 and out["unit"] == "GB/s"
    assert out["higher_is_better"] is True and out["vs_baseline"] is None and out["data"] == "synthetic"
    assert out["dtype"] == "f32" and "workload" in out["config"] and "model" not in out["config"]
    assert out["config"]["launch"] == ("hip graph replay" if launch == "graph" else "direct")
    roof = out["roofline"]
    assert roof["bound"] == "hbm" and roof["peak"] == 8000.0 and roof["unit"] == "GB/s"
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-3 and 0 < roof["frac"] < 1
    assert roof["algorithmic_bytes_per_launch"] == 3 * out["config"]["elements"] * 4
    cpu = out["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["unit"] == "GB/s" and cpu["cores"] >= 1 and cpu["value"] > 0
    assert out["value"] > 0 and out["ms_per_step"] > 0
