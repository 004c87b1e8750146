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
           "--kernel-warm-s", "0", "--kernel-rounds", "1", "--cpu-sample", "65536", "--launch", launch,
           "--no-per-config"]
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
    # the step is the method only (forward + backward per activation); the baselines sit under `kernels`
    assert out["config"]["kernels_per_step"] == 2 and out["config"]["bytes_per_step"] == 6 * out["config"]["elements"] * 4
    assert set(out["kernels"]["gelu_tanh"]) == {"nfad_fwd", "nfad_bwd", "recompute_fwd", "recompute_bwd",
                                                 "saveall_fwd", "saveall_bwd"}
    assert roof["kernel"] == "nfad_fwd(gelu_tanh)"
    ref = out["stream_reference"]
    assert ref is not None and ref["read_1_write_2 (pattern of nfad_fwd)"]["GB/s"] > 0


@pytest.mark.gpu
def test_default_workload_is_the_largest_and_every_configuration_is_reported():
    """The line the driver records: largest configuration as the headline, and nfad_fwd / nfad_bwd on all
    five configurations (eleven tensor x dtype x activation rows) in `per_config`."""
    cmd = [sys.executable, BENCH, "--steps", "5", "--warmup", "2", "--prewarm-s", "0", "--kernel-warm-s", "0",
           "--kernel-rounds", "1", "--no-cpu-baseline", "--no-stream-reference", "--no-baselines"]
    r = subprocess.run(cmd, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    out = json.loads([l for l in r.stdout.splitlines() if l.strip()][-1])
    assert out["config"]["workload"].startswith("C5") and out["config"]["elements"] == 134217728
    assert out["config"]["kernels_per_step"] == 8
    rows = out["per_config"]
    assert [r_["config"] for r_ in rows] == ["C1", "C2", "C3", "C3", "C3", "C4", "C4", "C5", "C5", "C5", "C5"]
    for r_ in rows:
        for k in ("nfad_fwd", "nfad_bwd"):
            assert r_[k]["us"] > 0 and abs(r_[k]["frac"] - r_[k]["GB/s"] / 8000.0) < 1e-3
        assert r_["launch"] in ("direct", "hip graph replay")
    assert rows[0]["launch"] == "hip graph replay" and rows[-1]["launch"] == "direct"
