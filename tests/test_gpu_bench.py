"""The benchmark's own contract on the GPU: one JSON line with the agreed fields, for the default workload at a few
steps (every code path of bench.py's main runs: timed region, both timing passes, roofline, traffic look-up), and the
refusal of more than one GPU."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True, timeout=280, cwd=ROOT)


def test_default_workload_prints_one_json_line_with_the_agreed_fields():
    r = _bench("--steps", "24", "--warmup", "4", "--no-cpu-baseline")
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling", "vs_baseline",
              "dtype", "data", "config", "roofline"):
        assert k in d, k
    assert d["n_gpus"] == 1 and d["steps"] == 24 and d["warmup"] == 4 and d["higher_is_better"] is True
    assert d["vs_baseline"] is None and d["data"] == "synthetic" and d["dtype"] == "f16" and "workload" in d["config"]
    assert d["value"] > 0 and abs(d["value"] - 8 * 1e3 / d["ms_per_step"]) < 1e-6 * d["value"] + 1e-3      # every frame met the SLO
    rf = d["roofline"]
    assert rf["bound"] == "mfma" and rf["unit"] == "TFLOP/s" and rf["peak"] == 2500.0
    assert 0 < rf["achieved"] < rf["peak"] and abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-9
    assert rf["avg_launch_us"] > 0 and rf["flop_per_launch"] > 0 and rf["launches_per_step"] >= 1
    assert "conv" in rf["kernel"]
    assert rf["traffic"] is None or rf["traffic"] > 0.5 * rf["bytes_per_launch"]


def test_more_than_one_gpu_is_refused_with_a_message():
    r = _bench("--gpus", "2")
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""


@pytest.mark.parametrize("args,keys", [
    (["--workload", "hires", "--steps", "3", "--warmup", "1", "--no-cpu-baseline"], ["roofline"]),
    (["--workload", "colocate", "--duration", "0.5"], ["portions", "no_portions", "static_batch", "schedule"]),
    (["--workload", "surge", "--duration", "1.5", "--camera-scale", "4"], ["scheduled_only", "lazy_dropping", "scaler", "scaler_and_dropping"]),
])
def test_other_workloads_print_one_json_line(args, keys):
    r = _bench(*args)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    assert d["n_gpus"] == 1 and d["vs_baseline"] is None and d["unit"] == "frames/s" and d["value"] > 0 and "workload" in d["config"]
    for k in keys:
        assert k in d, k
