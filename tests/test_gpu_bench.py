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
    """The default run: the high-resolution workload (32 x 3840x2160, bf16) with the traffic workload under its own key."""
    r = _bench("--steps", "6", "--warmup", "2", "--traffic-steps", "24", "--no-cpu-baseline")
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling", "vs_baseline",
              "dtype", "data", "config", "roofline", "roofline_hbm", "measured_peaks", "traffic"):
        assert k in d, k
    assert d["n_gpus"] == 1 and d["steps"] == 6 and d["warmup"] == 2 and d["higher_is_better"] is True
    assert d["vs_baseline"] is None and d["data"] == "synthetic" and d["dtype"] == "bf16"
    assert "3840x2160" in d["config"]["workload"] and d["config"]["batch_frames"] == 32 and d["config"]["instances"] == 1
    assert d["value"] > 0 and abs(d["value"] - 32 * 1e3 / d["ms_per_step"]) < 1e-6 * d["value"] + 1e-3     # every frame met the SLO
    for rf, dtype_peak in ((d["roofline"], 2500.0), (d["traffic"]["roofline"], 2500.0)):
        assert rf["bound"] == "mfma" and rf["unit"] == "TFLOP/s" and rf["peak"] == dtype_peak
        assert 0 < rf["achieved"] < rf["peak"] and abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-9
        assert rf["avg_launch_us"] > 0 and rf["flop_per_launch"] > 0 and rf["launches_per_step"] >= 1
        assert "conv" in rf["kernel"] and "traffic_source" in rf
        assert rf["traffic"] is None or rf["traffic"] > 0.5 * rf["bytes_per_launch"]
        assert 0 < rf["frac_of_measured"] < 1.2
    hb = {h["stage"]: h for h in d["roofline_hbm"]}
    assert set(hb) == {"letterbox", "decode", "crop0"}
    for h in hb.values():
        assert h["bound"] == "hbm" and h["unit"] == "GB/s" and h["peak"] == 8000.0 and h["algorithmic_bytes"] > 0 and h["stage_us"] > 0
        assert 0 < h["achieved"] < h["peak"] and abs(h["frac"] - h["achieved"] / h["peak"]) < 1e-9 and h["frac_of_measured"] > 0
    # the stated algorithmic bytes of the three kernels: 32 frames x (1280 x 720 source pixels tapped + 1280 x 1280 x 3 bf16),
    # 32 x 100800 candidates x 85 bf16 (+ 32 B per candidate found)
    assert abs(hb["letterbox"]["algorithmic_bytes"] - 32 * (3 * 1280 * 720 + 1280 * 1280 * 3 * 2)) < 1
    assert 32 * 100800 * 85 * 2 <= hb["decode"]["algorithmic_bytes"] <= 32 * 100800 * 85 * 2 + 32 * 32 * 8192
    mp = d["measured_peaks"]
    assert 2000 < mp["copy_gbps"] < 8000 and 800 < mp["mfma_tflops"] < 2500
    t = d["traffic"]
    assert t["dtype"] == "f16" and t["config"]["batch_frames"] == 8 and t["config"]["instances"] == 4 and t["value"] > 0


def test_more_than_one_gpu_is_refused_with_a_message():
    r = _bench("--gpus", "2")
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""


@pytest.mark.parametrize("args,keys", [
    (["--workload", "traffic", "--steps", "24", "--warmup", "4", "--no-cpu-baseline"], ["roofline", "roofline_hbm"]),
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


def test_e4m3_layer_comparison_prints_one_json_line():
    """bench.py --workload conv8: every layer timed in both types, the E4M3 roofline against the fp8 peak."""
    r = _bench("--workload", "conv8", "--steps", "3")
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    assert d["n_gpus"] == 1 and d["vs_baseline"] is None and d["dtype"] == "f8e4m3" and "workload" in d["config"]
    assert d["roofline"]["bound"] == "mfma" and d["roofline"]["peak"] == 5000.0 and 0 < d["roofline"]["frac"] < 1
    assert "f8" in d["roofline"]["kernel"] and d["measured_peaks"]["mfma_e4m3_tflops"] > d["measured_peaks"]["mfma_bf16_tflops"]
    assert len(d["layers"]) > 30 and all(L["f8"]["ms"] > 0 and L["bf16"]["ms"] > 0 for L in d["layers"])
    assert d["speedup"] > 1.0                      # the 8-bit variant must at least not lose over the whole list
