"""bench.py prints one JSON line with the fields the measurement contract names."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_line_has_the_contract_fields():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "2", "--warmup", "1", "--brief"],
                       capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1, lines
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "ms_per_step_median", "ms_per_step_min"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 2 and d["warmup"] == 1 and d["unit"] == "TFLOP/s"
    assert d["vs_baseline"] is None and d["dtype"] == "bf16" and d["data"] == "synthetic"
    assert "llama7b_32k_G8" in d["config"]["workload"] and "model" not in d["config"]
    roof = d["roofline"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic", "frac_counted", "kernel"):
        assert key in roof, key
    assert roof["bound"] == "mfma" and roof["peak"] == 2516.6 and roof["unit"] == "TFLOP/s"
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-9
    assert 0.0 < roof["frac_counted"] < roof["frac"] < 1.0          # five counted of seven executed contractions
    # the value is the counted FLOPs of the step over its wall-clock time
    flops = 3.5 * 4.0 * 4096 * 32768 * 128 * 32
    assert abs(d["value"] - flops / (d["ms_per_step"] * 1e-3) / 1e12) / d["value"] < 1e-6
    assert d["ms_per_step_min"] <= d["ms_per_step_median"] <= d["ms_per_step"] * 1.5


def test_sensor_sampler_reads_plausible_values_or_nothing():
    sys.path.insert(0, ROOT)
    import bench
    with bench.SensorSampler(period_s=0.005) as s:
        import time
        time.sleep(0.05)
    out = s.summary()
    assert out["nominal_clock_mhz"] == 2400
    for key in ("core_clock_mhz_median", "socket_power_w_median"):
        assert out[key] is None or 0 < out[key] < 5000
