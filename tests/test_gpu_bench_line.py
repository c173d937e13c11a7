"""The line bench.py prints (the driver reads it): one JSON object with the agreed fields, whose
figures agree with each other.  Runs the real thing on the GPU with few steps."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def bench_line(*args):
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "20", "--warmup", "3", *args],
                       capture_output=True, text=True, timeout=280, cwd=ROOT)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.startswith("{")]
    assert len(lines) == 1, r.stdout[-2000:]
    return json.loads(lines[0])


def test_headline_line_has_the_agreed_fields_and_consistent_figures():
    j = bench_line()
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in j, key
    assert j["n_gpus"] == 1 and j["steps"] == 20 and j["warmup"] == 3 and j["higher_is_better"] is True
    assert j["unit"] == "hypothesis-steps/s" and j["dtype"] == "bf16" and j["data"] == "synthetic"
    assert j["vs_baseline"] is None and "workload" in j["config"] and "model" not in j["config"]
    assert "V=65536" in j["metric"] and "H=512" in j["metric"] and "B=1024" in j["metric"]
    # throughput = raw queries of a step / time of a step
    assert abs(j["value"] * j["ms_per_step"] * 1e-3 / 1024 - 1.0) < 0.01
    r = j["roofline"]
    assert r["bound"] == "mfma" and r["unit"] == "TFLOP/s" and r["peak"] == 2500.0
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-3
    assert abs(r["achieved"] - r["flop_per_launch"] / (r["us_per_launch"] * 1e-6) / 1e12) < 1.0
    assert r["flop_per_launch"] == 2.0 * 1024 * 512 * 65536
    assert r["us_per_launch"] < j["ms_per_step"] * 1e3            # one kernel of the step is shorter than the step
    assert 0.3 < r["frac"] < 1.0
    assert r["traffic"] is None or r["traffic"] >= 65536 * 512 * 2   # at least the weights once
    c = j["cpu_baseline"]
    assert c["kind"] == "oracle" and c["unit"] == j["unit"] and c["cores"] >= 1 and c["value"] > 0
    assert c["max_abs_dlogprob_vs_gpu"] <= 2e-3                    # the oracle leg doubles as a parity check
    assert j["value"] > 100 * c["value"]


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=60, cwd=ROOT)
    assert r.returncode != 0 and "ONE GPU" in r.stderr
