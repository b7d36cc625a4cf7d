"""The command-line contract of bench.py: one JSON line with the agreed fields, one GPU only."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, cwd=ROOT)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stdout + r.stderr)


@pytest.mark.gpu
def test_one_json_line_with_the_agreed_fields():
    """A short run on the small workload with every leg on: the line parses and carries the fields."""
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "C1", "--steps", "5", "--warmup", "2",
                        "--no-all-workloads"], capture_output=True, text=True, cwd=ROOT, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, lines
    j = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in j, key
    assert j["n_gpus"] == 1 and j["steps"] == 5 and j["warmup"] == 2
    assert j["higher_is_better"] is True and j["dtype"] == "bf16" and j["data"].startswith("synthetic")
    assert j["config"]["workload"].startswith("C1") and "model" not in j["config"]
    assert j["value"] > 0 and j["ms_per_step"] > 0
    # tokens/s is the batch over the step time
    T = 256
    assert abs(j["value"] - T / (j["ms_per_step"] * 1e-3)) <= 1e-6 * j["value"]
    rf = j["roofline"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert key in rf, key
    assert rf["bound"] == "mfma" and rf["unit"] == "TFLOP/s" and rf["peak"] == 2500.0
    assert abs(rf["frac"] - rf["achieved"] / rf["peak"]) < 1e-9
    cb = j["cpu_baseline"]
    for key in ("value", "unit", "cores", "kind", "sample"):
        assert key in cb, key
    assert cb["kind"] == "oracle" and cb["value"] > 0 and cb["cores"] >= 1
