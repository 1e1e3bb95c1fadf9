"""bench.py's command line and the one JSON line it prints."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_bench(*args, timeout=300):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py")] + list(args), cwd=ROOT,
                          stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, timeout=timeout)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = run_bench("--gpus", "2", timeout=60)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stdout + r.stderr) and "--gpus 1" in (r.stdout + r.stderr)


@pytest.mark.gpu
def test_the_line_has_every_field_of_the_contract():
    """The smallest workload, two timed builds, a tiny oracle sample: seconds.  Checks the fields and their
    consistency, not the figures."""
    r = run_bench("--workload", "cfg1", "--also", "none", "--steps", "2", "--warmup", "1", "--cpu-sample", "2000",
                  "--queries", "100")
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.startswith("{")]
    assert len(lines) == 1, "exactly one JSON line"
    j = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in j, key
    assert j["n_gpus"] == 1 and j["steps"] == 2 and j["warmup"] == 1 and j["unit"] == "s"
    assert j["higher_is_better"] is False and j["vs_baseline"] is None and j["data"] == "synthetic"
    assert j["dtype"] == "u8" and "workload" in j["config"] and "model" not in j["config"]
    assert abs(j["value"] * 1000.0 - j["ms_per_step"]) < 1e-6 * j["ms_per_step"] + 1e-9
    roof = j["roofline"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert key in roof, key
    assert roof["bound"] in ("hbm", "mfma", "alu") and roof["peak"] == 8000.0 and roof["unit"] == "GB/s"
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-9
    assert roof["avg_launch_ms"] > 0 and roof["avg_launch_ms_device_clock"] > 0
    # the two clocks describe the same launches (events include one dispatch gap per round)
    assert 0.5 < roof["avg_launch_ms"] / roof["avg_launch_ms_device_clock"] < 2.0
    cpu = j["cpu_baseline"]
    for key in ("value", "unit", "cores", "kind", "sample"):
        assert key in cpu, key
    assert cpu["kind"] == "oracle" and cpu["cores"] == 1 and cpu["value"] > 0
    assert j["gpu_ms"]["scan"] <= j["gpu_ms"]["rounds"] <= j["gpu_ms"]["total"] * 1.02
    assert 0.9 < j["recall_at_10"] <= 1.0
