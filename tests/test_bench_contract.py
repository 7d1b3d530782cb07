"""The benchmark's command-line contract: one JSON line with the agreed keys; more than one GPU is refused."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_bench(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], cwd=ROOT, capture_output=True,
                          text=True, timeout=600)


def test_more_than_one_gpu_is_refused():
    p = run_bench("--gpus", "2")
    assert p.returncode == 2
    assert "ONE GPU" in p.stderr and p.stdout.strip() == ""


@pytest.mark.gpu
def test_json_line():
    p = run_bench("--gpus", "1", "--steps", "20", "--warmup", "5")
    assert p.returncode == 0, p.stderr[-2000:]
    lines = [l for l in p.stdout.strip().splitlines() if l.startswith("{")]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
              "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert k in d, k
    assert d["n_gpus"] == 1 and d["steps"] == 20 and d["warmup"] == 5
    assert d["unit"] == "TFLOP/s" and d["dtype"] == "bf16" and d["data"] == "synthetic" and d["vs_baseline"] is None
    assert d["higher_is_better"] is True and "workload" in d["config"] and "model" not in d["config"]
    # the untimed steps that precede the warm-up (clock ramp) are stated in the line
    assert d["config"]["clock_ramp"]["ms"] == 500.0 and d["config"]["clock_ramp"]["untimed_steps_before_warmup"] >= 50
    # value is the step's algorithmic flops over the measured step time
    assert abs(d["value"] - d["config"]["flops_per_step"] / (d["ms_per_step"] * 1e-3) / 1e12) <= 0.01 * d["value"]
    r = d["roofline"]
    assert r["bound"] == "mfma" and r["unit"] == "TFLOP/s" and r["peak"] == 2500.0
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-3 and r["traffic"] is not None
    # the matrix-core rate measured on the box lies between half the datasheet figure and the datasheet figure
    assert 0.5 * r["peak"] < r["measured_mfma_peak"] <= 1.02 * r["peak"]
    assert abs(r["frac_of_measured_peak"] - r["achieved"] / r["measured_mfma_peak"]) < 1e-3
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["unit"] == "TFLOP/s" and c["cores"] >= 1 and c["value"] > 0 and c["sample"]


def test_measurement_modes_need_a_gpu():
    """Without a GPU the measurement modes say so and exit with status 3 instead of falling back to anything."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is visible")
    for mode in ("--power", "--phases"):
        p = run_bench(mode)
        assert p.returncode == 3 and p.stdout.strip() == "" and "bench.py:" in p.stderr, (mode, p.stderr[-500:])


@pytest.mark.gpu
def test_power_report():
    """bench.py --power: one JSON line per case; the readings lie between idle and the board's limit."""
    p = run_bench("--power")
    if p.returncode == 3 and "hwmon" in p.stderr:
        pytest.skip("no board power reading on this box")
    assert p.returncode == 0, p.stderr[-2000:]
    rows = [json.loads(l) for l in p.stdout.splitlines() if l.startswith("{")]
    assert rows[0]["case"] == "idle" and len(rows) == 6
    for r in rows[1:]:
        assert rows[0]["watts_mean"] * 0.9 <= r["watts_min"] <= r["watts_mean"] <= r["watts_max"]
        assert r["watts_cap"] is None or r["watts_max"] <= 1.1 * r["watts_cap"]
        assert r["samples"] >= 20 and r["ms_per_pass"] > 0
