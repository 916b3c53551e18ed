"""The record bench.py prints: one JSON line with the metric, the roofline of the dominant kernel and,
unless switched off, the CPU baseline; more than one GPU is refused with a message."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BENCH = os.path.join(ROOT, "bench.py")


def test_more_than_one_gpu_is_refused_with_a_message():
    run = subprocess.run([sys.executable, BENCH, "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert run.returncode != 0
    assert "--gpus 1" in run.stderr and run.stdout.strip() == ""


@pytest.mark.gpu
def test_record_of_a_short_run():
    run = subprocess.run([sys.executable, BENCH, "--steps", "700", "--warmup", "50", "--no-sweep", "--no-cpu-baseline"],
                         capture_output=True, text=True, timeout=300)
    assert run.returncode == 0, run.stderr[-2000:]
    lines = [ln for ln in run.stdout.splitlines() if ln.startswith("{")]
    assert len(lines) == 1
    rec = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline"):
        assert key in rec, key
    assert rec["n_gpus"] == 1 and rec["steps"] == 700 and rec["warmup"] == 50
    assert rec["unit"] == "images/s" and rec["dtype"] == "f32" and rec["data"] == "synthetic"
    assert rec["vs_baseline"] is None and rec["higher_is_better"] is True
    assert "workload" in rec["config"] and rec["config"]["batch"] == 100
    # value and step time describe the same run
    assert abs(rec["value"] * rec["ms_per_step"] * 1e-3 / 100 - 1.0) < 1e-6
    roof = rec["roofline"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert key in roof, key
    assert roof["bound"] == "alu" and roof["unit"] == "TFLOP/s" and roof["peak"] == 157.3
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-9
    assert 0.0 < roof["frac"] < 1.0
    # the fused kernel cannot take longer than the step it is part of (plus the dispatch latency an
    # event pair includes), nor can the step beat what the kernel alone needs at the fp32 peak
    assert roof["kernel_ms"] <= rec["ms_per_step"] * 1.5
    assert rec["ms_per_step"] * 1e-3 >= roof["flop_per_launch"] / (roof["peak"] * 1e12)
    assert "cpu_baseline" not in rec and "sweep" not in rec
