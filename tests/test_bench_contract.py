"""The driver-facing entry points: bench.py prints one JSON line with the agreed keys and
refuses more than one GPU; smoke() runs."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    run = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                         capture_output=True, text=True, timeout=120)
    assert run.returncode != 0
    assert "ONE GPU" in run.stderr
    assert run.stdout.strip() == ""


@pytest.mark.gpu
def test_bench_prints_one_json_line_with_the_agreed_keys():
    run = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "tiny",
                          "--steps", "20", "--warmup", "5", "--profile-steps", "5"],
                         capture_output=True, text=True, timeout=280)
    assert run.returncode == 0, run.stderr[-2000:]
    lines = [l for l in run.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, lines
    line = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better",
                "scaling", "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in line, key
    assert line["n_gpus"] == 1 and line["steps"] == 20 and line["warmup"] == 5
    assert line["vs_baseline"] is None and line["data"] == "synthetic" and line["higher_is_better"] is True
    assert line["config"]["workload"] == "tiny" and "model" not in line["config"]
    roof = line["roofline"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert key in roof, key
    assert roof["bound"] == "hbm" and roof["peak"] == 8000.0 and roof["unit"] == "GB/s"
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-3
    cpu = line["cpu_baseline"]
    for key in ("value", "unit", "cores", "kind", "sample"):
        assert key in cpu, key
    assert cpu["kind"] == "oracle" and cpu["cores"] >= 1 and cpu["value"] > 0
    assert line["value"] > 0 and line["ms_per_step"] > 0
    # either HBM bytes measured with this very build of the library, or null with the reason
    assert (roof["traffic"] is None) == ("traffic_stale" in roof)
    assert line["library_build_id"] and line["step_us"] > 0
    for key in ("write_ceiling_gbps", "read_ceiling_gbps", "kernel_frac_of_read_write_bound",
                "modes_measured_in_turns", "other_workloads", "interleaved_caller_work"):
        assert key in line, key                 # the last three are filled on the headline workload only


@pytest.mark.gpu
def test_smoke_entry_point_runs():
    sys.path.insert(0, ROOT)
    import __graft_entry__ as entry
    entry.smoke()
