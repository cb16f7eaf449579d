"""The benchmark script's contract: one JSON line with the agreed fields, figures that follow from one another, and a
refusal of more than one GPU.  The GPU part runs the script as the driver does (a child process), with the per-configuration
rows switched off to keep it short."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


@pytest.mark.gpu
def test_default_line_keeps_the_contract():
    from workloads import w4a16 as wl
    steps, warmup = 40, 4
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--steps", str(steps), "--warmup", str(warmup),
                        "--no-per-config", "--no-prefill"], capture_output=True, text=True, timeout=600, cwd=ROOT)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1, lines
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == steps and d["warmup"] == warmup
    assert d["unit"] == "GB/s" and d["higher_is_better"] is True and d["vs_baseline"] is None
    assert d["dtype"] == "f16" and d["data"] == "synthetic"
    assert "configs[1]" in d["config"]["workload"] and "model" not in d["config"]
    # value = algorithmic bytes of one step (both layers of the decode configuration at M = 1, 4, 8, 16) / time per step
    step_bytes = sum(wl.algorithmic_bytes(M, 4096, N, 128) for N in (4096, 12288) for M in (1, 4, 8, 16))
    assert d["value"] == pytest.approx(step_bytes / (d["ms_per_step"] * 1e-3) / 1e9, rel=1e-6)
    assert 0.0 < d["value"] < 8000.0
    roof = d["roofline"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert key in roof, key
    assert roof["bound"] == "hbm" and roof["peak"] == 8000.0 and roof["unit"] == "GB/s"
    assert roof["frac"] == pytest.approx(roof["achieved"] / roof["peak"], rel=1e-9) and 0.0 < roof["frac"] < 1.0
    assert roof["achieved"] == pytest.approx(roof["algorithmic_bytes_per_launch"] / (roof["avg_launch_us"] * 1e-6) / 1e9, rel=1e-6)
    assert roof["read_ceiling_GBps"] < 8000.0 and 0.0 < roof["frac_of_read_ceiling"] < 1.2
    clock = roof["shader_clock_GHz_under_load"]             # None if the probe never ran beside the launches
    assert clock is None or 0.5 < clock < 3.0
    cpu = d["cpu_baseline"]
    for key in ("value", "unit", "cores", "kind", "sample"):
        assert key in cpu, key
    assert cpu["kind"] == "oracle" and cpu["unit"] == d["unit"] and cpu["cores"] >= 1 and 0.0 < cpu["value"] < d["value"]
