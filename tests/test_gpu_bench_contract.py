"""The benchmark script's output contract, on the smallest configuration: one JSON line with the fields the
measurement protocol names, consistent with each other."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*extra):
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "c0", "--only", "--steps", "4",
                        "--warmup", "1", *extra], capture_output=True, text=True, timeout=600, cwd=ROOT)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, lines
    return json.loads(lines[0])


def test_bench_line_on_the_smallest_configuration():
    d = _run("--cpu-sample-rows", "1024")
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 4 and d["warmup"] == 1 and d["higher_is_better"] is True
    assert d["data"] == "synthetic" and d["vs_baseline"] is None and d["dtype"] == "f32"
    assert "workload" in d["config"] and "configs[0]" in d["config"]["workload"]
    assert d["value"] > 0 and d["ms_per_step"] > 0
    ro = d["roofline"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic"):
        assert key in ro, key
    assert ro["bound"] == "hbm" and ro["peak"] == 8000.0 and ro["unit"] == "GB/s"
    assert abs(ro["frac"] - ro["achieved"] / ro["peak"]) < 1e-3
    assert ro["steps_with_events"] == 1                      # steps 0 of 4 (every fourth step carries events)
    cb = d["cpu_baseline"]
    for key in ("value", "unit", "cores", "kind", "sample"):
        assert key in cb, key
    assert cb["kind"] == "oracle" and cb["value"] > 0 and cb["cores"] >= 1
    assert d["update_history"]["mode"] == "copy" and d["update_history"]["step_ms_with_buffers_traded_instead"] > 0


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120, cwd=ROOT)
    assert r.returncode != 0 and "ONE GPU" in (r.stderr + r.stdout)
