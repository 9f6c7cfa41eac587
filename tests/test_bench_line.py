"""bench.py prints one JSON line with the agreed fields (run on the smallest workload)."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.gpu
def test_bench_prints_one_json_line_with_roofline():
    out = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "lsq", "--headline-only",
                          "--no-cpu-baseline"], capture_output=True, text=True, timeout=300, cwd=ROOT)
    assert out.returncode == 0, out.stderr[-2000:]
    lines = [l for l in out.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better",
                "scaling", "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 256 and d["config"]["workload"] == "lsq" and d["sync_rounds"] == 28
    assert d["sync_rounds_per_run"] == 28 and d["sync_schedule"]["averaging_after_iteration"][-1] == 256
    assert d["config"]["placement"] == "plain" and d["config"]["timed_window"] == [0, 256]
    assert d["value"] == pytest.approx(4 * 1024 * 256 / (d["ms_per_step"] * 256 * 1e-3), rel=1e-6)
    r = d["roofline"]
    for key in ("bound", "achieved", "peak", "unit", "frac", "traffic", "avg_ms", "median_ms", "min_ms"):
        assert key in r, key
    assert r["frac"] == pytest.approx(r["achieved"] / r["peak"]) and r["min_ms"] <= r["median_ms"]
    assert d["ms_per_step_no_event_brackets"] < d["ms_per_step"]


def test_bench_refuses_more_than_one_gpu():
    out = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True,
                         text=True, timeout=120, cwd=ROOT)
    assert out.returncode != 0 and "ONE GPU" in out.stderr
