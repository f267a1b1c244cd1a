"""bench.py's output contract: one JSON line with the metric, the roofline of the dominant kernel
and the CPU oracle baseline; more than one GPU is refused with a message."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BENCH = os.path.join(ROOT, "bench.py")


def test_more_than_one_gpu_is_refused():
    res = subprocess.run([sys.executable, BENCH, "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert res.returncode != 0
    assert "one GPU" in res.stderr and not res.stdout.strip()


@pytest.mark.gpu
@pytest.mark.parametrize("extra", [[], ["--center", "--one-call"], ["--bucket", "whole", "--norm", "max"], ["--path", "fixed"]])
def test_json_line(extra):
    res = subprocess.run([sys.executable, BENCH, "--config", "cfg2", "--steps", "3", "--warmup", "1", *extra],
                         capture_output=True, text=True, timeout=300)
    assert res.returncode == 0, res.stderr[-2000:]
    lines = [l for l in res.stdout.splitlines() if l.startswith("{")]
    assert len(lines) == 1
    o = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in o, key
    assert o["n_gpus"] == 1 and o["steps"] == 3 and o["warmup"] == 1 and o["unit"] == "GB/s"
    assert o["vs_baseline"] is None and o["dtype"] == "f32" and o["data"] == "synthetic"
    assert "workload" in o["config"] and "model" not in o["config"]
    r = o["roofline"]
    assert r["bound"] == "hbm" and r["peak"] == 8000.0 and r["unit"] == "GB/s"
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-3
    c = o["cpu_baseline"]
    assert c["kind"] == "oracle" and c["cores"] == 1 and c["value"] > 0 and c["sample"]
    assert o["value"] > 0 and o["ms_per_step"] > 0
