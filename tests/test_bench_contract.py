"""The benchmark's command-line contract: more than one GPU is refused with a message (this build
measures one GPU), and on a GPU the single JSON line carries the agreed fields."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                         timeout=300, cwd=ROOT)
    assert res.returncode != 0
    assert "ONE GPU" in res.stderr
    assert not res.stdout.strip().startswith("{")


@pytest.mark.gpu
def test_json_line_has_the_agreed_fields():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--only-main", "--steps", "20", "--warmup", "3"],
                         capture_output=True, text=True, timeout=600, cwd=ROOT)
    assert res.returncode == 0, res.stderr[-2000:]
    line = [x for x in res.stdout.splitlines() if x.startswith("{")][-1]
    r = json.loads(line)
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in r, key
    assert r["n_gpus"] == 1 and r["steps"] == 20 and r["warmup"] == 3 and r["unit"] == "GB/s"
    assert r["vs_baseline"] is None and "workload" in r["config"] and "model" not in r["config"]
    roof = r["roofline"]
    assert roof["bound"] == "hbm" and roof["peak"] == 8000.0 and roof["unit"] == "GB/s"
    assert abs(roof["frac"] - roof["achieved"] / roof["peak"]) < 1e-3
    # the whole-job rate and the kernel's own rate agree within launch gaps
    assert 0.5 * roof["achieved"] < r["value"] <= 1.02 * roof["achieved"]
    cpu = r["cpu_baseline"]
    assert cpu["kind"] == "oracle" and cpu["unit"] == "GB/s" and cpu["cores"] >= 1 and cpu["value"] > 0 and cpu["sample"]
