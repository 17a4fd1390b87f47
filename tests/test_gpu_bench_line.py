"""bench.py end to end on the device, small: the one JSON line carries the contract's fields, a roofline
block whose HBM fraction is a fraction, and (tiny workload, quick) a CPU baseline that agrees with the
device result."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
pytestmark = pytest.mark.gpu


def _bench(*args):
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True, timeout=280,
                       cwd=ROOT)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, "bench.py must print exactly one line"
    return json.loads(lines[0])


def test_bench_line_tiny_workload():
    j = _bench("--workload", "tiny", "--steps", "20", "--warmup", "3", "--batches", "4")
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
              "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert k in j, k
    assert j["n_gpus"] == 1 and j["steps"] == 20 and j["warmup"] == 3 and j["vs_baseline"] is None
    assert j["unit"] == "samples/s" and j["value"] > 0 and j["dtype"] == "f32" and j["data"] == "synthetic"
    assert "workload" in j["config"] and "model" not in j["config"]
    r = j["roofline"]
    assert r["bound"] == "hbm" and r["peak"] == 8000.0 and r["unit"] == "GB/s"
    assert 0.0 < r["frac"] <= 1.0 and abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-9
    assert r["traffic"] is None                                  # no counter figure exists for this workload
    assert "compulsory" in r["achieved_basis"] and r["frac_algorithmic"] >= r["frac"]
    c = j["cpu_baseline"]
    assert c["kind"] == "oracle" and c["value"] > 0 and 1 <= c["cores"] <= c["host_cpus"]
    assert j["max_abs_diff_vs_oracle"] < 1e-5
    assert len(j["timing"]["ms_per_step_each_repeat"]) == 5


def test_bench_only_mfma_leg():
    j = _bench("--only-mfma", "--steps", "5", "--warmup", "2")["mfma_roofline"]
    assert j["bound"] == "mfma" and j["peak"] == 2500.0 and j["unit"] == "TFLOP/s"
    assert set(j["batch_sweep"]) == {"1024", "4096", "16384"}
    assert 0.0 < j["frac"] < 1.0 and j["flops_per_launch"] == 2.0 * 1024 * 2560 * 1024
    assert all(0.0 < v["frac"] < 1.0 for v in j["batch_sweep"].values())
