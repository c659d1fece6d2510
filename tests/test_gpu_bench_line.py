"""bench.py on the GPU machine: one JSON line with the fields the contract names (small configuration,
few steps), `zero_ulp` true against the CPU oracle, and a roofline that is consistent with itself."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_bench_line_fields_and_consistency():
    out = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--config", "2", "--no-configs",
                          "--no-extras", "--steps", "5", "--warmup", "2"],
                         capture_output=True, text=True, timeout=600)
    assert out.returncode == 0, out.stderr[-2000:]
    lines = [l for l in out.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for k in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better",
              "scaling", "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert k in d, k
    assert d["n_gpus"] == 1 and d["steps"] == 5 and d["warmup"] == 2 and d["dtype"] == "f32"
    assert d["vs_baseline"] is None and d["config"]["workload"].startswith("config 2")
    r = d["roofline"]
    assert r["bound"] == "hbm" and r["peak"] == 8000.0 and r["unit"] == "GB/s"
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-3
    # the line prints the launch time to 1e-4 ms: allow for that rounding
    recomputed = r["bytes_per_launch"] / (r["avg_launch_ms"] * 1e-3) / 1e9
    assert abs(r["achieved"] - recomputed) <= recomputed * (1e-4 / r["avg_launch_ms"]) + 1.0
    assert r["min_launch_ms"] <= r["median_launch_ms"] and r["min_launch_ms"] <= r["avg_launch_ms"]
    assert 0.0 < r["frac"] < 1.0                      # below the vendor peak
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["cores"] == 1 and c["value"] > 0 and c["unit"] == "GB/s"
    assert d["cpu_baseline_all_cores"]["cores"] >= 1
    assert d["zero_ulp"] is True
    # the whole step cannot be faster than its parts
    assert d["ms_per_step"] >= r["avg_launch_ms"]
