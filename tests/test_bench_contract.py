"""The benchmark's command-line contract."""
import json
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused():
    out = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                         capture_output=True, text=True, timeout=120)
    assert out.returncode != 0
    assert "ONE GPU" in out.stderr and not out.stdout.strip()


@pytest.mark.gpu
def test_bench_prints_one_json_line_with_the_required_fields():
    out = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", "c1_tiny",
                          "--steps", "5", "--warmup", "2", "--cpu-budget", "1", "--no-per-config"], capture_output=True, text=True, timeout=300)
    assert out.returncode == 0, out.stderr
    lines = [l for l in out.stdout.splitlines() if l.strip()]
    assert len(lines) == 1
    d = json.loads(lines[0])
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better",
                "scaling", "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline", "parity"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 5 and d["warmup"] == 2 and d["unit"] == "rounds/s"
    assert d["dtype"] == "f32" and d["data"] == "synthetic" and d["vs_baseline"] is None
    assert d["config"]["workload"] == "c1_tiny" and "model" not in d["config"]
    r = d["roofline"]
    assert r["bound"] == "hbm" and r["peak"] == 8000.0 and r["unit"] == "GB/s"
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-12
    assert r["traffic"] is None or r["traffic"] > 0
    assert (r["traffic"] is None) == (r["traffic_source"] is None)
    # HBM bytes, not the (R+1)-reads figure, are what is priced against the HBM peak
    assert r["bytes_per_launch"] <= r["compulsory_bytes_per_launch"] * 1.05
    assert r["algorithmic_bytes_per_launch"] == 4 * (2 + 2) * 4 * 65536
    p = d["parity"]
    assert p["ok"] and p["tables_bit_exact"] and p["max_rel_err"] <= 1e-6
    assert p["columns_checked"] == p["of_columns"] == 65536
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["cores"] == 1 and c["value"] > 0 and c["sample"] and c["cpu_model"]
