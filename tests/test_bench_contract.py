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
    # against the binary64 oracle: R adds and one scale, each within 2^-24 relative, on sums of
    # R+1 values; max|x| / max|result| stays below 8 for the workloads' distributions
    n64 = p["normwise_err_vs_f64_oracle"]
    assert n64 is None or 0 < n64 <= 8 * (8 + 3) * 2.0 ** -24
    assert p["columns_checked"] == p["of_columns"] == 65536
    c = d["cpu_baseline"]
    assert c["kind"] == "oracle" and c["cores"] == 1 and c["value"] > 0 and c["sample"] and c["cpu_model"]
    # the same steps replayed from one HIP graph: launch overhead gone, so at least as fast here
    g = d["graph_replay"]
    assert "error" not in g and g["steps_per_graph"] == 5 and g["rounds_per_s"] > 0.8 * d["value"]
    # beside the single-thread figure of record: the same library from parallel threads
    assert c["all_cores"]["value"] > 0 and c["all_cores"]["equals_single_call_on_sampled_windows"]


def test_committed_counter_profiles_match_the_kernel_sources():
    """roofline.traffic is taken from the committed rocprofv3 --pmc summaries only while the
    digest of the kernel sources stored in them is current: a kernel edit without a fresh
    counter run would silently turn the field into null."""
    sys.path.insert(0, ROOT)
    import bench
    for wl, layout in (("c5_bertlarge", "tiled"), ("c5_bertlarge", "rows"), ("c2_resnet18", "tiled"),
                       ("c2_resnet18", "rows"), ("c3_resnet50", "tiled"), ("c3_resnet50", "rows"),
                       ("c4_prime_fused", "tiled"), ("c4_prime_fused", "rows")):
        nbytes, source = bench.recorded_traffic(wl, layout)
        assert nbytes is not None and os.path.exists(os.path.join(ROOT, source)), (wl, layout)
        from paper_1908_07782_amd.workloads import WORKLOADS
        w = WORKLOADS[wl]
        compulsory = (12 if w.fused else 8) * w.N * w.P
        assert abs(nbytes / compulsory - 1.0) < 0.01, (wl, layout, nbytes, compulsory)
