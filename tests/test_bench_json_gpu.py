"""bench.py end to end on a small workload: exactly one JSON line on stdout, with the fields the
benchmark contract names (throughput line, roofline object, cpu_baseline object)."""
import json
import os
import subprocess
import sys

import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_bench(*args):
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [l for l in r.stdout.splitlines() if l.strip()]
    assert len(lines) == 1, f"stdout must hold one JSON line, got {len(lines)}"
    return json.loads(lines[0])


def test_bench_line_small_workload():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    o = run_bench("--gpus", "1", "--workload", "c1", "--steps", "20", "--warmup", "5")
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in o, key
    assert o["unit"] == "G(edge*dim)/s" and o["n_gpus"] == 1 and o["steps"] == 20 and o["warmup"] == 5
    assert o["higher_is_better"] is True and o["vs_baseline"] is None and o["dtype"] == "f32" and o["data"] == "synthetic"
    assert o["config"]["workload"] == "c1" and "model" not in o["config"]
    assert o["value"] > 0 and abs(o["value"] - o["config"]["nnz"] * o["config"]["d"] / (o["ms_per_step"] * 1e-3) / 1e9) < 1e-6 * o["value"]
    r = o["roofline"]
    assert r["bound"] == "hbm" and r["unit"] == "GB/s" and r["peak"] == 8000.0
    assert abs(r["frac"] - r["achieved"] / r["peak"]) < 1e-12 and r["kernel_ms"] > 0 and "traffic" in r
    assert 0.0 < r["frac"] <= 1.0 and r["traffic_source"] and r["achieved_basis"]
    priced = r["traffic"] if r["traffic"] is not None else r["compulsory_bytes"]
    assert abs(r["achieved"] - priced / (r["kernel_ms"] * 1e-3) / 1e9) < 1e-6 * r["achieved"]
    assert abs(r["algorithmic_GBs"] - r["algorithmic_bytes"] / (r["kernel_ms"] * 1e-3) / 1e9) < 1e-6 * r["algorithmic_GBs"]
    assert abs(r["algorithmic_over_peak"] - r["algorithmic_GBs"] / r["peak"]) < 1e-12
    assert "all_workloads" not in o["config"]      # only the default line carries the other workloads
    c = o["cpu_baseline"]
    assert c["kind"] == "oracle" and c["unit"] == o["unit"] and c["value"] > 0 and c["cores"] >= 1 and c["sample"]
    p = c["parity_of_timed_result"]
    assert p["nonzero_where_all_terms_zero"] == 0 and p["max_rel_err"] <= p["tolerance"] == 1e-4


def test_bench_epoch_workload_line():
    o = run_bench("--workload", "e1", "--steps", "5", "--warmup", "2")
    assert o["config"]["workload"] == "e1" and o["config"]["n_batches"] == 11 and o["value"] > 0
    assert o["cpu_baseline"]["kind"] == "oracle" and o["cpu_baseline"]["parity_of_one_epoch"]["ok"] is True
