"""bench.py's command-line contract that can be checked without a GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run_bench(*args, env=None):
    e = dict(os.environ)
    e.update(env or {})
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          env=e, timeout=120)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = run_bench("--gpus", "2")
    assert r.returncode != 0 and "one GPU" in (r.stderr + r.stdout)
    r = run_bench("--gpus", "1", env={"WORLD_SIZE": "4"})
    assert r.returncode != 0 and "one GPU" in (r.stderr + r.stdout)


def test_defaults_name_the_headline_workload():
    r = run_bench("--help")
    assert r.returncode == 0
    text = r.stdout
    for flag in ("--gpus", "--steps", "--warmup", "--workload", "--no-cpu-baseline"):
        assert flag in text
    assert "default c5" in text and "--natural-order" in text and "--all-workloads" in text


def test_traffic_table_rows_are_well_formed():
    """profiles/hbm_traffic_per_launch.txt is read by bench.py: every data row has the nine fields it parses,
    and a row only counts for the build whose kernel sources it names."""
    sys.path.insert(0, ROOT)
    import bench
    sha = bench.kernel_sources_sha16()
    assert len(sha) == 16 and int(sha, 16) >= 0
    if os.path.exists(bench.TRAFFIC_TABLE):
        for line in open(bench.TRAFFIC_TABLE):
            f = line.split("#")[0].split()
            if not f:
                continue
            assert len(f) == 9, line
            assert len(f[1]) == 16 and all(int(x) >= 0 for x in f[2:7]) and 0.0 <= float(f[7]) <= 1.0
    t, hit, why = bench.measured_traffic("no-such-workload", {"partials": 0, "tile_segments": 0, "column_classes": 1})
    assert t is None and hit is None and why


def test_traffic_table_belongs_to_the_current_kernel_sources():
    """bench.py prices roofline.frac on the measured bytes only when the table was written for the kernel sources
    in the tree; after a change to csrc/ the table has to be regenerated (profile_summary.py says how).  The
    headline workload and the three others bench.py reports must all be there."""
    sys.path.insert(0, ROOT)
    import bench
    sha = bench.kernel_sources_sha16()
    rows = {}
    for line in open(bench.TRAFFIC_TABLE):
        f = line.split("#")[0].split()
        if f:
            rows[f[0]] = f[1]
    for w in ("c2", "c3", "c4", "c5"):
        assert rows.get(w) == sha, f"profiles/hbm_traffic_per_launch.txt: the row of {w} is for other kernel sources"

