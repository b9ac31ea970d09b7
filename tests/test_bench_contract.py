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
    assert "default c2" in text
