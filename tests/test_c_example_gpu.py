"""The library used from plain C (csrc/example_c_abi.c: gcc, C99, no Python or torch in the process): a GCN sum
over integer features on a graph with hub rows, compared bit for bit with its closed form inside the program."""
import os
import subprocess

import pytest

from paper_2011_06391_amd import build

pytestmark = pytest.mark.gpu


def test_plain_c_program_runs_the_library():
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (torch.cuda.is_available() is False)")
    if not os.path.exists(build.LIB):
        pytest.fail("libfusedmm.so is not built")
    if not os.path.exists(build.EXAMPLE):
        build.build_example()     # gcc only: seconds
    r = subprocess.run([build.EXAMPLE], capture_output=True, text=True, timeout=110)
    assert r.returncode == 0, r.stdout + r.stderr
    assert r.stdout.strip().endswith("ok"), r.stdout
    assert "tiled rows 100" in r.stdout, r.stdout      # the hub rows were cut by column class and merged
