"""Build libfusedmm.so (HIP, gfx950) in-tree with hipcc.

Cross-compiles without a GPU.  Objects go to ``_build/`` (not committed); the
shared library lands next to this file so that it travels with the tree.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libfusedmm.so")

SOURCES = [
    "fusedmm_api.hip",
    "fusedmm_plan.hip",
    "fusedmm_generic.hip",
    "fusedmm_minibatch.hip",
    "fusedmm_small.hip",
    "fusedmm_fast_d32.hip",
    "fusedmm_fast_d64.hip",
    "fusedmm_fast_d96.hip",
    "fusedmm_fast_d128.hip",
    "fusedmm_fast_d192.hip",
    "fusedmm_fast_d256.hip",
    "fusedmm_fast_d384.hip",
    "fusedmm_fast_d512.hip",
    "fusedmm_fast_d768.hip",
    "fusedmm_fast_d1024.hip",
    "fusedmm_fast_d1536.hip",
    "fusedmm_fast_d2048.hip",
    "fusedmm_fast_f64_d32.hip",
    "fusedmm_fast_f64_d64.hip",
    "fusedmm_fast_f64_d128.hip",
    "fusedmm_fast_f64_d256.hip",
    "fusedmm_fast_f64_d512.hip",
    "fusedmm_fast_f64_d1024.hip",
    "fusedmm_fast_f64_d2048.hip",
]

# packed FP32 instructions are switched off for all device code
HIPCC_FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def _compile(src: str) -> str:
    obj = os.path.join(BUILD, os.path.splitext(src)[0] + ".o")
    cmd = ["hipcc", *HIPCC_FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{r.stdout}\n{r.stderr}")
    return obj


def build(jobs: int = 8, verbose: bool = False) -> str:
    os.makedirs(BUILD, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = ["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    if verbose:
        print(f"built {LIB}")
    return LIB


MICROBENCH_SRC = "bench_l2_delivery.hip"
MICROBENCH = os.path.join(HERE, "bench_l2_delivery")


def build_microbench(verbose: bool = False) -> str:
    """The load-only delivery-rate microbenchmark: a stand-alone program, not linked into the library."""
    cmd = ["hipcc", *[f for f in HIPCC_FLAGS if f != "-fPIC"], "-o", MICROBENCH, os.path.join(CSRC, MICROBENCH_SRC)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {MICROBENCH_SRC}:\n{r.stdout}\n{r.stderr}")
    if verbose:
        print(f"built {MICROBENCH}")
    return MICROBENCH


EXAMPLE_SRC = "example_c_abi.c"
EXAMPLE = os.path.join(HERE, "example_c_abi")


def build_example(verbose: bool = False) -> str:
    """The plain-C user of the library (gcc, C99): links libfusedmm.so and the HIP runtime, nothing else."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-std=c99", "-O2", "-Wall", "-Wextra", "-I", os.path.join(rocm, "include"), os.path.join(CSRC, EXAMPLE_SRC),
           "-o", EXAMPLE, "-L", HERE, "-lfusedmm", "-L", os.path.join(rocm, "lib"), "-lamdhip64",
           "-Wl,-rpath,$ORIGIN", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"gcc failed for {EXAMPLE_SRC}:\n{r.stdout}\n{r.stderr}")
    if verbose:
        print(f"built {EXAMPLE}")
    return EXAMPLE


if __name__ == "__main__":
    if sys.argv[1:] == ["microbench"]:
        build_microbench(verbose=True)
    elif sys.argv[1:] == ["example"]:
        build_example(verbose=True)
    else:
        build(verbose=True)
    sys.exit(0)
