"""Seeded synthetic workloads: graphs in CSR and dense feature matrices.

Inputs only.  Nothing in this sub-package computes any step of the fused
SDDMM-SpMM method; both the GPU library's tests and the CPU oracle's tests are
fed from here, and neither depends on it for anything but arrays.

The heavy lifting is in ``graphgen.c`` (plain C + OpenMP), loaded through
ctypes.  The graphs stand in for the paper's real-world graphs and R-MAT
sweeps (Section V, Table V and the parameter-sensitivity experiment), which
are not available offline: same shapes, degree skew and value distributions,
not the same data.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "graphgen.c")
_LIB = os.path.join(_HERE, "libgraphgen.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile graphgen.c with gcc (host code only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB):
        build()
    lib = ctypes.CDLL(_LIB)
    i32, i64, u64, f32, f64 = ctypes.c_int32, ctypes.c_int64, ctypes.c_uint64, ctypes.c_float, ctypes.c_double
    vp = ctypes.c_void_p
    lib.synth_ctr_u64.restype = u64
    lib.synth_ctr_u64.argtypes = [u64, u64, u64]
    lib.synth_fill_uniform.restype = None
    lib.synth_fill_uniform.argtypes = [vp, i64, u64, f32, f32]
    lib.synth_fill_normal.restype = None
    lib.synth_fill_normal.argtypes = [vp, i64, u64]
    lib.synth_fill_int.restype = None
    lib.synth_fill_int.argtypes = [vp, i64, u64, i32, i32]
    lib.synth_permutation.restype = ctypes.c_int
    lib.synth_permutation.argtypes = [i64, u64, vp]
    lib.synth_rmat_pairs.restype = None
    lib.synth_rmat_pairs.argtypes = [i32, i64, f64, f64, f64, u64, vp, vp]
    lib.synth_chunglu_pairs.restype = None
    lib.synth_chunglu_pairs.argtypes = [i64, i64, f64, u64, vp, vp]
    lib.synth_er_pairs.restype = i64
    lib.synth_er_pairs.argtypes = [i64, i64, u64, vp, vp]
    lib.synth_build_csr.restype = i64
    lib.synth_build_csr.argtypes = [i64, i64, vp, vp, vp, i32, vp, vp]
    lib.synth_sym_norm_values.restype = None
    lib.synth_sym_norm_values.argtypes = [i64, vp, vp, vp]
    lib.synth_num_threads.restype = i32
    lib.synth_num_threads.argtypes = []
    _lib = lib
    return lib


def _p(a: np.ndarray) -> int:
    return a.ctypes.data


def num_threads() -> int:
    return int(_load().synth_num_threads())


# --------------------------------------------------------------------------- #
# dense fills
# --------------------------------------------------------------------------- #

def fill_uniform(shape, seed: int, lo: float, hi: float) -> np.ndarray:
    out = np.empty(shape, dtype=np.float32)
    _load().synth_fill_uniform(_p(out), out.size, seed, lo, hi)
    return out


def fill_normal(shape, seed: int) -> np.ndarray:
    out = np.empty(shape, dtype=np.float32)
    _load().synth_fill_normal(_p(out), out.size, seed)
    return out


def fill_int(shape, seed: int, lo: int, hi: int) -> np.ndarray:
    out = np.empty(shape, dtype=np.float32)
    _load().synth_fill_int(_p(out), out.size, seed, lo, hi)
    return out


# --------------------------------------------------------------------------- #
# graphs
# --------------------------------------------------------------------------- #

@dataclass
class CSR:
    """m x n sparsity pattern, 0-based, int64 rowptr, int32 colidx."""
    m: int
    n: int
    rowptr: np.ndarray
    colidx: np.ndarray
    values: Optional[np.ndarray] = None

    @property
    def nnz(self) -> int:
        return int(self.rowptr[-1])

    def degrees(self) -> np.ndarray:
        return np.diff(self.rowptr)

    def take_rows(self, rows: np.ndarray) -> "CSR":
        """Rectangular slice: the chosen rows of A, all n columns (a minibatch)."""
        rows = np.asarray(rows, dtype=np.int64)
        deg = (self.rowptr[rows + 1] - self.rowptr[rows]).astype(np.int64)
        rp = np.zeros(len(rows) + 1, dtype=np.int64)
        np.cumsum(deg, out=rp[1:])
        idx = np.repeat(self.rowptr[rows] - rp[:-1], deg) + np.arange(rp[-1], dtype=np.int64)
        vals = None if self.values is None else self.values[idx].copy()
        return CSR(len(rows), self.n, rp, self.colidx[idx].copy(), vals)


def permutation(n: int, seed: int) -> np.ndarray:
    perm = np.empty(n, dtype=np.int32)
    if _load().synth_permutation(n, seed, _p(perm)) != 0:
        raise MemoryError("synth_permutation")
    return perm


def csr_from_pairs(n: int, src: np.ndarray, dst: np.ndarray, perm: Optional[np.ndarray],
                   symmetrise: bool = True) -> CSR:
    src = np.ascontiguousarray(src, dtype=np.int32)
    dst = np.ascontiguousarray(dst, dtype=np.int32)
    npairs = len(src)
    rowptr = np.empty(n + 1, dtype=np.int64)
    colidx = np.empty(max(1, npairs * (2 if symmetrise else 1)), dtype=np.int32)
    pp = 0 if perm is None else _p(np.ascontiguousarray(perm, dtype=np.int32))
    nnz = _load().synth_build_csr(n, npairs, _p(src), _p(dst), pp, int(symmetrise), _p(rowptr), _p(colidx))
    if nnz < 0:
        raise MemoryError("synth_build_csr")
    return CSR(n, n, rowptr, colidx[:nnz].copy())


def erdos_renyi(n: int, n_undirected: int, seed: int) -> CSR:
    """G(n, M): M distinct unordered pairs, no loops, stored in both directions."""
    src = np.empty(max(1, n_undirected), dtype=np.int32)
    dst = np.empty(max(1, n_undirected), dtype=np.int32)
    got = _load().synth_er_pairs(n, n_undirected, seed, _p(src), _p(dst))
    if got < 0:
        raise MemoryError("synth_er_pairs")
    return csr_from_pairs(n, src[:got], dst[:got], None, True)


def rmat(scale: int, n_pairs: int, seed: int, a: float = 0.57, b: float = 0.19, c: float = 0.19,
         relabel: bool = True, symmetrise: bool = True) -> CSR:
    """R-MAT pairs -> drop loops -> (relabel) -> symmetrise -> dedup -> CSR."""
    n = 1 << scale
    src = np.empty(n_pairs, dtype=np.int32)
    dst = np.empty(n_pairs, dtype=np.int32)
    _load().synth_rmat_pairs(scale, n_pairs, a, b, c, seed, _p(src), _p(dst))
    perm = permutation(n, seed + 7919) if relabel else None
    return csr_from_pairs(n, src, dst, perm, symmetrise)


def chung_lu(n: int, n_pairs: int, i0: float, seed: int, relabel: bool = True) -> CSR:
    """Power-law expected degrees, weight of vertex i ~ (i + i0)^(-1/2)."""
    src = np.empty(n_pairs, dtype=np.int32)
    dst = np.empty(n_pairs, dtype=np.int32)
    _load().synth_chunglu_pairs(n, n_pairs, i0, seed, _p(src), _p(dst))
    perm = permutation(n, seed + 7919) if relabel else None
    return csr_from_pairs(n, src, dst, perm, True)


def sym_norm_values(csr: CSR) -> np.ndarray:
    """a_uv = 1/sqrt(deg_u deg_v) on a square symmetric pattern."""
    assert csr.m == csr.n
    vals = np.empty(max(1, csr.nnz), dtype=np.float32)
    _load().synth_sym_norm_values(csr.m, _p(csr.rowptr), _p(csr.colidx), _p(vals))
    return vals[:csr.nnz]


# --------------------------------------------------------------------------- #
# the five benchmark workloads
# --------------------------------------------------------------------------- #

@dataclass
class Workload:
    name: str
    pattern: str          # "one_minus_sigmoid" | "gcn" | "tdist" | ...
    d: int
    csr: CSR
    X: np.ndarray
    Y: np.ndarray         # may be the same object as X
    description: str


WORKLOADS = ("c1", "c2", "c3", "c4", "c5")


def make_workload(name: str, d: Optional[int] = None, relabel: bool = True) -> Workload:
    """The five synthetic configurations (graph, features, pattern).

    c1  Erdos-Renyi n=4096, 16384 undirected pairs, d=64, 1-sigmoid embedding
    c2  R-MAT scale 17, 2^16*16 pairs, d=128, 1-sigmoid embedding
    c3  Chung-Lu n=232965, 57e6 pairs (avg degree ~490), d=128, GCN sum
    c4  R-MAT scale 20, 2^20*16 pairs, d=128, t-distribution
    c5  R-MAT scale 22, 2^21*32 pairs, d=256, 1-sigmoid embedding, X != Y
    """
    name = name.lower()
    if name == "c1":
        dd = d or 64
        g = erdos_renyi(4096, 16384, 1001)
        X = fill_uniform((g.m, dd), 2001, -0.5, 0.5)
        return Workload(name, "one_minus_sigmoid", dd, g, X, X,
                        "Erdos-Renyi n=4096 M=16384 undirected, X=Y U[-0.5,0.5)")
    if name == "c2":
        dd = d or 128
        g = rmat(17, (1 << 16) * 16, 1002, relabel=relabel)
        X = fill_uniform((g.m, dd), 2002, -0.5, 0.5)
        return Workload(name, "one_minus_sigmoid", dd, g, X, X,
                        "R-MAT(0.57,0.19,0.19,0.05) scale 17, 2^20 pairs symmetrised, X=Y U[-0.5,0.5)")
    if name == "c3":
        dd = d or 128
        g = chung_lu(232965, 57_000_000, 200.0, 1003, relabel=relabel)
        g.values = sym_norm_values(g)
        X = fill_normal((g.m, dd), 2003)
        return Workload(name, "gcn", dd, g, X, X,
                        "Chung-Lu n=232965, 57M pairs symmetrised, a_uv=1/sqrt(deg_u deg_v), X=Y N(0,1)")
    if name == "c4":
        dd = d or 128
        g = rmat(20, (1 << 20) * 16, 1004, relabel=relabel)
        X = fill_uniform((g.m, dd), 2004, -1.0, 1.0)
        return Workload(name, "tdist", dd, g, X, X,
                        "R-MAT scale 20, 2^24 pairs symmetrised, X=Y U[-1,1)")
    if name == "c5":
        dd = d or 256
        g = rmat(22, (1 << 21) * 32, 1005, relabel=relabel)
        X = fill_uniform((g.m, dd), 2005, -0.5, 0.5)
        Y = fill_uniform((g.n, dd), 3005, -0.5, 0.5)
        return Workload(name, "one_minus_sigmoid", dd, g, X, Y,
                        "R-MAT scale 22, 2^26 pairs symmetrised, X!=Y U[-0.5,0.5)")
    if name.startswith("rmat:"):
        # density sweeps (the paper's sensitivity experiment: an R-MAT graph whose edge count is doubled
        # repeatedly): "rmat:SCALE:PAIRS", sigmoid-embedding pattern, features as c2
        try:
            _, scale, pairs = name.split(":")
            scale, pairs = int(scale), int(pairs)
        except ValueError:
            raise ValueError(f"workload {name!r}: expected rmat:SCALE:PAIRS") from None
        if not (4 <= scale <= 24 and 1 <= pairs <= (1 << 28)):
            raise ValueError(f"workload {name!r}: scale 4..24, pairs 1..2^28")
        dd = d or 128
        g = rmat(scale, pairs, 1100 + scale, relabel=relabel)
        X = fill_uniform((g.m, dd), 2100 + scale, -0.5, 0.5)
        return Workload(name, "one_minus_sigmoid", dd, g, X, X,
                        f"R-MAT scale {scale}, {pairs} pairs symmetrised, X=Y U[-0.5,0.5)")
    raise ValueError(f"unknown workload {name!r}")


# --------------------------------------------------------------------------- #
# minibatch embedding epochs (inputs of the end-to-end training experiment)
# --------------------------------------------------------------------------- #

@dataclass
class EpochWorkload:
    name: str
    d: int
    batch_rows: int
    n_negative: int
    lr: float
    csr: CSR
    X0: np.ndarray
    negatives: np.ndarray   # (n_batches, n_negative) int32, shared by the rows of a batch
    description: str


EPOCH_WORKLOADS = ("e1", "e2")


def make_epoch_workload(name: str) -> EpochWorkload:
    """Synthetic stand-ins with the sizes of the two citation graphs the paper trains on
    (2 708 vertices / 5 278 edges and 19 717 / 44 324; maximum degree about 170): Chung-Lu
    patterns with a power-law tail, d = 128, batches of 256 vertices, 5 negative samples per
    batch, embedding U[-0.5, 0.5)."""
    name = name.lower()
    spec = {"e1": (2708, 5278, 0.5, 1101, 2101, 3101), "e2": (19717, 44324, 4.0, 1102, 2102, 3102)}
    if name not in spec:
        raise ValueError(f"unknown epoch workload {name!r}")
    n, pairs, i0, gseed, xseed, nseed = spec[name]
    d, batch_rows, s = 128, 256, 5
    g = chung_lu(n, pairs, i0, gseed)
    X0 = fill_uniform((n, d), xseed, -0.5, 0.5)
    nb = (n + batch_rows - 1) // batch_rows
    negatives = fill_int((nb, s), nseed, 0, n - 1).astype(np.int32)
    return EpochWorkload(name, d, batch_rows, s, 0.02, g, X0, negatives,
                         f"Chung-Lu n={n}, {pairs} pairs symmetrised, d={d}, batch {batch_rows}, {s} negatives per batch")
