"""CPU oracle for FusedMM -- TEST INFRASTRUCTURE ONLY.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  The GPU library never does, and this
package never imports the GPU library or its binding.

``fusedmm_oracle.c`` is compiled twice with gcc: ``ORACLE_REAL=double`` (the
parity reference) and ``ORACLE_REAL=float`` (only timed, as the unfused CPU
baseline).  See the header of that file for what is computed and which
passages of the paper it follows.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fusedmm_oracle.c")
_LIBS = {"f64": os.path.join(_HERE, "liboracle_f64.so"), "f32": os.path.join(_HERE, "liboracle_f32.so")}
_loaded = {}

VOP = {"MUL": 0, "SEL2ND": 1, "SUB": 2, "ADD": 3}
ROP = {"NOOP": 0, "RSUM": 1, "SUMSQ": 2, "NORM": 3, "RMUL": 4}
SOP = {"EDGE_VALUE": 0, "SIGMOID": 1, "ONE_MINUS_SIGMOID": 2, "INV1P": 3, "SCAL": 4, "NOOP": 5}
MOP = {"MUL_Y": 0, "MUL_T": 1, "SEL2ND": 2}
AOP = {"ASUM": 0, "AMAX": 1, "AMIN": 2, "AMEAN": 3}

# (VOP, ROP, SOP, MOP) of the application patterns; AOP is always ASUM.
# Table III rows 1-3 and the t-distribution pattern of the author notes.
PATTERNS = {
    "sigmoid": ("MUL", "RSUM", "SIGMOID", "MUL_Y"),
    "one_minus_sigmoid": ("MUL", "RSUM", "ONE_MINUS_SIGMOID", "MUL_Y"),
    "gcn": ("SEL2ND", "NOOP", "EDGE_VALUE", "MUL_Y"),
    "tdist": ("SUB", "SUMSQ", "INV1P", "MUL_T"),
    "fr": ("SUB", "NORM", "SCAL", "MUL_T"),
}


def build(force: bool = False) -> None:
    for suffix, real in (("f64", "double"), ("f32", "float")):
        out = _LIBS[suffix]
        if force or not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(_SRC):
            cmd = ["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared", "-std=c11",
                   f"-DORACLE_REAL={real}", f"-DORACLE_SUFFIX={suffix}", "-o", out, _SRC, "-lm"]
            subprocess.run(cmd, check=True)


def _lib(suffix: str):
    if suffix not in _loaded:
        if not os.path.exists(_LIBS[suffix]):
            build()
        _loaded[suffix] = ctypes.CDLL(_LIBS[suffix])
    return _loaded[suffix]


def _ptr(a: Optional[np.ndarray]) -> ctypes.c_void_p:
    return ctypes.c_void_p(0 if a is None else a.ctypes.data)


def _prep(rowptr, colidx, values, X, Y):
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int64)
    colidx = np.ascontiguousarray(colidx, dtype=np.int32)
    values = None if values is None else np.ascontiguousarray(values, dtype=np.float32)
    X = None if X is None else np.ascontiguousarray(X, dtype=np.float32)
    Y = np.ascontiguousarray(Y, dtype=np.float32)
    return rowptr, colidx, values, X, Y


def _codes(ops):
    if isinstance(ops, str):
        ops = PATTERNS[ops]
    v, r, s, mo = ops
    if v == "ADD" or r == "RMUL" or s == "NOOP" or mo == "SEL2ND" or (r == "NOOP") != (s == "EDGE_VALUE"):
        raise ValueError(f"{ops}: outside the scalar-message patterns; use unfused_general")
    return VOP[v], ROP[r], SOP[s], MOP[mo]


def unfused(rowptr, colidx, values, X, Y, ops, alpha: float = 1.0, precision: str = "f64",
            want_abs: bool = True) -> Tuple[np.ndarray, Optional[np.ndarray], np.ndarray]:
    """Two-phase reference: SDDMM writes H (nnz scalars), SpMM reads it.

    Returns (Z, S, H): Z the m x d result, S the per-entry sum of |terms| (or
    None), H the materialised edge messages.  ``X`` may be None for the GCN
    pattern.  ``precision`` "f64" is the parity reference; "f32" exists only to
    be timed.
    """
    rowptr, colidx, values, X, Y = _prep(rowptr, colidx, values, X, Y)
    vop, rop, sop, mop = _codes(ops)
    m = len(rowptr) - 1
    d = Y.shape[1]
    nnz = int(rowptr[-1])
    real = np.float64 if precision == "f64" else np.float32
    lib = _lib(precision)
    H = np.empty(max(1, nnz), dtype=real)
    Z = np.empty((m, d), dtype=real)
    S = np.empty((m, d), dtype=real) if want_abs else None
    ldx = 0 if X is None else X.shape[1]
    i64, dbl, ci = ctypes.c_int64, ctypes.c_double, ctypes.c_int
    rc = getattr(lib, f"fmm_oracle_sddmm_{precision}")(
        i64(m), i64(d), _ptr(rowptr), _ptr(colidx), _ptr(values), _ptr(X), i64(ldx), _ptr(Y), i64(d),
        ci(vop), ci(rop), ci(sop), dbl(alpha), _ptr(H))
    if rc != 0:
        raise ValueError(f"oracle sddmm failed ({rc}): EDGE_VALUE needs values")
    rc = getattr(lib, f"fmm_oracle_spmm_{precision}")(
        i64(m), i64(d), _ptr(rowptr), _ptr(colidx), _ptr(X), i64(ldx), _ptr(Y), i64(d),
        ci(vop), ci(mop), _ptr(H), _ptr(Z), _ptr(S))
    if rc != 0:
        raise ValueError(f"oracle spmm failed ({rc})")
    return Z, S, H[:nnz]


def unfused_general(rowptr, colidx, values, X, Y, ops, aop: str = "ASUM", alpha: float = 1.0):
    """The general five-step path (all operations of Table II), two phases, fp64.

    ``ops`` = (VOP, ROP, SOP, MOP) names, ``aop`` in ASUM / AMAX / AMIN / AMEAN.  Returns (Z, S, H);
    H is nnz scalars, or nnz x d when the message is a vector (ROP is NOOP and SOP is not
    EDGE_VALUE).  S is sum|w| for ASUM, max|w| for AMAX / AMIN and mean|w| for AMEAN.
    """
    rowptr, colidx, values, X, Y = _prep(rowptr, colidx, values, X, Y)
    v, r, s_, mo = ops
    vop, rop, sop, mop, aopc = VOP[v], ROP[r], SOP[s_], MOP[mo], AOP[aop]
    m = len(rowptr) - 1
    d = Y.shape[1]
    nnz = int(rowptr[-1])
    lib = _lib("f64")
    vec = int(lib.fmm_oracle_h_is_vector_f64(ctypes.c_int(rop), ctypes.c_int(sop)))
    H = np.empty(max(1, nnz) * (d if vec else 1), dtype=np.float64)
    Z = np.empty((m, d), dtype=np.float64)
    S = np.empty((m, d), dtype=np.float64)
    ldx = 0 if X is None else X.shape[1]
    i64, dbl, ci = ctypes.c_int64, ctypes.c_double, ctypes.c_int
    rc = lib.fmm_oracle_sddmm_general_f64(i64(m), i64(d), _ptr(rowptr), _ptr(colidx), _ptr(values), _ptr(X), i64(ldx),
                                          _ptr(Y), i64(d), ci(vop), ci(rop), ci(sop), dbl(alpha), _ptr(H))
    if rc != 0:
        raise ValueError(f"oracle general sddmm failed ({rc})")
    rc = lib.fmm_oracle_spmm_general_f64(i64(m), i64(d), _ptr(rowptr), _ptr(colidx), _ptr(X), i64(ldx), _ptr(Y), i64(d),
                                         ci(vop), ci(mop), ci(aopc), ci(vec), _ptr(H), _ptr(Z), _ptr(S))
    if rc != 0:
        raise ValueError(f"oracle general spmm failed ({rc})")
    H = H[:nnz * d].reshape(nnz, d) if vec else H[:nnz]
    return Z, S, H


def message_tensor(rowptr, colidx, values, X, Y, ops, alpha: float = 1.0):
    """(W, Z): the full nnz x d message tensor and its row-wise aggregation."""
    rowptr, colidx, values, X, Y = _prep(rowptr, colidx, values, X, Y)
    vop, rop, sop, mop = _codes(ops)
    m = len(rowptr) - 1
    d = Y.shape[1]
    nnz = int(rowptr[-1])
    lib = _lib("f64")
    W = np.empty((max(1, nnz), d), dtype=np.float64)
    Z = np.empty((m, d), dtype=np.float64)
    ldx = 0 if X is None else X.shape[1]
    i64, dbl, ci = ctypes.c_int64, ctypes.c_double, ctypes.c_int
    rc = lib.fmm_oracle_message_tensor_f64(
        i64(m), i64(d), _ptr(rowptr), _ptr(colidx), _ptr(values), _ptr(X), i64(ldx), _ptr(Y), i64(d),
        ci(vop), ci(rop), ci(sop), ci(mop), dbl(alpha), _ptr(W))
    if rc != 0:
        raise ValueError("oracle message_tensor failed")
    lib.fmm_oracle_aggregate_tensor_f64(i64(m), i64(d), _ptr(rowptr), _ptr(W), _ptr(Z))
    return W[:nnz], Z


def update_u(rowptr, colidx, values, X, Y, ops, alpha: float = 1.0) -> np.ndarray:
    """Algorithm 1 (UpdateU for every row), five steps per stored entry, in double."""
    rowptr, colidx, values, X, Y = _prep(rowptr, colidx, values, X, Y)
    vop, rop, sop, mop = _codes(ops)
    m = len(rowptr) - 1
    d = Y.shape[1]
    Z = np.empty((m, d), dtype=np.float64)
    ldx = 0 if X is None else X.shape[1]
    i64, dbl, ci = ctypes.c_int64, ctypes.c_double, ctypes.c_int
    rc = _lib("f64").fmm_oracle_update_u_all_f64(
        i64(m), i64(d), _ptr(rowptr), _ptr(colidx), _ptr(values), _ptr(X), i64(ldx), _ptr(Y), i64(d),
        ci(vop), ci(rop), ci(sop), ci(mop), dbl(alpha), _ptr(Z))
    if rc != 0:
        raise ValueError("oracle update_u failed")
    return Z


def compare(Z_test: np.ndarray, Z_ref: np.ndarray, S: np.ndarray):
    """Error measure of the parity tests.

    err[u,k] = |Z_test - Z_ref| / S where S > 0; where S == 0 (empty row, or
    every term zero) Z_test must be exactly 0.  Returns (max_err, argmax_flat,
    n_exact_zero_violations).
    """
    Zt = np.asarray(Z_test, dtype=np.float64)
    diff = np.abs(Zt - Z_ref)
    pos = S > 0
    viol = int(np.count_nonzero(Zt[~pos] != 0.0))
    if not pos.any():
        return 0.0, -1, viol
    rel = np.zeros_like(diff)
    rel[pos] = diff[pos] / S[pos]
    if not np.isfinite(Zt).all():
        return float("inf"), int(np.argmax(~np.isfinite(Zt))), viol
    am = int(np.argmax(rel))
    return float(rel.flat[am]), am, viol


# --------------------------------------------------------------------------- #
# minibatch embedding epoch (the end-to-end experiment of Section V, Table VIII)
# --------------------------------------------------------------------------- #

def embedding_epoch(rowptr, colidx, X0, batch_rows: int, negatives, lr: float):
    """One epoch of minibatch graph embedding built from two FusedMM calls per batch.

    The paper's end-to-end experiment (Section V, Table VIII: d = 128, batches of 256 vertices)
    trains an embedding with the sigmoid pattern of Table III but does not print the update
    rule; minibatching is left to the application (Section III-C).  The reading taken here, for
    batch B_i = rows [i*batch_rows, (i+1)*batch_rows) of the square adjacency matrix, in order:

        Zpos = FusedMM(A[B_i, :], X[B_i], X)   with (MUL, RSUM, 1-SIGMOID, MUL, ASUM)
        Zneg = FusedMM(N_i,       X[B_i], X)   with (MUL, RSUM,   SIGMOID, MUL, ASUM)
        X[B_i] <- X[B_i] + lr * (Zpos - Zneg)

    where N_i is the |B_i| x n pattern whose every row holds the batch's negative samples
    ``negatives[i]`` (shared by the rows of a batch).  This is one ascent step, with respect to
    the batch's own rows, on  sum_{v in N(u)} log sigma(x_u.x_v) + sum_{w in neg} log(1 - sigma(x_u.x_w)).
    The embedding is stored in fp32 (the paper's storage type): both FusedMM calls of a batch read
    the matrix as the batches before it left it, the update is computed in double and rounded to
    fp32 once per batch.  Returns (X, S): the embedding after the epoch (float32) and, per
    element, lr * (sum of |terms| of both calls), the scale its rounding error is measured on.
    """
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int64)
    colidx = np.ascontiguousarray(colidx, dtype=np.int32)
    negatives = np.ascontiguousarray(negatives, dtype=np.int32)
    X = np.array(X0, dtype=np.float32, copy=True)
    n, d = X.shape
    assert len(rowptr) == n + 1, "square adjacency matrix expected"
    n_batches = (n + batch_rows - 1) // batch_rows
    assert negatives.shape[0] == n_batches
    s = negatives.shape[1]
    S = np.zeros((n, d), dtype=np.float64)
    for i in range(n_batches):
        b0, b1 = i * batch_rows, min(n, (i + 1) * batch_rows)
        rows = b1 - b0
        rp = rowptr[b0:b1 + 1] - rowptr[b0]
        ci = colidx[rowptr[b0]:rowptr[b1]]
        Xb = X[b0:b1].copy()
        Zpos, Spos, _ = unfused(rp, ci, None, Xb, X, "one_minus_sigmoid")
        nrp = np.arange(rows + 1, dtype=np.int64) * s
        nci = np.tile(negatives[i], rows)
        Zneg, Sneg, _ = unfused(nrp, nci, None, Xb, X, "sigmoid")
        X[b0:b1] = (Xb.astype(np.float64) + lr * (Zpos - Zneg)).astype(np.float32)
        S[b0:b1] = lr * (Spos + Sneg)
    return X, S
