"""ctypes binding of libfusedmm.so -- argument marshalling only.

Function names mirror ``include/fusedmm.h``.  Device arrays are torch tensors
(PyTorch is used for device memory and streams, nothing else); their
``data_ptr()`` is handed to the C ABI.  There is no fallback: if the shared
library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfusedmm.so")

FUSEDMM_OK = 0
FUSEDMM_ERR_INVALID_ARG = 1
FUSEDMM_ERR_UNSUPPORTED_OPS = 2
FUSEDMM_ERR_UNSUPPORTED_DIM = 3
FUSEDMM_ERR_ALIAS = 4
FUSEDMM_ERR_ALLOC = 5
FUSEDMM_ERR_HIP = 6
FUSEDMM_ERR_NOT_RESERVED = 7
FUSEDMM_ERR_SCRATCH_LIMIT = 8
FUSEDMM_STATIC_SCRATCH_BYTES = 64 << 20

FUSEDMM_MAX_D = 2048

VOP = {"MUL": 0, "SEL2ND": 1, "SUB": 2, "ADD": 3}
ROP = {"NOOP": 0, "RSUM": 1, "SUMSQ": 2, "NORM2": 3, "RMUL": 4}
SOP = {"EDGE_VALUE": 0, "SIGMOID": 1, "ONE_MINUS_SIGMOID": 2, "INV_1P": 3, "SCAL": 4, "NOOP": 5}
MOP = {"MUL_Y": 0, "MUL_T": 1, "SEL2ND": 2}
AOP = {"SUM": 0, "MAX": 1, "MIN": 2, "MEAN": 3}
PATTERN = {"sigmoid": 0, "one_minus_sigmoid": 1, "gcn": 2, "tdist": 3, "fr": 4}

EXPORTS = (
    "fusedmm_version", "fusedmm_status_string", "fusedmm_ops_preset", "fusedmm_plan_create",
    "fusedmm_plan_reserve", "fusedmm_plan_reserve_f64", "fusedmm_plan_workspace_bytes", "fusedmm_plan_stats", "fusedmm_execute",
    "fusedmm_execute_static_scratch", "fusedmm_debug_edge_visits", "fusedmm_plan_set_profiling", "fusedmm_plan_read_profile",
    "fusedmm_plan_read_profile_samples",
    "fusedmm_plan_destroy", "fusedmm_debug_copy", "fusedmm_debug_kernel_size", "fusedmm_plan_create_tuned", "fusedmm_execute_bf16y",
    "fusedmm_to_bf16", "fusedmm_execute_f16y", "fusedmm_to_f16", "fusedmm_execute_f64",
    "fusedmm_minibatch_create", "fusedmm_minibatch_reserve", "fusedmm_minibatch_epoch",
    "fusedmm_minibatch_info", "fusedmm_minibatch_destroy",
)


class fusedmm_ops_t(ctypes.Structure):
    _fields_ = [("vop", ctypes.c_int32), ("rop", ctypes.c_int32), ("sop", ctypes.c_int32),
                ("mop", ctypes.c_int32), ("aop", ctypes.c_int32), ("alpha", ctypes.c_float)]


class fusedmm_plan_options_t(ctypes.Structure):
    _fields_ = [("small_row_max", ctypes.c_int32), ("split_row_min", ctypes.c_int32),
                ("chunk_edges", ctypes.c_int32), ("column_classes", ctypes.c_int32),
                ("tile_row_min", ctypes.c_int32), ("feature_dim_hint", ctypes.c_int32),
                ("general_kernel_only", ctypes.c_int32), ("host_threads", ctypes.c_int32)]


class FusedMMError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: status {status} ({fusedmm_status_string(status)})")


_lib = None


def load():
    """Load libfusedmm.so (built by paper_2011_06391_amd.build).  Raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            f"{LIB_PATH} not found: build it with `python -m paper_2011_06391_amd.build` "
            "(there is no CPU fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    lib.fusedmm_version.restype = ctypes.c_int
    lib.fusedmm_version.argtypes = []
    lib.fusedmm_status_string.restype = ctypes.c_char_p
    lib.fusedmm_status_string.argtypes = [ctypes.c_int]
    lib.fusedmm_ops_preset.restype = ctypes.c_int
    lib.fusedmm_ops_preset.argtypes = [ctypes.c_int, ctypes.POINTER(fusedmm_ops_t)]
    lib.fusedmm_plan_create.restype = ctypes.c_int
    lib.fusedmm_plan_create.argtypes = [ctypes.POINTER(vp), i64, i64, i64, vp, vp,
                                        ctypes.POINTER(fusedmm_plan_options_t), vp]
    lib.fusedmm_plan_create_tuned.restype = ctypes.c_int
    lib.fusedmm_plan_create_tuned.argtypes = [ctypes.POINTER(vp), i64, i64, i64, vp, vp, ctypes.POINTER(fusedmm_ops_t),
                                              i32, vp, vp, i64, vp, i64, vp, i64, vp,
                                              ctypes.POINTER(fusedmm_plan_options_t), ctypes.POINTER(ctypes.c_float)]
    lib.fusedmm_plan_reserve.restype = ctypes.c_int
    lib.fusedmm_plan_reserve.argtypes = [vp, i32]
    lib.fusedmm_plan_reserve_f64.restype = ctypes.c_int
    lib.fusedmm_plan_reserve_f64.argtypes = [vp, i32]
    lib.fusedmm_plan_workspace_bytes.restype = ctypes.c_int
    lib.fusedmm_plan_workspace_bytes.argtypes = [vp, i32, ctypes.POINTER(ctypes.c_size_t)]
    lib.fusedmm_plan_stats.restype = ctypes.c_int
    lib.fusedmm_plan_stats.argtypes = [vp] + [ctypes.POINTER(i64)] * 8
    lib.fusedmm_execute.restype = ctypes.c_int
    lib.fusedmm_execute.argtypes = [vp, ctypes.POINTER(fusedmm_ops_t), i32, vp, vp, i64, vp, i64, vp, i64, vp]
    lib.fusedmm_execute_static_scratch.restype = ctypes.c_int
    lib.fusedmm_execute_static_scratch.argtypes = [vp, ctypes.POINTER(fusedmm_ops_t), i32, vp, vp, i64, vp, i64, vp, i64, vp]
    lib.fusedmm_execute_bf16y.restype = ctypes.c_int
    lib.fusedmm_execute_bf16y.argtypes = [vp, ctypes.POINTER(fusedmm_ops_t), i32, vp, vp, i64, vp, i64, vp, i64, vp]
    lib.fusedmm_to_bf16.restype = ctypes.c_int
    lib.fusedmm_to_bf16.argtypes = [vp, vp, ctypes.c_size_t, vp]
    lib.fusedmm_execute_f16y.restype = ctypes.c_int
    lib.fusedmm_execute_f16y.argtypes = [vp, ctypes.POINTER(fusedmm_ops_t), i32, vp, vp, i64, vp, i64, vp, i64, vp]
    lib.fusedmm_to_f16.restype = ctypes.c_int
    lib.fusedmm_to_f16.argtypes = [vp, vp, ctypes.c_size_t, vp]
    lib.fusedmm_execute_f64.restype = ctypes.c_int
    lib.fusedmm_execute_f64.argtypes = [vp, ctypes.POINTER(fusedmm_ops_t), i32, vp, vp, i64, vp, i64, vp, i64, vp]
    lib.fusedmm_debug_edge_visits.restype = ctypes.c_int
    lib.fusedmm_debug_edge_visits.argtypes = [vp, i32, i32, vp, vp]
    lib.fusedmm_plan_set_profiling.restype = ctypes.c_int
    lib.fusedmm_plan_set_profiling.argtypes = [vp, i32]
    lib.fusedmm_plan_read_profile.restype = ctypes.c_int
    lib.fusedmm_plan_read_profile.argtypes = [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double),
                                              ctypes.POINTER(i64)]
    lib.fusedmm_plan_read_profile_samples.restype = ctypes.c_int
    lib.fusedmm_plan_read_profile_samples.argtypes = [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double),
                                                      i64, ctypes.POINTER(i64)]
    lib.fusedmm_debug_kernel_size.restype = ctypes.c_int
    lib.fusedmm_debug_kernel_size.argtypes = [ctypes.c_int32, ctypes.c_int32]
    lib.fusedmm_debug_copy.restype = ctypes.c_int
    lib.fusedmm_debug_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
    lib.fusedmm_plan_destroy.restype = ctypes.c_int
    lib.fusedmm_plan_destroy.argtypes = [vp]
    lib.fusedmm_minibatch_create.restype = ctypes.c_int
    lib.fusedmm_minibatch_create.argtypes = [ctypes.POINTER(vp), i64, i64, vp, vp, i32, i32, vp, vp]
    lib.fusedmm_minibatch_reserve.restype = ctypes.c_int
    lib.fusedmm_minibatch_reserve.argtypes = [vp, i32]
    lib.fusedmm_minibatch_epoch.restype = ctypes.c_int
    lib.fusedmm_minibatch_epoch.argtypes = [vp, i32, ctypes.c_float, vp, i64, vp]
    lib.fusedmm_minibatch_info.restype = ctypes.c_int
    lib.fusedmm_minibatch_info.argtypes = [vp, ctypes.POINTER(i32), ctypes.POINTER(i64)]
    lib.fusedmm_minibatch_destroy.restype = ctypes.c_int
    lib.fusedmm_minibatch_destroy.argtypes = [vp]
    _lib = lib
    return lib


def _dptr(t) -> ctypes.c_void_p:
    return ctypes.c_void_p(0 if t is None else t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _check(status: int, where: str) -> None:
    if status != FUSEDMM_OK:
        raise FusedMMError(status, where)


# ---- thin mirrors of the C entry points ------------------------------------

def fusedmm_version() -> int:
    return int(load().fusedmm_version())


def fusedmm_status_string(status: int) -> str:
    return load().fusedmm_status_string(int(status)).decode()


def fusedmm_ops_preset(pattern) -> fusedmm_ops_t:
    ops = fusedmm_ops_t()
    code = PATTERN[pattern] if isinstance(pattern, str) else int(pattern)
    _check(load().fusedmm_ops_preset(code, ctypes.byref(ops)), "fusedmm_ops_preset")
    return ops


def make_ops(vop: str, rop: str, sop: str, mop: str, aop: str = "SUM", alpha: float = 1.0) -> fusedmm_ops_t:
    return fusedmm_ops_t(VOP[vop], ROP[rop], SOP[sop], MOP[mop], AOP[aop], alpha)


def fusedmm_plan_create(m: int, n: int, nnz: int, d_rowptr, d_colidx, options=None, stream=None) -> ctypes.c_void_p:
    plan = ctypes.c_void_p()
    opt = None
    if options is not None:
        opt = ctypes.byref(fusedmm_plan_options_t(options.get("small_row_max", 0), options.get("split_row_min", 0),
                                                  options.get("chunk_edges", 0), options.get("column_classes", 0),
                                                  options.get("tile_row_min", 0), options.get("feature_dim_hint", 0),
                                                  options.get("general_kernel_only", 0), options.get("host_threads", 0)))
    st = load().fusedmm_plan_create(ctypes.byref(plan), m, n, nnz, _dptr(d_rowptr), _dptr(d_colidx), opt,
                                    _stream(stream))
    _check(st, "fusedmm_plan_create")
    return plan


def fusedmm_plan_create_tuned(m: int, n: int, nnz: int, d_rowptr, d_colidx, ops: fusedmm_ops_t, d: int, d_values, d_X,
                              ldx: int, d_Y, ldy: int, d_Z, ldz: int, stream=None):
    """Returns (plan, chosen options as a dict, milliseconds per execute of the winner)."""
    plan, chosen, ms = ctypes.c_void_p(), fusedmm_plan_options_t(), ctypes.c_float()
    st = load().fusedmm_plan_create_tuned(ctypes.byref(plan), m, n, nnz, _dptr(d_rowptr), _dptr(d_colidx),
                                          ctypes.byref(ops), d, _dptr(d_values), _dptr(d_X), ldx, _dptr(d_Y), ldy,
                                          _dptr(d_Z), ldz, _stream(stream), ctypes.byref(chosen), ctypes.byref(ms))
    _check(st, "fusedmm_plan_create_tuned")
    opts = {"small_row_max": chosen.small_row_max, "split_row_min": chosen.split_row_min, "chunk_edges": chosen.chunk_edges,
            "column_classes": chosen.column_classes, "tile_row_min": chosen.tile_row_min,
            "feature_dim_hint": chosen.feature_dim_hint}
    return plan, opts, float(ms.value)


def fusedmm_plan_reserve(plan, d: int) -> None:
    _check(load().fusedmm_plan_reserve(plan, d), "fusedmm_plan_reserve")


def fusedmm_plan_reserve_f64(plan, d: int) -> None:
    _check(load().fusedmm_plan_reserve_f64(plan, d), "fusedmm_plan_reserve_f64")


def fusedmm_plan_workspace_bytes(plan, d: int) -> int:
    out = ctypes.c_size_t()
    _check(load().fusedmm_plan_workspace_bytes(plan, d, ctypes.byref(out)), "fusedmm_plan_workspace_bytes")
    return int(out.value)


def fusedmm_plan_stats(plan) -> dict:
    v = [ctypes.c_int64() for _ in range(8)]
    _check(load().fusedmm_plan_stats(plan, *[ctypes.byref(x) for x in v]), "fusedmm_plan_stats")
    keys = ("packed_rows", "wave_rows", "chunks", "split_rows", "partials", "tiled_rows", "tile_segments",
            "column_classes")
    return {k: int(x.value) for k, x in zip(keys, v)}


def fusedmm_execute(plan, ops: fusedmm_ops_t, d: int, d_values, d_X, ldx: int, d_Y, ldy: int, d_Z, ldz: int,
                    stream=None) -> None:
    st = load().fusedmm_execute(plan, ctypes.byref(ops), d, _dptr(d_values), _dptr(d_X), ldx, _dptr(d_Y), ldy,
                                _dptr(d_Z), ldz, _stream(stream))
    _check(st, "fusedmm_execute")


def fusedmm_execute_static_scratch(plan, ops: fusedmm_ops_t, d: int, d_values, d_X, ldx: int, d_Y, ldy: int, d_Z, ldz: int,
                                   stream=None) -> None:
    st = load().fusedmm_execute_static_scratch(plan, ctypes.byref(ops), d, _dptr(d_values), _dptr(d_X), ldx, _dptr(d_Y), ldy,
                                               _dptr(d_Z), ldz, _stream(stream))
    _check(st, "fusedmm_execute_static_scratch")


def fusedmm_execute_bf16y(plan, ops: fusedmm_ops_t, d: int, d_values, d_X, ldx: int, d_Y_bf16, ldy: int, d_Z, ldz: int,
                          stream=None) -> None:
    st = load().fusedmm_execute_bf16y(plan, ctypes.byref(ops), d, _dptr(d_values), _dptr(d_X), ldx, _dptr(d_Y_bf16), ldy,
                                      _dptr(d_Z), ldz, _stream(stream))
    _check(st, "fusedmm_execute_bf16y")


def fusedmm_to_bf16(d_dst, d_src, count: int, stream=None) -> None:
    _check(load().fusedmm_to_bf16(_dptr(d_dst), _dptr(d_src), count, _stream(stream)), "fusedmm_to_bf16")


def fusedmm_execute_f16y(plan, ops: fusedmm_ops_t, d: int, d_values, d_X, ldx: int, d_Y_f16, ldy: int, d_Z, ldz: int,
                         stream=None) -> None:
    st = load().fusedmm_execute_f16y(plan, ctypes.byref(ops), d, _dptr(d_values), _dptr(d_X), ldx, _dptr(d_Y_f16), ldy,
                                     _dptr(d_Z), ldz, _stream(stream))
    _check(st, "fusedmm_execute_f16y")


def fusedmm_execute_f64(plan, ops: fusedmm_ops_t, d: int, d_values, d_X, ldx: int, d_Y, ldy: int, d_Z, ldz: int,
                        stream=None) -> None:
    st = load().fusedmm_execute_f64(plan, ctypes.byref(ops), d, _dptr(d_values), _dptr(d_X), ldx, _dptr(d_Y), ldy,
                                    _dptr(d_Z), ldz, _stream(stream))
    _check(st, "fusedmm_execute_f64")


def fusedmm_to_f16(d_dst, d_src, count: int, stream=None) -> None:
    _check(load().fusedmm_to_f16(_dptr(d_dst), _dptr(d_src), count, _stream(stream)), "fusedmm_to_f16")


def fusedmm_debug_edge_visits(plan, d: int, fast_path, d_counts, stream=None) -> None:
    """fast_path: False / 0 the general kernel, True / 1 the specialised kernels, 2 their fp64 instances."""
    st = load().fusedmm_debug_edge_visits(plan, d, int(fast_path), _dptr(d_counts), _stream(stream))
    _check(st, "fusedmm_debug_edge_visits")


def fusedmm_plan_set_profiling(plan, enabled: bool) -> None:
    _check(load().fusedmm_plan_set_profiling(plan, int(enabled)), "fusedmm_plan_set_profiling")


def fusedmm_plan_read_profile(plan):
    """(main kernel ms sum incl. bracket cost, empty-bracket ms sum, calls)."""
    ms, empty, calls = ctypes.c_double(), ctypes.c_double(), ctypes.c_int64()
    _check(load().fusedmm_plan_read_profile(plan, ctypes.byref(ms), ctypes.byref(empty), ctypes.byref(calls)),
           "fusedmm_plan_read_profile")
    return float(ms.value), float(empty.value), int(calls.value)


def fusedmm_plan_read_profile_samples(plan, capacity: int = 4096):
    """(list of main-kernel ms incl. bracket cost, list of empty-bracket ms), one entry per timed call."""
    ms = (ctypes.c_double * capacity)()
    empty = (ctypes.c_double * capacity)()
    calls = ctypes.c_int64()
    _check(load().fusedmm_plan_read_profile_samples(plan, ms, empty, capacity, ctypes.byref(calls)),
           "fusedmm_plan_read_profile_samples")
    return list(ms[:calls.value]), list(empty[:calls.value])


def fusedmm_debug_kernel_size(d: int, storage: str = "f32") -> int:
    return load().fusedmm_debug_kernel_size(d, {"f32": 0, "bf16": 1, "f16": 1, "f64": 2}[storage])


def fusedmm_debug_copy(d_dst, d_src, nbytes: int, stream=None) -> None:
    _check(load().fusedmm_debug_copy(_dptr(d_dst), _dptr(d_src), nbytes, _stream(stream)), "fusedmm_debug_copy")


def fusedmm_plan_destroy(plan) -> None:
    _check(load().fusedmm_plan_destroy(plan), "fusedmm_plan_destroy")


def fusedmm_minibatch_create(n: int, nnz: int, d_rowptr, d_colidx, batch_rows: int, n_negative: int, d_negatives,
                             stream=None) -> ctypes.c_void_p:
    h = ctypes.c_void_p()
    _check(load().fusedmm_minibatch_create(ctypes.byref(h), n, nnz, _dptr(d_rowptr), _dptr(d_colidx), batch_rows,
                                           n_negative, _dptr(d_negatives), _stream(stream)), "fusedmm_minibatch_create")
    return h


def fusedmm_minibatch_reserve(mb, d: int) -> None:
    _check(load().fusedmm_minibatch_reserve(mb, d), "fusedmm_minibatch_reserve")


def fusedmm_minibatch_epoch(mb, d: int, lr: float, d_X, ldx: int, stream=None) -> None:
    _check(load().fusedmm_minibatch_epoch(mb, d, ctypes.c_float(lr), _dptr(d_X), ldx, _stream(stream)),
           "fusedmm_minibatch_epoch")


def fusedmm_minibatch_info(mb):
    nb, launches = ctypes.c_int32(), ctypes.c_int64()
    _check(load().fusedmm_minibatch_info(mb, ctypes.byref(nb), ctypes.byref(launches)), "fusedmm_minibatch_info")
    return {"n_batches": nb.value, "launches_per_epoch": launches.value}


def fusedmm_minibatch_destroy(mb) -> None:
    _check(load().fusedmm_minibatch_destroy(mb), "fusedmm_minibatch_destroy")


# ---- convenience wrapper (still marshalling only) ----------------------------

def _check_csr(rowptr, colidx) -> None:
    if not (rowptr.is_cuda and str(rowptr.dtype) == "torch.int64" and rowptr.is_contiguous()):
        raise TypeError("rowptr must be a contiguous CUDA int64 tensor")
    if colidx.numel() and not (colidx.is_cuda and str(colidx.dtype) == "torch.int32" and colidx.is_contiguous()):
        raise TypeError("colidx must be a contiguous CUDA int32 tensor")


class Plan:
    """Owns a fusedmm_plan_t for one CSR pattern held in torch device tensors."""

    @classmethod
    def tuned(cls, m: int, n: int, rowptr, colidx, ops, X, Y, Z, values=None, stream=None):
        """Plan chosen by timing candidate schedules with these operands (fusedmm_plan_create_tuned)."""
        if isinstance(ops, str):
            ops = fusedmm_ops_preset(ops)
        _check_csr(rowptr, colidx)
        self = cls.__new__(cls)
        self.m, self.n, self.nnz = int(m), int(n), int(colidx.numel())
        self.rowptr, self.colidx = rowptr, colidx
        ldx = 0 if X is None else X.stride(0)
        self._plan, self.tuned_options, self.tuned_ms = fusedmm_plan_create_tuned(
            self.m, self.n, self.nnz, rowptr, colidx if self.nnz else None, ops, int(Z.shape[1]), values, X, ldx,
            Y, Y.stride(0), Z, Z.stride(0), stream)
        return self

    def __init__(self, m: int, n: int, rowptr, colidx, options: Optional[dict] = None, stream=None):
        _check_csr(rowptr, colidx)
        self.m, self.n, self.nnz = int(m), int(n), int(colidx.numel())
        self.rowptr, self.colidx = rowptr, colidx  # keep alive: the plan borrows them
        self._plan = fusedmm_plan_create(self.m, self.n, self.nnz, rowptr, colidx if self.nnz else None, options,
                                         stream)

    def execute(self, ops, X, Y, Z, values=None, stream=None) -> None:
        if isinstance(ops, str):
            ops = fusedmm_ops_preset(ops)
        d = int(Z.shape[1]) if Z is not None and Z.dim() == 2 else 0
        for t in (X, Y, Z, values):
            if t is not None and not (t.is_cuda and str(t.dtype) == "torch.float32" and (t.dim() < 2 or t.stride(-1) == 1)):
                raise TypeError("operands must be CUDA float32 tensors with unit stride along the feature dimension")
        ldx = 0 if X is None else X.stride(0)
        fusedmm_execute(self._plan, ops, d, values, X, ldx, Y, Y.stride(0), Z, Z.stride(0), stream)

    def bind(self, ops, X, Y, Z, values=None, stream=None, y_format: str = "f32"):
        """The same call as execute / execute_bf16y / execute_f16y / execute_f64 with the arguments marshalled once: returns
        a function of no arguments that issues it (for loops that repeat one call: per-call cost is the C
        call alone).  The stream is the one given, or the current stream at the time of binding; the tensors
        are kept alive by the returned function."""
        if isinstance(ops, str):
            ops = fusedmm_ops_preset(ops)
        if y_format not in ("f32", "bf16", "f16", "f64"):
            raise ValueError("y_format must be 'f32', 'bf16', 'f16' or 'f64' (everything in double precision)")
        want = "torch.float64" if y_format == "f64" else "torch.float32"
        for t in (X, Z, values) + ((Y,) if y_format in ("f32", "f64") else ()):
            if t is not None and not (t.is_cuda and str(t.dtype) == want and (t.dim() < 2 or t.stride(-1) == 1)):
                raise TypeError(f"operands must be CUDA {want[6:]} tensors with unit stride along the feature dimension")
        if y_format in ("bf16", "f16") and not (Y.is_cuda and Y.element_size() == 2 and Y.stride(-1) == 1):
            raise TypeError("Y must be a CUDA tensor of 2-byte elements with unit stride along the feature dimension")
        lib = load()
        fn = {"f32": lib.fusedmm_execute, "bf16": lib.fusedmm_execute_bf16y, "f16": lib.fusedmm_execute_f16y,
              "f64": lib.fusedmm_execute_f64}[y_format]
        args = (self._plan, ctypes.byref(ops), int(Z.shape[1]), _dptr(values), _dptr(X), 0 if X is None else X.stride(0),
                _dptr(Y), Y.stride(0), _dptr(Z), Z.stride(0), _stream(stream))
        keep = (ops, X, Y, Z, values, self)

        def call(fn=fn, args=args, keep=keep) -> None:
            st = fn(*args)
            if st != FUSEDMM_OK:
                raise FusedMMError(st, "fusedmm_execute (bound call)")

        return call

    def execute_bf16y(self, ops, X, Y_bf16, Z, values=None, stream=None) -> None:
        """Y_bf16: CUDA tensor of 2-byte elements (torch.bfloat16, int16 or uint16 bits), n x d."""
        if isinstance(ops, str):
            ops = fusedmm_ops_preset(ops)
        if not (Y_bf16.is_cuda and Y_bf16.element_size() == 2 and Y_bf16.stride(-1) == 1):
            raise TypeError("Y_bf16 must be a CUDA tensor of 2-byte elements with unit stride along the feature dimension")
        ldx = 0 if X is None else X.stride(0)
        fusedmm_execute_bf16y(self._plan, ops, int(Z.shape[1]), values, X, ldx, Y_bf16, Y_bf16.stride(0), Z, Z.stride(0),
                              stream)

    def execute_f64(self, ops, X, Y, Z, values=None, stream=None) -> None:
        if isinstance(ops, str):
            ops = fusedmm_ops_preset(ops)
        for t in (X, Y, Z, values):
            if t is not None and not (t.is_cuda and str(t.dtype) == "torch.float64" and (t.dim() < 2 or t.stride(-1) == 1)):
                raise TypeError("operands must be CUDA float64 tensors with unit stride along the feature dimension")
        ldx = 0 if X is None else X.stride(0)
        fusedmm_execute_f64(self._plan, ops, int(Z.shape[1]), values, X, ldx, Y, Y.stride(0), Z, Z.stride(0), stream)

    def execute_f16y(self, ops, X, Y_f16, Z, values=None, stream=None) -> None:
        """Y_f16: CUDA tensor of 2-byte elements (torch.float16, int16 or uint16 bits), n x d."""
        if isinstance(ops, str):
            ops = fusedmm_ops_preset(ops)
        if not (Y_f16.is_cuda and Y_f16.element_size() == 2 and Y_f16.stride(-1) == 1):
            raise TypeError("Y_f16 must be a CUDA tensor of 2-byte elements with unit stride along the feature dimension")
        ldx = 0 if X is None else X.stride(0)
        fusedmm_execute_f16y(self._plan, ops, int(Z.shape[1]), values, X, ldx, Y_f16, Y_f16.stride(0), Z, Z.stride(0),
                             stream)

    def edge_visits(self, d: int, fast_path, counts, stream=None) -> None:
        fusedmm_debug_edge_visits(self._plan, d, fast_path, counts, stream)

    def reserve(self, d: int) -> None:
        fusedmm_plan_reserve(self._plan, d)

    def reserve_f64(self, d: int) -> None:
        fusedmm_plan_reserve_f64(self._plan, d)

    def workspace_bytes(self, d: int) -> int:
        return fusedmm_plan_workspace_bytes(self._plan, d)

    def stats(self) -> dict:
        return fusedmm_plan_stats(self._plan)

    def set_profiling(self, enabled: bool) -> None:
        fusedmm_plan_set_profiling(self._plan, enabled)

    def read_profile(self):
        return fusedmm_plan_read_profile(self._plan)

    def read_profile_samples(self):
        return fusedmm_plan_read_profile_samples(self._plan)

    def close(self) -> None:
        if self._plan is not None:
            fusedmm_plan_destroy(self._plan)
            self._plan = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Minibatch:
    """Owns a fusedmm_minibatch_t: the per-batch plans of one graph for embedding epochs."""

    def __init__(self, n: int, rowptr, colidx, batch_rows: int, negatives=None, stream=None):
        _check_csr(rowptr, colidx)
        self.n, self.nnz = int(n), int(colidx.numel())
        self.rowptr, self.colidx = rowptr, colidx  # keep alive: the plans borrow them
        n_negative = 0
        if negatives is not None:
            if not (negatives.is_cuda and str(negatives.dtype) == "torch.int32" and negatives.is_contiguous()
                    and negatives.dim() == 2):
                raise TypeError("negatives must be a contiguous CUDA int32 tensor of shape (n_batches, n_negative)")
            if negatives.shape[0] != (self.n + batch_rows - 1) // batch_rows:
                raise ValueError("negatives needs one row per batch")
            n_negative = int(negatives.shape[1])
        self._mb = fusedmm_minibatch_create(self.n, self.nnz, rowptr, colidx if self.nnz else None, int(batch_rows),
                                            n_negative, negatives if n_negative else None, stream)

    def reserve(self, d: int) -> None:
        fusedmm_minibatch_reserve(self._mb, d)

    def epoch(self, X, lr: float, stream=None) -> None:
        if not (X.is_cuda and str(X.dtype) == "torch.float32" and X.dim() == 2 and X.stride(1) == 1
                and X.shape[0] == self.n):
            raise TypeError("X must be a CUDA float32 tensor of n rows with unit stride along the feature dimension")
        fusedmm_minibatch_epoch(self._mb, int(X.shape[1]), float(lr), X, X.stride(0), stream)

    def info(self) -> dict:
        return fusedmm_minibatch_info(self._mb)

    def close(self) -> None:
        if self._mb is not None:
            fusedmm_minibatch_destroy(self._mb)
            self._mb = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
