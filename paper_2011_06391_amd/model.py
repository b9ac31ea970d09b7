"""Byte / flop model of FusedMM (host arithmetic only; used by bench.py).

Two models live here:

* the paper's own arithmetic-intensity bound (Section IV-C, Eq. 4), which
  assumes 8-byte indices: 12 B per stored entry, X and Z moved once, one row of
  Y moved per stored entry;
* the model of this library's data layout (int32 column indices, int64 row
  pointers, fp32 values), which is what the roofline fraction is priced on.
"""
from __future__ import annotations

from dataclasses import dataclass


def paper_arithmetic_intensity(avg_degree: float, d: int) -> float:
    """Eq. 4: AI = 4 d m delta / (12 m delta + 8 m d + 4 d m delta) flop/byte
    = 1 / (3/d + 2/delta + 1)."""
    delta = float(avg_degree)
    return (4.0 * d * delta) / (12.0 * delta + 8.0 * d + 4.0 * d * delta)


def paper_attainable_gflops(avg_degree: float, d: int, stream_gbs: float) -> float:
    """Roofline ceiling of Section V-B: AI x sustained memory bandwidth."""
    return paper_arithmetic_intensity(avg_degree, d) * stream_gbs


@dataclass(frozen=True)
class Traffic:
    """Bytes one execute call has to move, and the flops it performs."""
    per_edge_bytes: int
    per_row_bytes: int
    model_bytes: int      # no reuse of Y rows assumed (one row per stored entry)
    min_bytes: int        # every array touched exactly once (infinite cache)
    flops: int


def traffic(m: int, n: int, nnz: int, d: int, uses_x: bool, uses_values: bool,
            x_is_y: bool, y_bytes: int = 0, elem_bytes: int = 4) -> Traffic:
    """Algorithmic traffic with fp32 data (elem_bytes = 8: fp64), int32 colidx, int64 rowptr.

    per stored entry : 4 (colidx) + 4d (row of Y; 2d when Y is stored as bfloat16) [+ 4 (edge value)]
    per row          : 8 (rowptr) + 4d (store z_u) [+ 4d (load x_u)]
    """
    e = elem_bytes
    y_bytes = y_bytes or e
    per_edge = 4 + y_bytes * d + (e if uses_values else 0)
    per_row = 8 + e * d + (e * d if uses_x else 0)
    model = nnz * per_edge + m * per_row
    mn = nnz * (4 + (e if uses_values else 0)) + 8 * m + y_bytes * n * d + e * m * d
    if uses_x and (not x_is_y or y_bytes != e):
        mn += e * m * d
    flops = nnz * (4 * d if uses_x else 2 * d)
    return Traffic(per_edge, per_row, model, mn, flops)


MI355X_HBM_PEAK_GBS = 8000.0
