"""Small numpy-only helpers shared by the test modules (no method arithmetic)."""
import numpy as np


def random_csr(rng: np.random.Generator, m: int, n: int, density: float, empty_rows=(), duplicates: bool = False,
               sort_cols: bool = True):
    """Small random m x n CSR pattern built with numpy only (independent of the C generators)."""
    rows = []
    for u in range(m):
        if u in empty_rows:
            rows.append(np.zeros(0, dtype=np.int32))
            continue
        cols = np.nonzero(rng.random(n) < density)[0].astype(np.int32)
        if duplicates and len(cols) > 0:
            cols = np.concatenate([cols, cols[: max(1, len(cols) // 3)]])
        if sort_cols:
            cols = np.sort(cols)
        else:
            rng.shuffle(cols)
        rows.append(cols)
    rowptr = np.zeros(m + 1, dtype=np.int64)
    rowptr[1:] = np.cumsum([len(r) for r in rows])
    colidx = np.concatenate(rows).astype(np.int32) if rowptr[-1] > 0 else np.zeros(0, dtype=np.int32)
    return rowptr, colidx
