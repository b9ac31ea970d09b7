"""Host logic: the Eq. 4 model against the numbers the paper prints, and the
seeded generators (structure, determinism, statistics)."""
import os

import numpy as np
import pytest

from paper_2011_06391_amd import model, synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "roofline_orkut.txt")


def _golden():
    out = {}
    for line in open(GOLDEN):
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            out[k] = float(v)
    return out


def test_eq4_matches_printed_roofline_numbers():
    g = _golden()
    ai = model.paper_arithmetic_intensity(g["avg_degree"], int(g["d"]))
    assert round(ai, 2) == g["arithmetic_intensity"]
    assert abs(model.paper_attainable_gflops(g["avg_degree"], int(g["d"]), g["stream_gbs"]) - g["attainable_gflops"]) < 0.005
    # Section IV-C: worst AI 1/6 at delta = 1, d = 1; AI -> 1 for dense graphs and large d
    assert abs(model.paper_arithmetic_intensity(1, 1) - g["worst_case_ai_delta1_d1"]) < 1e-9
    assert 0.99 < model.paper_arithmetic_intensity(1e6, 4096) < 1.0
    # rearranged form (3/d + 2/delta + 1)^-1
    assert abs(ai - 1.0 / (3 / 128 + 2 / 76.28 + 1)) < 1e-12


def test_traffic_model():
    t = model.traffic(m=10, n=20, nnz=100, d=128, uses_x=True, uses_values=False, x_is_y=False)
    assert t.per_edge_bytes == 4 + 512 and t.per_row_bytes == 8 + 1024
    assert t.model_bytes == 100 * 516 + 10 * 1032
    assert t.min_bytes == 400 + 80 + 4 * 20 * 128 + 2 * 4 * 10 * 128
    assert t.flops == 100 * 4 * 128
    g = model.traffic(m=10, n=10, nnz=100, d=128, uses_x=False, uses_values=True, x_is_y=True)
    assert g.per_edge_bytes == 8 + 512 and g.per_row_bytes == 8 + 512 and g.flops == 100 * 2 * 128


def _check_simple_symmetric(g):
    deg = g.degrees()
    assert g.rowptr[0] == 0 and g.rowptr[-1] == len(g.colidx)
    rows = np.repeat(np.arange(g.m, dtype=np.int64), deg)
    assert (rows != g.colidx).all(), "self loop"
    keys = rows * g.n + g.colidx
    assert (np.diff(keys) > 0).all(), "columns sorted within rows, no duplicates"
    rev = np.sort(g.colidx.astype(np.int64) * g.n + rows)
    assert np.array_equal(rev, keys), "pattern symmetric"
    assert g.colidx.min() >= 0 and g.colidx.max() < g.n


def test_erdos_renyi_c1_shape():
    w = synth.make_workload("c1")
    g = w.csr
    assert g.m == 4096 and g.nnz == 32768 and w.d == 64 and w.X is w.Y
    _check_simple_symmetric(g)
    assert w.X.dtype == np.float32 and w.X.min() >= -0.5 and w.X.max() < 0.5
    assert abs(float(w.X.mean())) < 0.01 and abs(float(w.X.std()) - 1 / np.sqrt(12)) < 0.01
    deg = g.degrees()
    assert 15 <= deg.max() <= 30 and abs(deg.mean() - 8.0) < 1e-9


def test_rmat_structure_and_skew():
    g = synth.rmat(12, (1 << 11) * 16, seed=77)
    _check_simple_symmetric(g)
    deg = g.degrees()
    assert g.m == 4096 and g.nnz <= 2 * (1 << 11) * 16
    assert deg.max() > 20 * deg.mean()      # heavy tail
    assert (deg == 0).sum() > 0.1 * g.m     # R-MAT leaves many isolated vertices
    # relabelling hides the hub ids: the largest-degree vertices are not the smallest ids
    assert np.argsort(-deg)[:8].min() > 8 or np.argsort(-deg)[:8].max() > 64
    g2 = synth.rmat(12, (1 << 11) * 16, seed=77, relabel=False)
    assert np.array_equal(np.sort(deg), np.sort(g2.degrees()))  # same graph up to labels
    assert np.argmax(g2.degrees()) == 0                         # as generated, vertex 0 is the hub


def test_generators_are_deterministic():
    a = synth.rmat(10, 4096, seed=5)
    b = synth.rmat(10, 4096, seed=5)
    c = synth.rmat(10, 4096, seed=6)
    assert np.array_equal(a.rowptr, b.rowptr) and np.array_equal(a.colidx, b.colidx)
    assert not (len(a.colidx) == len(c.colidx) and np.array_equal(a.colidx, c.colidx))
    assert np.array_equal(synth.fill_uniform((7, 5), 9, -1, 1), synth.fill_uniform((7, 5), 9, -1, 1))
    assert np.array_equal(synth.fill_normal((7, 5), 9), synth.fill_normal((7, 5), 9))


def test_chung_lu_degrees_and_norm_values():
    n = 5000
    g = synth.chung_lu(n, 200_000, 50.0, seed=3, relabel=False)
    _check_simple_symmetric(g)
    deg = g.degrees()
    # expected degree falls with the vertex id as (i + i0)^(-1/2): the first 1% of ids carry far more than the last 1%
    assert deg[:50].mean() > 3 * deg[-50:].mean()
    vals = synth.sym_norm_values(g)
    u, e = 123, int(g.rowptr[123])
    v = int(g.colidx[e])
    assert vals[e] == np.float32(1.0 / np.sqrt(float(deg[u]) * float(deg[v])))
    assert np.isfinite(vals).all() and (vals > 0).all()


def test_fills():
    x = synth.fill_normal((200000,), 11)
    assert abs(float(x.mean())) < 0.01 and abs(float(x.std()) - 1.0) < 0.01
    k = synth.fill_int((1000, 8), 4, -8, 8)
    assert k.min() == -8 and k.max() == 8 and (k == np.round(k)).all()
    p = synth.permutation(1000, 1)
    assert np.array_equal(np.sort(p), np.arange(1000))


def test_take_rows_slice():
    g = synth.rmat(8, 1024, seed=2)
    rows = np.array([5, 0, 200, 5])
    s = g.take_rows(rows)
    assert s.m == 4 and s.n == g.n
    for i, r in enumerate(rows):
        assert np.array_equal(s.colidx[s.rowptr[i]:s.rowptr[i + 1]], g.colidx[g.rowptr[r]:g.rowptr[r + 1]])


def test_epoch_workloads():
    """Stand-ins for the two citation graphs of the end-to-end experiment: sizes, symmetry, determinism."""
    import scipy.sparse as sp
    for name, n, pairs in (("e1", 2708, 5278), ("e2", 19717, 44324)):
        w = synth.make_epoch_workload(name)
        g = w.csr
        assert (g.m, g.n, w.d, w.batch_rows) == (n, n, 128, 256)
        assert 1.8 * pairs < g.nnz <= 2 * pairs and 60 <= g.degrees().max() <= 400
        A = sp.csr_matrix((np.ones(g.nnz), g.colidx, g.rowptr), shape=(n, n))
        assert A.max() == 1 and (A != A.T).nnz == 0 and A.diagonal().sum() == 0
        assert w.negatives.shape == ((n + 255) // 256, 5) and w.negatives.dtype == np.int32
        assert w.negatives.min() >= 0 and w.negatives.max() < n
        w2 = synth.make_epoch_workload(name)
        assert np.array_equal(w.negatives, w2.negatives) and np.array_equal(w.X0, w2.X0)
        assert np.array_equal(g.colidx, w2.csr.colidx)


def test_density_sweep_workload_spec():
    """rmat:SCALE:PAIRS builds an R-MAT graph of that size (deterministic, symmetric); bad specs are rejected."""
    a = synth.make_workload("rmat:10:4096", d=8)
    b = synth.make_workload("rmat:10:4096", d=8)
    assert a.csr.m == 1024 and a.d == 8 and a.pattern == "one_minus_sigmoid"
    assert np.array_equal(a.csr.colidx, b.csr.colidx) and np.array_equal(a.X, b.X)
    dense = np.zeros((1024, 1024), dtype=bool)
    rows = np.repeat(np.arange(1024), np.diff(a.csr.rowptr))
    dense[rows, a.csr.colidx] = True
    assert (dense == dense.T).all() and not dense.diagonal().any()
    assert synth.make_workload("rmat:10:8192", d=8).csr.nnz > a.csr.nnz
    for bad in ("rmat:10", "rmat:x:5", "rmat:40:5", "rmat:10:0"):
        with pytest.raises(ValueError):
            synth.make_workload(bad)
