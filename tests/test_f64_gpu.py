"""Double precision entry point (fusedmm_execute_f64) against the fp64 oracle.

The oracle reads fp32 inputs and computes in double; here the GPU is handed the same values
widened to double, so both sides do fp64 arithmetic on identical numbers and may differ only by
the order of the sums: bound 1e-12 * sum|terms| per element (fp32 arithmetic anywhere in the kernel
would miss it by five orders of magnitude).  A second test feeds genuinely 64-bit inputs and
compares with a dense numpy product, so that the low mantissa bits are known to be read."""
import numpy as np
import pytest

import oracle
from helpers import random_csr
from paper_2011_06391_amd import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL64 = 1e-12


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    from paper_2011_06391_amd import binding
    binding.load()
    return binding


def dev(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()


CASES = [
    ("sigmoid", "SUM", oracle.PATTERNS["sigmoid"], "ASUM"),
    ("one_minus_sigmoid", "SUM", oracle.PATTERNS["one_minus_sigmoid"], "ASUM"),
    ("gcn", "SUM", oracle.PATTERNS["gcn"], "ASUM"),
    ("tdist", "SUM", oracle.PATTERNS["tdist"], "ASUM"),
    ("fr", "SUM", oracle.PATTERNS["fr"], "ASUM"),
    (("SUB", "NOOP", "SIGMOID", "MUL_T"), "MAX", ("SUB", "NOOP", "SIGMOID", "MUL_T"), "AMAX"),
    (("MUL", "RSUM", "SIGMOID", "MUL_Y"), "MEAN", ("MUL", "RSUM", "SIGMOID", "MUL_Y"), "AMEAN"),
    (("ADD", "NORM2", "SCAL", "SEL2ND"), "MIN", ("ADD", "NORM", "SCAL", "SEL2ND"), "AMIN"),
]


# every lane-group width and register count of the general kernel, and whatever instance takes d by default
@pytest.mark.parametrize("d", (2, 3, 5, 13, 27, 64, 128, 200, 301, 700))
@pytest.mark.parametrize("case", CASES, ids=[str(c[0]) + "-" + c[1] for c in CASES])
def test_f64_matches_oracle(B, case, d):
    gpu_ops, gpu_aop, oracle_ops, oracle_aop = case
    g = synth.rmat(10, (1 << 9) * 24, seed=300 + d)        # skewed: rows of 0 .. several hundred entries
    m = n = g.m
    rng = np.random.default_rng(17 + d)
    X = rng.uniform(-0.7, 0.7, (m, d)).astype(np.float32)
    Y = rng.uniform(-0.7, 0.7, (n, d)).astype(np.float32)
    vals = rng.uniform(-1, 1, g.nnz).astype(np.float32)
    alpha = float(np.float32(0.41))   # alpha travels as fp32 in the op struct: the oracle gets the same value
    Zr_alpha, S, _ = oracle.unfused_general(g.rowptr, g.colidx, vals, X, Y, oracle_ops, oracle_aop, alpha=alpha)
    if isinstance(gpu_ops, str):
        ops = B.fusedmm_ops_preset(gpu_ops)
    else:
        ops = B.make_ops(*gpu_ops, aop=gpu_aop)
    ops.alpha = alpha
    uses_x = ops.vop != B.VOP["SEL2ND"]
    for options in (None, {"general_kernel_only": 1}):   # the kernel that takes d by default; the general kernel
        plan = B.Plan(m, n, dev(g.rowptr), dev(g.colidx), options)
        plan.reserve_f64(d)
        Z = torch.full((m, d), float("nan"), dtype=torch.float64, device="cuda")
        plan.execute_f64(ops, dev(X.astype(np.float64)) if uses_x else None, dev(Y.astype(np.float64)), Z,
                         dev(vals.astype(np.float64)))
        torch.cuda.synchronize()
        Zg = Z.cpu().numpy()
        scale = np.where(S > 0, S, 1.0)
        err = np.abs(Zg - Zr_alpha) / scale
        assert (Zg[S == 0] == 0).all()
        assert err.max() <= TOL64, f"{case[0]} {gpu_aop} d={d} {options}: {err.max():.3e}"
        plan.close()


# the specialised schedule's double-precision instances: instance sizes and dimensions between them, on a plan
# whose options put rows into every bin (packed, wave, chunks, column-class tiles with partial rows)
@pytest.mark.parametrize("d", (32, 64, 128, 256, 512, 20, 100, 200, 300, 13, 30, 97, 301, 1, 2, 6, 8, 16, 700, 1024, 1500, 2048))
@pytest.mark.parametrize("case", CASES, ids=[str(c[0]) + "-" + c[1] for c in CASES])
def test_f64_specialised_schedule_all_bins(B, case, d):
    gpu_ops, gpu_aop, oracle_ops, oracle_aop = case
    rng = np.random.default_rng(4000 + d)
    m, n = 300, 500
    degs = rng.integers(0, 9, m)
    degs[[0, 7, 299]] = 0
    degs[5], degs[20], degs[33], degs[47], degs[290] = 40, 70, 300, 450, 130
    rowptr = np.zeros(m + 1, dtype=np.int64)
    rowptr[1:] = np.cumsum(degs)
    colidx = np.concatenate([np.sort(rng.choice(n, k, replace=False)) for k in degs]).astype(np.int32)
    X = rng.uniform(-0.7, 0.7, (m, d)).astype(np.float32)
    Y = rng.uniform(-0.7, 0.7, (n, d)).astype(np.float32)
    vals = rng.uniform(-1, 1, len(colidx)).astype(np.float32)
    alpha = float(np.float32(0.41))
    Zr, S, _ = oracle.unfused_general(rowptr, colidx, vals, X, Y, oracle_ops, oracle_aop, alpha=alpha)
    ops = B.fusedmm_ops_preset(gpu_ops) if isinstance(gpu_ops, str) else B.make_ops(*gpu_ops, aop=gpu_aop)
    ops.alpha = alpha
    plan = B.Plan(m, n, dev(rowptr), dev(colidx), {"small_row_max": 4, "split_row_min": 32, "chunk_edges": 256,
                                                   "column_classes": 8, "tile_row_min": 64, "feature_dim_hint": d})
    st = plan.stats()
    assert st["tiled_rows"] > 0 and st["wave_rows"] > 0 and st["packed_rows"] > 0 and st["partials"] > 0
    uses_x = ops.vop != B.VOP["SEL2ND"]
    Z = torch.full((m, d), float("nan"), dtype=torch.float64, device="cuda")
    args = (ops, dev(X.astype(np.float64)) if uses_x else None, dev(Y.astype(np.float64)), Z, dev(vals.astype(np.float64)))
    # the plan has reserved partial rows of d floats: rows of d doubles are refused until they are reserved
    with pytest.raises(B.FusedMMError) as ei:
        plan.execute_f64(*args)
    assert ei.value.status == B.FUSEDMM_ERR_NOT_RESERVED
    torch.cuda.synchronize()
    assert torch.isnan(Z).all()
    plan.reserve_f64(d)
    plan.execute_f64(*args)
    torch.cuda.synchronize()
    Zg = Z.cpu().numpy()
    err = np.abs(Zg - Zr) / np.where(S > 0, S, 1.0)
    assert (Zg[S == 0] == 0).all()
    assert err.max() <= TOL64, f"{case[0]} {gpu_aop} d={d}: {err.max():.3e}"
    # every stored entry exactly once under the double-precision instances' lane groups
    counts = torch.zeros(len(colidx), dtype=torch.int32, device="cuda")
    plan.edge_visits(d, 2, counts)
    torch.cuda.synchronize()
    assert (counts == 1).all()
    plan.close()


def test_f64_specialised_schedule_is_the_one_that_runs(B):
    """fusedmm_execute_f64 at d = 128 must be several times faster than the general kernel at the same d (a plan
    that asks for it) -- a silent fall-back of the instance sizes to the general kernel would show here.
    Rows that start at an odd element run the same instances (the kernels read element-aligned vectors)."""
    g = synth.rmat(14, (1 << 14) * 32, seed=77)
    m = n = g.m
    rng = np.random.default_rng(3)
    rp, ci = dev(g.rowptr), dev(g.colidx)
    plan_fast = B.Plan(m, n, rp, ci)
    plan_general = B.Plan(m, n, rp, ci, {"general_kernel_only": 1})
    for p in (plan_fast, plan_general):
        p.reserve_f64(128)
    ops = B.fusedmm_ops_preset("sigmoid")

    def timed(plan, d, off):
        Xw = torch.from_numpy(rng.uniform(-0.5, 0.5, (m, d + 4))).cuda()
        Zw = torch.empty((m, d + 4), dtype=torch.float64, device="cuda")
        X, Z = Xw[:, off:off + d], Zw[:, off:off + d]
        for _ in range(3):
            plan.execute_f64(ops, X, X, Z)
        torch.cuda.synchronize()
        t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0.record()
        for _ in range(10):
            plan.execute_f64(ops, X, X, Z)
        t1.record()
        torch.cuda.synchronize()
        return t0.elapsed_time(t1) / 10 / d

    t_fast, t_odd, t_gen = timed(plan_fast, 128, 0), timed(plan_fast, 128, 1), timed(plan_general, 128, 0)
    assert t_fast * 2 < t_gen and t_odd * 2 < t_gen, (t_fast, t_odd, t_gen)
    plan_fast.close()
    plan_general.close()


def test_f64_reads_all_64_bits(B):
    """Inputs that differ from their fp32 roundings only in the low mantissa bits: the product with a
    0/1 pattern (GCN, unit values) must match numpy's fp64 product, not the product of the roundings."""
    rng = np.random.default_rng(5)
    m, n, d = 37, 53, 24
    rowptr, colidx = random_csr(rng, m, n, 0.3, empty_rows=(4,))
    Y = rng.uniform(1.0, 2.0, (n, d))                      # full 53-bit mantissas
    assert np.abs(Y - Y.astype(np.float32)).max() > 1e-9
    A = np.zeros((m, n))
    for u in range(m):
        A[u, colidx[rowptr[u]:rowptr[u + 1]]] = 1.0
    ref = A @ Y
    plan = B.Plan(m, n, dev(rowptr), dev(colidx))
    Z = torch.full((m, d), float("nan"), dtype=torch.float64, device="cuda")
    ones = torch.ones(len(colidx), dtype=torch.float64, device="cuda")
    plan.execute_f64("gcn", None, dev(Y), Z, ones)
    torch.cuda.synchronize()
    Zg = Z.cpu().numpy()
    assert np.abs(Zg - ref).max() <= 1e-13 * np.abs(ref).max()
    assert np.abs(A @ Y.astype(np.float32).astype(np.float64) - ref).max() > 1e-8   # the roundings would not pass
    assert (Zg[4] == 0).all()
    plan.close()


def test_f64_strides_and_errors(B):
    rng = np.random.default_rng(6)
    m, n, d = 30, 40, 16
    rowptr, colidx = random_csr(rng, m, n, 0.25)
    X = rng.uniform(-0.5, 0.5, (m, d + 3)).astype(np.float32)
    Y = rng.uniform(-0.5, 0.5, (n, d + 5)).astype(np.float32)
    Zr, S, _ = oracle.unfused(rowptr, colidx, None, X[:, :d], Y[:, :d], "tdist")
    plan = B.Plan(m, n, dev(rowptr), dev(colidx))
    Xd, Yd = dev(X.astype(np.float64)), dev(Y.astype(np.float64))
    Zb = torch.full((m, d + 2), 3.0, dtype=torch.float64, device="cuda")
    plan.execute_f64("tdist", Xd[:, :d], Yd[:, :d], Zb[:, :d])
    torch.cuda.synchronize()
    out = Zb.cpu().numpy()
    assert (np.abs(out[:, :d] - Zr) <= TOL64 * np.where(S > 0, S, 1.0)).all() and (out[:, d:] == 3.0).all()
    ops = B.fusedmm_ops_preset("tdist")
    with pytest.raises(B.FusedMMError) as ei:   # Z overlapping Y
        B.fusedmm_execute_f64(plan._plan, ops, d, None, Xd, d + 3, Yd, d + 5, Yd, d + 5)
    assert ei.value.status == B.FUSEDMM_ERR_ALIAS
    with pytest.raises(B.FusedMMError) as ei:   # leading dimension below d
        B.fusedmm_execute_f64(plan._plan, ops, d, None, Xd, d - 1, Yd, d + 5, Zb, d + 2)
    assert ei.value.status == B.FUSEDMM_ERR_INVALID_ARG
    with pytest.raises(TypeError):              # fp32 tensors are refused by the wrapper
        plan.execute_f64("tdist", dev(X), dev(Y), Zb[:, :d])
    plan.close()
