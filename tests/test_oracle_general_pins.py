"""Pins for the oracle's general five-step path (the standard operations of Table II that lie
outside the application patterns: ADD, RMUL, SOP no-op, vector-valued messages, SEL2ND as MOP,
AMAX / AMIN).  References are dense numpy formulas written from the definitions."""
import numpy as np
import pytest

import oracle
from helpers import random_csr


def dense_mask(rowptr, colidx, m, n):
    A = np.zeros((m, n), dtype=bool)
    for u in range(m):
        A[u, colidx[rowptr[u]:rowptr[u + 1]]] = True
    return A


def sigmoid(x):
    return 1.0 / (1.0 + np.exp(-x))


@pytest.fixture
def problem(rng):
    m, n, d = 19, 31, 6
    rowptr, colidx = random_csr(rng, m, n, 0.25, empty_rows=(0, 11))
    X = rng.uniform(-1, 1, (m, d)).astype(np.float32)
    Y = rng.uniform(-1, 1, (n, d)).astype(np.float32)
    vals = rng.uniform(-1, 1, len(colidx)).astype(np.float32)
    return m, n, d, rowptr, colidx, X, Y, vals


def test_general_path_reproduces_the_scalar_patterns(problem):
    m, n, d, rowptr, colidx, X, Y, vals = problem
    for name, ops in oracle.PATTERNS.items():
        Z0, S0, H0 = oracle.unfused(rowptr, colidx, vals, X, Y, name, alpha=0.3)
        Z1, S1, H1 = oracle.unfused_general(rowptr, colidx, vals, X, Y, ops, "ASUM", alpha=0.3)
        np.testing.assert_array_equal(Z0, Z1)
        np.testing.assert_array_equal(S0, S1)
        np.testing.assert_array_equal(H0, H1)


def test_amax_amin_of_weighted_neighbours(problem):
    """SEL2ND, NOOP, EDGE_VALUE, MUL, AMAX: z_u[k] = max(0, max_v a_uv y_v[k]) -- the accumulator
    starts at zero (Algorithm 1), so a row without entries gives 0 and negative maxima clip to 0."""
    m, n, d, rowptr, colidx, X, Y, vals = problem
    A = dense_mask(rowptr, colidx, m, n)
    V = np.zeros((m, n))
    rows = np.repeat(np.arange(m), np.diff(rowptr))
    V[rows, colidx] = vals
    W = V[:, :, None] * Y.astype(np.float64)[None, :, :]          # m x n x d candidate messages
    Wmax = np.where(A[:, :, None], W, -np.inf).max(axis=1)
    Wmin = np.where(A[:, :, None], W, np.inf).min(axis=1)
    ops = ("SEL2ND", "NOOP", "EDGE_VALUE", "MUL_Y")
    Zmax, Smax, _ = oracle.unfused_general(rowptr, colidx, vals, None, Y, ops, "AMAX")
    Zmin, Smin, _ = oracle.unfused_general(rowptr, colidx, vals, None, Y, ops, "AMIN")
    np.testing.assert_allclose(Zmax, np.maximum(0.0, Wmax), rtol=0, atol=0)
    np.testing.assert_allclose(Zmin, np.minimum(0.0, Wmin), rtol=0, atol=0)
    assert (Zmax[[0, 11]] == 0).all() and (Zmin[[0, 11]] == 0).all()
    assert (Zmax > 0).any() and (Zmax == 0).any()  # both branches of the clip occur
    np.testing.assert_allclose(Smax, np.where(A[:, :, None], np.abs(W), 0).max(axis=1))
    # mirror image: AMIN(w) = -AMAX(-w)
    Zneg, _, _ = oracle.unfused_general(rowptr, colidx, -vals, None, Y, ops, "AMAX")
    np.testing.assert_array_equal(Zmin, -Zneg)


def test_vector_messages_elementwise_sigmoid(problem):
    """MUL, NOOP, SIGMOID, MUL, ASUM: no reduction, so h = sigma(x_u (.) y_v) is a vector and
    z_u = sum_v h (.) y_v.  Also with AMAX (the shape of the GNN row of Table III)."""
    m, n, d, rowptr, colidx, X, Y, vals = problem
    A = dense_mask(rowptr, colidx, m, n)
    Xd, Yd = X.astype(np.float64), Y.astype(np.float64)
    Hd = sigmoid(Xd[:, None, :] * Yd[None, :, :])                  # m x n x d
    Wd = Hd * Yd[None, :, :]
    ops = ("MUL", "NOOP", "SIGMOID", "MUL_Y")
    Z, S, H = oracle.unfused_general(rowptr, colidx, None, X, Y, ops, "ASUM")
    np.testing.assert_allclose(Z, np.where(A[:, :, None], Wd, 0).sum(axis=1), rtol=1e-13, atol=1e-14)
    assert H.shape == (len(colidx), d)
    rows = np.repeat(np.arange(m), np.diff(rowptr))
    np.testing.assert_allclose(H, Hd[rows, colidx], rtol=1e-14)
    Zm, _, _ = oracle.unfused_general(rowptr, colidx, None, X, Y, ops, "AMAX")
    np.testing.assert_allclose(Zm, np.maximum(0, np.where(A[:, :, None], Wd, -np.inf).max(axis=1)), rtol=1e-14)


def test_add_rmul_and_noop_sop(problem):
    """ADD as VOP, RMUL as ROP, SOP skipped: h = prod_k (x_u[k] + y_v[k]); MUL_T scales t = x_u + y_v."""
    m, n, d, rowptr, colidx, X, Y, vals = problem
    A = dense_mask(rowptr, colidx, m, n)
    Xd, Yd = X.astype(np.float64), Y.astype(np.float64)
    T = Xd[:, None, :] + Yd[None, :, :]
    Hs = T.prod(axis=2)
    Z, S, H = oracle.unfused_general(rowptr, colidx, None, X, Y, ("ADD", "RMUL", "NOOP", "MUL_T"), "ASUM")
    ref = np.where(A[:, :, None], Hs[:, :, None] * T, 0).sum(axis=1)
    np.testing.assert_allclose(Z, ref, rtol=1e-12, atol=1e-13)
    rows = np.repeat(np.arange(m), np.diff(rowptr))
    np.testing.assert_allclose(H, Hs[rows, colidx], rtol=1e-13)
    # SOP no-op on a vector message: h = t, so MUL_T gives t (.) t
    Z2, _, _ = oracle.unfused_general(rowptr, colidx, None, X, Y, ("SUB", "NOOP", "NOOP", "MUL_T"), "ASUM")
    D = Xd[:, None, :] - Yd[None, :, :]
    np.testing.assert_allclose(Z2, np.where(A[:, :, None], D * D, 0).sum(axis=1), rtol=1e-12, atol=1e-13)


def test_sel2nd_as_mop_counts_neighbours(problem):
    """MOP = SEL2ND forwards y_v whatever h is: ASUM gives A1 @ Y, AMAX the clipped feature-wise max."""
    m, n, d, rowptr, colidx, X, Y, vals = problem
    A = dense_mask(rowptr, colidx, m, n).astype(np.float64)
    Z, _, _ = oracle.unfused_general(rowptr, colidx, None, X, Y, ("MUL", "RSUM", "SIGMOID", "SEL2ND"), "ASUM")
    np.testing.assert_allclose(Z, A @ Y.astype(np.float64), rtol=1e-13, atol=1e-14)
    ones = np.ones_like(Y)
    Zc, _, _ = oracle.unfused_general(rowptr, colidx, None, X, ones, ("MUL", "RSUM", "SIGMOID", "SEL2ND"), "ASUM")
    np.testing.assert_array_equal(Zc[:, 0], np.diff(rowptr).astype(np.float64))  # neighbour counts


def test_scalar_pattern_wrapper_rejects_general_ops(problem):
    m, n, d, rowptr, colidx, X, Y, vals = problem
    with pytest.raises(ValueError):
        oracle.unfused(rowptr, colidx, None, X, Y, ("ADD", "RSUM", "SIGMOID", "MUL_Y"))
    with pytest.raises(ValueError):
        oracle.unfused(rowptr, colidx, None, X, Y, ("MUL", "NOOP", "SIGMOID", "MUL_Y"))


def test_mean_pooling_is_the_row_normalised_product(problem):
    """SEL2ND, NOOP, EDGE_VALUE, MUL, AMEAN with unit edge values: z_u is the mean of the
    neighbours' feature rows, i.e. D^-1 A Y through scipy's sparse product; a row without
    stored entries gives 0 (Section III-B: GCN variants pool by mean instead of sum)."""
    import scipy.sparse as sp
    m, n, d, rowptr, colidx, X, Y, vals = problem
    ones = np.ones(len(colidx), dtype=np.float32)
    A = sp.csr_matrix((ones.astype(np.float64), colidx, rowptr), shape=(m, n))
    deg = np.diff(rowptr)
    inv = np.where(deg > 0, 1.0 / np.maximum(deg, 1), 0.0)
    ref = sp.diags(inv) @ (A @ Y.astype(np.float64))
    Z, S, _ = oracle.unfused_general(rowptr, colidx, ones, None, Y, ("SEL2ND", "NOOP", "EDGE_VALUE", "MUL_Y"), "AMEAN")
    np.testing.assert_allclose(Z, ref, rtol=1e-13, atol=1e-15)
    assert (Z[[0, 11]] == 0).all() and (S[[0, 11]] == 0).all()
    np.testing.assert_allclose(S, sp.diags(inv) @ (A @ np.abs(Y.astype(np.float64))), rtol=1e-13, atol=1e-15)


def test_mean_of_identical_messages_is_the_message(rng):
    """If every neighbour carries the same feature row c, the mean is c whatever the degree:
    a missing or misplaced division by the row length cannot pass."""
    m, n, d = 12, 40, 5
    rowptr, colidx = random_csr(rng, m, n, 0.4, empty_rows=(3,))
    c = rng.uniform(-2, 2, d).astype(np.float32)
    Y = np.tile(c, (n, 1))
    Z, _, _ = oracle.unfused_general(rowptr, colidx, None, None, Y, ("SEL2ND", "NOOP", "NOOP", "SEL2ND"), "AMEAN")
    deg = np.diff(rowptr)
    assert len(set(deg[deg > 0])) > 3
    np.testing.assert_allclose(Z[deg > 0], np.tile(c.astype(np.float64), ((deg > 0).sum(), 1)), rtol=1e-14)
    assert (Z[3] == 0).all()


def test_mean_is_sum_over_degree_for_a_nonlinear_tuple(problem):
    """AMEAN of the sigmoid-embedding messages equals the pinned ASUM result divided by the
    row lengths (dense numpy reference for the sum)."""
    m, n, d, rowptr, colidx, X, Y, vals = problem
    A = dense_mask(rowptr, colidx, m, n)
    X64, Y64 = X.astype(np.float64), Y.astype(np.float64)
    ref_sum = (A * sigmoid(X64 @ Y64.T)) @ Y64
    deg = np.diff(rowptr)
    Z, _, _ = oracle.unfused_general(rowptr, colidx, None, X, Y, ("MUL", "RSUM", "SIGMOID", "MUL_Y"), "AMEAN")
    np.testing.assert_allclose(Z[deg > 0], ref_sum[deg > 0] / deg[deg > 0, None], rtol=1e-12, atol=1e-14)
