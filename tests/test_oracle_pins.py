"""Pins for the CPU oracle: what the paper and the mathematics fix, checked
against code that shares nothing with oracle/fusedmm_oracle.c.

Each reference here is written from the formulas directly (dense loops over
all (u, v) pairs with an adjacency-count matrix, dense matrix products, closed
forms), never through the oracle's op codes or its CSR traversal.
"""
import math

import numpy as np
import pytest

import oracle
from helpers import random_csr

ALPHA = 0.37


def dense_counts(rowptr, colidx, m, n):
    """A[u, v] = number of stored entries (u, v) (1 for simple graphs)."""
    A = np.zeros((m, n), dtype=np.float64)
    for u in range(m):
        for e in range(rowptr[u], rowptr[u + 1]):
            A[u, colidx[e]] += 1.0
    return A


def brute_force(pattern, A, X, Y, values_dense=None, alpha=ALPHA):
    """z_u = sum_v A[u,v] * phi(x_u, y_v, psi(x_u, y_v, a_uv)) by plain loops
    (Eq. 1 with the per-application psi / phi of Table III and the
    t-distribution note)."""
    m, n = A.shape
    d = Y.shape[1]
    Z = np.zeros((m, d))
    X = None if X is None else X.astype(np.float64)
    Y = Y.astype(np.float64)
    for u in range(m):
        for v in range(n):
            if A[u, v] == 0:
                continue
            if pattern == "sigmoid":
                msg = 1.0 / (1.0 + math.exp(-float(np.dot(X[u], Y[v])))) * Y[v]
            elif pattern == "one_minus_sigmoid":
                msg = (1.0 - 1.0 / (1.0 + math.exp(-float(np.dot(X[u], Y[v]))))) * Y[v]
            elif pattern == "gcn":
                msg = values_dense[u, v] * Y[v]
            elif pattern == "tdist":
                diff = X[u] - Y[v]
                msg = diff / (1.0 + float(np.dot(diff, diff)))
            elif pattern == "fr":
                diff = X[u] - Y[v]
                msg = alpha * math.sqrt(float(np.dot(diff, diff))) * diff
            else:
                raise AssertionError(pattern)
            Z[u] += A[u, v] * msg
    return Z


@pytest.mark.parametrize("pattern", ["sigmoid", "one_minus_sigmoid", "gcn", "tdist", "fr"])
@pytest.mark.parametrize("d", [1, 3, 4, 32, 33, 64])
def test_brute_force_rectangular(pattern, d, rng):
    m, n = 23, 41  # m != n and X != Y so a transposed operand or swapped X/Y cannot pass
    rowptr, colidx = random_csr(rng, m, n, 0.2, empty_rows=(0, 7, m - 1))
    X = rng.uniform(-1, 1, (m, d)).astype(np.float32)
    Y = rng.uniform(-1, 1, (n, d)).astype(np.float32)
    vals = rng.uniform(0.1, 2.0, len(colidx)).astype(np.float32)
    A = dense_counts(rowptr, colidx, m, n)
    Vd = np.zeros((m, n))
    for u in range(m):
        for e in range(rowptr[u], rowptr[u + 1]):
            Vd[u, colidx[e]] = vals[e]
    Zb = brute_force(pattern, A, X, Y, Vd)
    Z, S, H = oracle.unfused(rowptr, colidx, vals, X, Y, pattern, alpha=ALPHA)
    np.testing.assert_allclose(Z, Zb, rtol=1e-12, atol=1e-13)
    assert (Z[[0, 7, m - 1]] == 0).all() and (S[[0, 7, m - 1]] == 0).all()


@pytest.mark.parametrize("pattern", ["sigmoid", "tdist", "fr"])
def test_brute_force_square_shared_features_and_duplicates(pattern, rng):
    n, d = 48, 8
    rowptr, colidx = random_csr(rng, n, n, 0.15, duplicates=True, sort_cols=False)
    X = rng.uniform(-1, 1, (n, d)).astype(np.float32)
    A = dense_counts(rowptr, colidx, n, n)  # duplicates count twice: every stored entry is one visit
    Zb = brute_force(pattern, A, X, X)
    Z, _, _ = oracle.unfused(rowptr, colidx, None, X, X, pattern, alpha=ALPHA)
    np.testing.assert_allclose(Z, Zb, rtol=1e-12, atol=1e-13)


def test_gcn_equals_dense_matmul(rng):
    """Table III row 3: the GCN pattern is SpMM, so Z = A @ Y for the dense A."""
    m, n, d = 700, 2048, 16
    rowptr, colidx = random_csr(rng, m, n, 0.01, empty_rows=(3,))
    vals = rng.normal(size=len(colidx)).astype(np.float32)
    Y = rng.normal(size=(n, d)).astype(np.float32)
    A = np.zeros((m, n))
    rows = np.repeat(np.arange(m), np.diff(rowptr))
    A[rows, colidx] = vals
    Z, S, H = oracle.unfused(rowptr, colidx, vals, None, Y, "gcn")
    np.testing.assert_allclose(Z, A @ Y.astype(np.float64), rtol=1e-12, atol=1e-12)
    np.testing.assert_array_equal(H, vals.astype(np.float64))  # the message is the edge value
    # linearity in Y
    Y2 = rng.normal(size=(n, d)).astype(np.float32)
    Z2, _, _ = oracle.unfused(rowptr, colidx, vals, None, Y2, "gcn")
    Zs, _, _ = oracle.unfused(rowptr, colidx, vals, None, (Y + Y2).astype(np.float32), "gcn")
    np.testing.assert_allclose(Zs, A @ (Y + Y2).astype(np.float32).astype(np.float64), rtol=1e-12, atol=1e-12)
    assert np.abs(Zs - (Z + Z2)).max() < 1e-5  # only the fp32 rounding of Y + Y2 separates them


def test_sddmm_matches_masked_dense_product(rng):
    """Eq. 2: H = (X Y^T) (.) A -- the messages before SOP are sampled entries of X Y^T."""
    m, n, d = 60, 90, 12
    rowptr, colidx = random_csr(rng, m, n, 0.1)
    X = rng.normal(size=(m, d)).astype(np.float32)
    Y = rng.normal(size=(n, d)).astype(np.float32)
    # SCAL with alpha = 1 leaves s = x_u . y_v untouched
    _, _, H = oracle.unfused(rowptr, colidx, None, X, Y, ("MUL", "RSUM", "SCAL", "MUL_Y"), alpha=1.0)
    P = X.astype(np.float64) @ Y.astype(np.float64).T
    rows = np.repeat(np.arange(m), np.diff(rowptr))
    np.testing.assert_allclose(H, P[rows, colidx], rtol=1e-12, atol=1e-13)


def test_sigmoid_plus_complement_is_plain_spmm(rng):
    """sigma(s) + (1 - sigma(s)) = 1  =>  Z_sigma + Z_(1-sigma) = A1 @ Y."""
    m, n, d = 50, 70, 16
    rowptr, colidx = random_csr(rng, m, n, 0.12)
    X = rng.uniform(-2, 2, (m, d)).astype(np.float32)
    Y = rng.uniform(-2, 2, (n, d)).astype(np.float32)
    Za, _, Ha = oracle.unfused(rowptr, colidx, None, X, Y, "sigmoid")
    Zb, _, Hb = oracle.unfused(rowptr, colidx, None, X, Y, "one_minus_sigmoid")
    A1 = dense_counts(rowptr, colidx, m, n)
    np.testing.assert_allclose(Za + Zb, A1 @ Y.astype(np.float64), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(Ha + Hb, 1.0, rtol=0, atol=1e-15)
    assert (Ha > 0).all() and (Ha < 1).all()


def test_sigmoid_zero_features_gives_half_spmm(rng):
    """x_u = 0 => s = 0 => sigma = 1/2 exactly => Z = A1 @ Y / 2."""
    m, n, d = 30, 45, 8
    rowptr, colidx = random_csr(rng, m, n, 0.2)
    X = np.zeros((m, d), dtype=np.float32)
    Y = rng.normal(size=(n, d)).astype(np.float32)
    A1 = dense_counts(rowptr, colidx, m, n)
    for pat in ("sigmoid", "one_minus_sigmoid"):
        Z, _, H = oracle.unfused(rowptr, colidx, None, X, Y, pat)
        assert (H == 0.5).all()
        np.testing.assert_allclose(Z, 0.5 * (A1 @ Y.astype(np.float64)), rtol=1e-14, atol=1e-14)


def test_sigmoid_orthogonal_features(rng):
    """Rows of X orthogonal to every row of Y: same as s = 0."""
    m, n, d = 10, 12, 8
    rowptr, colidx = random_csr(rng, m, n, 0.4)
    X = np.zeros((m, d), dtype=np.float32)
    Y = np.zeros((n, d), dtype=np.float32)
    X[:, :4] = rng.integers(-3, 4, (m, 4))
    Y[:, 4:] = rng.integers(-3, 4, (n, 4))
    Z, _, H = oracle.unfused(rowptr, colidx, None, X, Y, "sigmoid")
    assert (H == 0.5).all()


def test_sigmoid_extreme_arguments_stay_finite():
    rowptr = np.array([0, 2], dtype=np.int64)
    colidx = np.array([0, 1], dtype=np.int32)
    X = np.full((1, 4), 100.0, dtype=np.float32)
    Y = np.array([[100.0] * 4, [-100.0] * 4], dtype=np.float32)
    Z, _, H = oracle.unfused(rowptr, colidx, None, X, Y, "sigmoid")
    assert np.isfinite(Z).all() and H[0] == 1.0 and H[1] == 0.0


@pytest.mark.parametrize("s", [37.0, 40.0, 100.0, 700.0])
def test_one_minus_sigmoid_tail_is_not_cancelled(s):
    """Large positive s: 1 - sigmoid(s) = e^-s / (1 + e^-s), still a positive number (2e-304 at s = 700)
    although the literal difference 1 - 1/(1 + e^-s) is exactly 0 in double from s = 37 on.  One edge,
    x = (s, 0), y = (1, 1): the scalar pattern, the general path with a reduction, and the vector message
    (no reduction: SOP on each element of t = x * y = (s, 0), whose second element pins the value 1/2)."""
    expected = math.exp(-s) / (1.0 + math.exp(-s))           # no subtraction from 1 anywhere
    alt = math.exp(-s - math.log1p(math.exp(-s)))            # the same number through its logarithm
    assert expected > 0.0 and abs(alt - expected) <= 4e-14 * expected   # exp of an argument near 700 loses ~|arg| ulps
    assert 1.0 - 1.0 / (1.0 + math.exp(-s)) == 0.0            # the cancellation this pin is about
    rowptr = np.array([0, 1], dtype=np.int64)
    colidx = np.array([0], dtype=np.int32)
    X = np.array([[s, 0.0]], dtype=np.float32)
    Y = np.array([[1.0, 1.0]], dtype=np.float32)
    Z, S, H = oracle.unfused(rowptr, colidx, None, X, Y, "one_minus_sigmoid")
    assert H[0] > 0.0 and abs(H[0] - expected) <= 1e-15 * expected
    np.testing.assert_allclose(Z[0], [expected, expected], rtol=1e-15, atol=0.0)
    np.testing.assert_allclose(S[0], [expected, expected], rtol=1e-15, atol=0.0)
    Zg, _, Hg = oracle.unfused_general(rowptr, colidx, None, X, Y, ("MUL", "RSUM", "ONE_MINUS_SIGMOID", "MUL_Y"))
    assert Hg[0] > 0.0 and abs(Hg[0] - expected) <= 1e-15 * expected and np.array_equal(Zg, Z)
    Zv, _, Hv = oracle.unfused_general(rowptr, colidx, None, X, Y, ("MUL", "NOOP", "ONE_MINUS_SIGMOID", "MUL_Y"))
    assert Hv.shape == (1, 2) and Hv[0, 1] == 0.5
    assert Hv[0, 0] > 0.0 and abs(Hv[0, 0] - expected) <= 1e-15 * expected
    np.testing.assert_allclose(Zv[0], [expected, 0.5], rtol=1e-15, atol=0.0)
    # and the two halves still add up to one where both are representable
    _, _, Hs = oracle.unfused(rowptr, colidx, None, X, Y, "sigmoid")
    assert Hs[0] + H[0] == 1.0


@pytest.mark.parametrize("pattern", ["tdist", "fr"])
def test_difference_patterns_vanish_on_equal_rows(pattern, rng):
    n, d = 40, 6
    rowptr, colidx = random_csr(rng, n, n, 0.2)
    X = np.tile(rng.normal(size=(1, d)).astype(np.float32), (n, 1))
    Z, S, _ = oracle.unfused(rowptr, colidx, None, X, X, pattern, alpha=ALPHA)
    assert (Z == 0).all() and (S == 0).all()


@pytest.mark.parametrize("pattern", ["tdist", "fr"])
def test_difference_patterns_antisymmetric_total(pattern, rng):
    """Symmetric graph, Y = X: the message on (u,v) is minus the one on (v,u),
    so the sum of all z_u vanishes up to rounding."""
    n, d = 60, 10
    up = np.triu(rng.random((n, n)) < 0.1, 1)
    A = up | up.T
    rowptr = np.zeros(n + 1, dtype=np.int64)
    rowptr[1:] = np.cumsum(A.sum(1))
    colidx = np.nonzero(A)[1].astype(np.int32)
    X = rng.normal(size=(n, d)).astype(np.float32)
    Z, S, _ = oracle.unfused(rowptr, colidx, None, X, X, pattern, alpha=ALPHA)
    assert np.abs(Z.sum(0)).max() <= 1e-12 * S.sum(0).max()
    assert np.abs(Z).max() > 1e-3  # not trivially zero


def test_two_vertex_closed_forms():
    """One edge 0 -> 1: z_0 = t/(1+|t|^2) (t-dist) and alpha*|t|*t (FR) with t = x_0 - y_1;
    z_0 = sigma(x_0.y_1) y_1 for the embedding pattern.  Fixes sign and operand order."""
    rowptr = np.array([0, 1, 1], dtype=np.int64)
    colidx = np.array([1], dtype=np.int32)
    X = np.array([[1.0, 2.0, -1.0], [9.0, 9.0, 9.0]], dtype=np.float32)
    Y = np.array([[7.0, 7.0, 7.0], [0.5, -1.0, 2.0]], dtype=np.float32)
    t = np.array([0.5, 3.0, -3.0])
    n2 = 0.25 + 9.0 + 9.0
    Z, _, H = oracle.unfused(rowptr, colidx, None, X, Y, "tdist")
    np.testing.assert_allclose(Z[0], t / (1.0 + n2), rtol=1e-15)
    assert H[0] == 1.0 / (1.0 + n2) and (Z[1] == 0).all()
    Z, _, H = oracle.unfused(rowptr, colidx, None, X, Y, "fr", alpha=0.25)
    np.testing.assert_allclose(Z[0], 0.25 * math.sqrt(n2) * t, rtol=1e-15)
    s = 1.0 * 0.5 + 2.0 * -1.0 + -1.0 * 2.0  # = -3.5
    Z, _, H = oracle.unfused(rowptr, colidx, None, X, Y, "sigmoid")
    np.testing.assert_allclose(Z[0], (1.0 / (1.0 + math.exp(3.5))) * Y[1].astype(np.float64), rtol=1e-15)
    Z, _, H = oracle.unfused(rowptr, colidx, None, X, Y, "one_minus_sigmoid")
    np.testing.assert_allclose(H[0], 1.0 / (1.0 + math.exp(-3.5)), rtol=1e-15)


def test_all_rows_empty():
    rowptr = np.zeros(6, dtype=np.int64)
    colidx = np.zeros(0, dtype=np.int32)
    X = np.ones((5, 4), dtype=np.float32)
    for pat in oracle.PATTERNS:
        Z, S, H = oracle.unfused(rowptr, colidx, np.zeros(0, np.float32), X, X, pat)
        assert Z.shape == (5, 4) and (Z == 0).all() and (S == 0).all() and len(H) == 0


@pytest.mark.parametrize("pattern", ["sigmoid", "gcn", "tdist", "fr"])
def test_neighbour_order_only_changes_rounding(pattern, rng):
    m, n, d = 30, 50, 16
    rowptr, colidx = random_csr(rng, m, n, 0.3)
    vals = rng.uniform(0.1, 1.0, len(colidx)).astype(np.float32)
    X = rng.normal(size=(m, d)).astype(np.float32)
    Y = rng.normal(size=(n, d)).astype(np.float32)
    Z0, S0, _ = oracle.unfused(rowptr, colidx, vals, X, Y, pattern, alpha=ALPHA)
    col2, val2 = colidx.copy(), vals.copy()
    for u in range(m):
        p = rng.permutation(rowptr[u + 1] - rowptr[u]) + rowptr[u]
        col2[rowptr[u]:rowptr[u + 1]] = colidx[p]
        val2[rowptr[u]:rowptr[u + 1]] = vals[p]
    Z1, S1, _ = oracle.unfused(rowptr, col2, val2, X, Y, pattern, alpha=ALPHA)
    assert np.abs(Z1 - Z0).max() <= 1e-12 * S0.max()
    err, _, viol = oracle.compare(Z1, Z0, S0)
    assert err <= 1e-12 and viol == 0


@pytest.mark.parametrize("pattern", list(oracle.PATTERNS))
def test_fused_order_equals_two_phase_bitwise(pattern, rng):
    """The paper: fusing does not alter the computation.  Algorithm 1's per-row
    five-step loop, the two-phase pipeline with scalar H, and the pipeline with
    the full nnz x d message tensor agree bit for bit in double."""
    m, n, d = 25, 35, 7
    rowptr, colidx = random_csr(rng, m, n, 0.25, empty_rows=(4,))
    vals = rng.uniform(0.1, 1.0, len(colidx)).astype(np.float32)
    X = rng.normal(size=(m, d)).astype(np.float32)
    Y = rng.normal(size=(n, d)).astype(np.float32)
    Z2, _, _ = oracle.unfused(rowptr, colidx, vals, X, Y, pattern, alpha=ALPHA)
    Zf = oracle.update_u(rowptr, colidx, vals, X, Y, pattern, alpha=ALPHA)
    W, Zw = oracle.message_tensor(rowptr, colidx, vals, X, Y, pattern, alpha=ALPHA)
    np.testing.assert_array_equal(Z2, Zf)
    np.testing.assert_array_equal(Z2, Zw)
    assert W.shape == (len(colidx), d)


def test_row_independence(rng):
    """Row u of Z depends only on row u of A, x_u and Y (no write sharing between rows)."""
    m, n, d = 20, 30, 5
    rowptr, colidx = random_csr(rng, m, n, 0.3)
    X = rng.normal(size=(m, d)).astype(np.float32)
    Y = rng.normal(size=(n, d)).astype(np.float32)
    Z, _, _ = oracle.unfused(rowptr, colidx, None, X, Y, "sigmoid")
    for u in (0, 9, m - 1):
        rp = np.array([0, rowptr[u + 1] - rowptr[u]], dtype=np.int64)
        ci = colidx[rowptr[u]:rowptr[u + 1]]
        Zu, _, _ = oracle.unfused(rp, ci, None, X[u:u + 1], Y, "sigmoid")
        np.testing.assert_array_equal(Zu[0], Z[u])


def test_float_instantiation_close_to_double(rng):
    """The fp32 build (timed as the CPU baseline) computes the same thing."""
    m, n, d = 40, 40, 32
    rowptr, colidx = random_csr(rng, m, n, 0.2)
    X = rng.uniform(-0.5, 0.5, (m, d)).astype(np.float32)
    Z64, S, _ = oracle.unfused(rowptr, colidx, None, X, X, "one_minus_sigmoid")
    Z32, _, _ = oracle.unfused(rowptr, colidx, None, X, X, "one_minus_sigmoid", precision="f32")
    err, _, viol = oracle.compare(Z32, Z64, S)
    assert err < 1e-5 and viol == 0


def test_compare_rule():
    Zr = np.array([[1.0, 0.0]])
    S = np.array([[2.0, 0.0]])
    assert oracle.compare(np.array([[1.0002, 0.0]]), Zr, S)[0] == pytest.approx(1e-4)
    assert oracle.compare(np.array([[1.0, 1e-30]]), Zr, S)[2] == 1  # S == 0 demands an exact zero
    assert oracle.compare(np.array([[np.nan, 0.0]]), Zr, S)[0] == float("inf")


def test_planted_mistakes_are_caught(rng):
    """The pins above are sharp enough: typical slips change the brute-force result
    by far more than the tolerance, so an oracle carrying one would fail them."""
    m, n, d = 12, 17, 5
    rowptr, colidx = random_csr(rng, m, n, 0.3)
    X = rng.uniform(-1, 1, (m, d)).astype(np.float32)
    Y = rng.uniform(-1, 1, (n, d)).astype(np.float32)
    A = dense_counts(rowptr, colidx, m, n)
    Z, S, _ = oracle.unfused(rowptr, colidx, None, X, Y, "tdist")
    wrong_sign = -brute_force("tdist", A, X, Y)
    assert np.abs(Z - wrong_sign).max() > 1e-2
    Zs, _, _ = oracle.unfused(rowptr, colidx, None, X, Y, "sigmoid")
    swapped = brute_force("one_minus_sigmoid", A, X, Y)  # complement in place of sigma
    assert np.abs(Zs - swapped).max() > 1e-2
