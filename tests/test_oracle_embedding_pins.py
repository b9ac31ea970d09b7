"""Pins for the oracle's minibatch embedding epoch: the update direction is the gradient of the
stated objective (finite differences of an independent numpy objective), one batch that covers
the graph is one dense full-gradient step, and later batches see the rows earlier batches wrote."""
import numpy as np

import oracle
from helpers import random_csr


def sigmoid(x):
    return 1.0 / (1.0 + np.exp(-x))


def objective_row(xu, Ypos, Yneg):
    """sum_v log sigma(x_u.y_v) + sum_w log(1 - sigma(x_u.y_w)); neighbours with multiplicity."""
    return np.log(sigmoid(Ypos @ xu)).sum() + np.log(1.0 - sigmoid(Yneg @ xu)).sum()


def symmetric_pattern(rng, n, density):
    rowptr, colidx = random_csr(rng, n, n, density, empty_rows=(1,))
    return rowptr, colidx


def test_update_is_the_gradient_of_the_objective(rng):
    n, d, s, lr = 9, 4, 3, 1.0
    rowptr, colidx = symmetric_pattern(rng, n, 0.4)
    X0 = rng.uniform(-1, 1, (n, d)).astype(np.float32)
    neg = rng.integers(0, n, (1, s)).astype(np.int32)
    # one batch covering every row: X1 - X0 = lr * gradient, every y held at its old value
    X1, _ = oracle.embedding_epoch(rowptr, colidx, X0, n, neg, lr)
    Y = X0.astype(np.float64)
    eps = 1e-6
    for u in range(n):
        nb = colidx[rowptr[u]:rowptr[u + 1]]
        g = np.zeros(d)
        for k in range(d):
            e = np.zeros(d); e[k] = eps
            g[k] = (objective_row(Y[u] + e, Y[nb], Y[neg[0]]) - objective_row(Y[u] - e, Y[nb], Y[neg[0]])) / (2 * eps)
        step = X1[u].astype(np.float64) - Y[u]
        np.testing.assert_allclose(step, lr * g, rtol=0, atol=2e-6 * max(1.0, np.abs(g).max()))


def test_single_batch_is_one_dense_step(rng):
    n, d, s, lr = 23, 6, 4, 0.05
    rowptr, colidx = symmetric_pattern(rng, n, 0.3)
    X0 = rng.uniform(-1, 1, (n, d)).astype(np.float32)
    neg = rng.integers(0, n, (1, s)).astype(np.int32)
    A = np.zeros((n, n))
    for u in range(n):
        np.add.at(A[u], colidx[rowptr[u]:rowptr[u + 1]], 1.0)
    N = np.zeros((n, n))
    np.add.at(N, (np.repeat(np.arange(n), s), np.tile(neg[0], n)), 1.0)
    Y = X0.astype(np.float64)
    P = Y @ Y.T
    ref = Y + lr * ((A * (1.0 - sigmoid(P))) @ Y - (N * sigmoid(P)) @ Y)
    X1, S = oracle.embedding_epoch(rowptr, colidx, X0, 64, neg, lr)
    np.testing.assert_allclose(X1, ref.astype(np.float32), rtol=0, atol=1e-7)
    np.testing.assert_allclose(S, lr * ((A * (1.0 - sigmoid(P))) @ np.abs(Y) + (N * sigmoid(P)) @ np.abs(Y)), rtol=1e-12)
    assert np.abs(X1[1].astype(np.float64) - ref[1]).max() < 1e-7  # row without neighbours: repulsion only


def test_batches_are_sequential(rng):
    """Two batches: the second reads the rows the first one has already updated."""
    n, d, s, lr, b = 20, 5, 2, 0.1, 10
    rowptr, colidx = symmetric_pattern(rng, n, 0.5)
    X0 = rng.uniform(-1, 1, (n, d)).astype(np.float32)
    neg = rng.integers(0, n, (2, s)).astype(np.int32)
    X1, _ = oracle.embedding_epoch(rowptr, colidx, X0, b, neg, lr)
    Y = X0.astype(np.float64)
    for i in range(2):
        new = Y.copy()
        for u in range(i * b, (i + 1) * b):
            nb = colidx[rowptr[u]:rowptr[u + 1]]
            g = ((1.0 - sigmoid(Y[nb] @ Y[u]))[:, None] * Y[nb]).sum(0) - (sigmoid(Y[neg[i]] @ Y[u])[:, None] * Y[neg[i]]).sum(0)
            new[u] = Y[u] + lr * g
        Y = new.astype(np.float32).astype(np.float64)   # stored in fp32 between batches
    np.testing.assert_allclose(X1, Y.astype(np.float32), rtol=0, atol=1e-7)
    # and it differs from the all-at-once step, so the order is really observed
    Xall, _ = oracle.embedding_epoch(rowptr, colidx, X0, n, neg[:1], lr)
    assert np.abs(Xall[b:] - X1[b:]).max() > 1e-4
