"""Pins of the oracle's aggregate-then-update (one GCN layer, Eq. 1 / Section 2.1: a fully
connected update on the aggregation result).  None of them repeats the oracle's own matmul: exact
rational arithmetic on a graph whose normalised adjacency is rational, reductions to the (already
pinned) aggregation, and algebraic identities."""
from fractions import Fraction

import numpy as np

import oracle


def complete_graph(n):
    r, c = np.nonzero(~np.eye(n, dtype=bool))
    return r.astype(np.int32), c.astype(np.int32)


def test_complete_graph_with_integer_data_matches_exact_rational_arithmetic():
    # K_n: every entry of D^-1/2 (A+I) D^-1/2 is 1/n, so H = (column means of X) W + b exactly
    n, F, Fo = 5, 3, 4
    rng = np.random.default_rng(0)
    X = rng.integers(-9, 10, size=(n, F)).astype(np.float32)
    W = rng.integers(-5, 6, size=(F, Fo)).astype(np.float32)
    b = rng.integers(-3, 4, size=Fo).astype(np.float32)
    rows, cols = complete_graph(n)
    H, B2 = oracle.aggregate_update(n, rows, cols, X, W, b)
    for o in range(Fo):
        exact = Fraction(int(b[o]))
        scale = Fraction(abs(int(b[o])))
        for f in range(F):
            mean = sum(Fraction(int(X[j, f])) for j in range(n)) / n
            mean_abs = sum(Fraction(abs(int(X[j, f]))) for j in range(n)) / n
            exact += mean * int(W[f, o])
            scale += mean_abs * abs(int(W[f, o]))
        for i in range(n):
            assert abs(H[i, o] - float(exact)) <= 1e-13 * max(1.0, float(scale))
            assert abs(B2[i, o] - float(scale)) <= 1e-13 * max(1.0, float(scale))


def test_identity_weights_reduce_to_the_aggregation():
    rng = np.random.default_rng(1)
    n, F = 40, 6
    M = rng.random((n, n)) < 0.1
    np.fill_diagonal(M, False)
    rows, cols = [a.astype(np.int32) for a in np.nonzero(M)]
    X = rng.standard_normal((n, F)).astype(np.float32)
    _, yd, bound, _ = oracle.aggregate(n, rows, cols, X)
    H, B2 = oracle.aggregate_update(n, rows, cols, X, np.eye(F, dtype=np.float32))
    assert np.array_equal(H, yd) and np.array_equal(B2, bound)
    # a permutation matrix permutes the columns, a single column picks one out with its bias
    perm = rng.permutation(F)
    P = np.zeros((F, F), dtype=np.float32)
    P[perm, np.arange(F)] = 1.0
    Hp, _ = oracle.aggregate_update(n, rows, cols, X, P)
    assert np.array_equal(Hp, yd[:, perm])
    e2 = np.zeros((F, 1), dtype=np.float32)
    e2[2, 0] = -2.0
    H2, B22 = oracle.aggregate_update(n, rows, cols, X, e2, np.array([0.5], dtype=np.float32))
    assert np.allclose(H2[:, 0], -2.0 * yd[:, 2] + 0.5, rtol=0, atol=1e-15)
    assert np.allclose(B22[:, 0], 2.0 * bound[:, 2] + 0.5, rtol=0, atol=1e-15)


def test_empty_graph_is_a_plain_fully_connected_layer():
    # no edges: the aggregation copies X, so H[i, o] = sum_f X[i, f] W[f, o] + b[o], summed here term by term
    n, F, Fo = 7, 5, 3
    rng = np.random.default_rng(2)
    X = rng.standard_normal((n, F)).astype(np.float32)
    W = rng.standard_normal((F, Fo)).astype(np.float32)
    b = rng.standard_normal(Fo).astype(np.float32)
    empty = np.zeros(0, dtype=np.int32)
    H, B2 = oracle.aggregate_update(n, empty, empty, X, W, b)
    for i in range(n):
        for o in range(Fo):
            acc = float(b[o])
            for f in range(F):
                acc += float(X[i, f]) * float(W[f, o])
            assert abs(H[i, o] - acc) <= 1e-14 * B2[i, o]


def test_linear_in_the_weights_and_associative_with_a_second_layer():
    rng = np.random.default_rng(3)
    n, F, Fo = 30, 4, 5
    M = rng.random((n, n)) < 0.15
    np.fill_diagonal(M, False)
    rows, cols = [a.astype(np.int32) for a in np.nonzero(M)]
    X = rng.standard_normal((n, F)).astype(np.float32)
    W1 = rng.integers(-4, 5, size=(F, Fo)).astype(np.float32)
    W2 = rng.integers(-4, 5, size=(F, Fo)).astype(np.float32)
    Ha, _ = oracle.aggregate_update(n, rows, cols, X, W1)
    Hb, _ = oracle.aggregate_update(n, rows, cols, X, W2)
    Hs, B2 = oracle.aggregate_update(n, rows, cols, X, W1 + W2)
    assert np.all(np.abs(Hs - (Ha + Hb)) <= 1e-13 * np.maximum(B2, 1e-300))
    # aggregating X W (update first) gives the same as updating the aggregation: A^(XW) = (A^X)W.
    # X W is formed exactly (small integers) so that it is a valid float32 input
    Xi = rng.integers(-6, 7, size=(n, F)).astype(np.float32)
    XW = (Xi.astype(np.float64) @ W1.astype(np.float64)).astype(np.float32)
    _, y_of_xw, _, _ = oracle.aggregate(n, rows, cols, XW)
    H, B2 = oracle.aggregate_update(n, rows, cols, Xi, W1)
    assert np.all(np.abs(H - y_of_xw) <= 1e-12 * np.maximum(B2, 1e-300))
