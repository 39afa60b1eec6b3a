"""Pins of the oracle's transposed aggregation (the operator of the backward pass).  The forward
oracle is pinned on its own; here the transposed one is tied to it through the adjoint identity, to
a hand-worked directed example, to a dense matrix built entry by entry, and to the symmetric case."""
import math

import numpy as np

import oracle


def random_directed(rng, n, p):
    M = rng.random((n, n)) < p
    np.fill_diagonal(M, False)
    r, c = np.nonzero(M)
    return r.astype(np.int32), c.astype(np.int32), M


def test_hand_worked_two_node_example():
    # one edge 0 -> 1: rows of A + I are {0, 1} and {1}, so d = (2, 1),
    # A^ = [[1/2, 1/sqrt 2], [0, 1]] and A^T X = [a / 2, a / sqrt 2 + b]
    a, b = 3.0, -5.0
    X = np.array([[a], [b]], dtype=np.float32)
    Z, B = oracle.aggregate_transposed(2, np.array([0], dtype=np.int32), np.array([1], dtype=np.int32), X)
    assert abs(Z[0, 0] - a / 2) < 1e-15 and abs(Z[1, 0] - (a / math.sqrt(2) + b)) < 1e-14
    assert abs(B[1, 0] - (abs(a) / math.sqrt(2) + abs(b))) < 1e-14
    # and the forward operator on the same graph, for contrast: [a / 2 + b / sqrt 2, b]
    _, yd, _, _ = oracle.aggregate(2, np.array([0], dtype=np.int32), np.array([1], dtype=np.int32), X)
    assert abs(yd[0, 0] - (a / 2 + b / math.sqrt(2))) < 1e-14 and abs(yd[1, 0] - b) < 1e-15


def test_adjoint_identity_against_the_forward_oracle():
    rng = np.random.default_rng(0)
    for n, p in ((1, 0.0), (7, 0.4), (50, 0.1), (200, 0.02)):
        r, c, _ = random_directed(rng, n, p)
        X = rng.standard_normal((n, 3)).astype(np.float32)
        G = rng.standard_normal((n, 3)).astype(np.float32)
        _, yd, bound, _ = oracle.aggregate(n, r, c, X)
        Z, _ = oracle.aggregate_transposed(n, r, c, G)
        lhs = float(np.sum(yd * G.astype(np.float64)))
        rhs = float(np.sum(X.astype(np.float64) * Z))
        assert abs(lhs - rhs) <= 1e-12 * float(np.sum(bound * np.abs(G)))


def test_dense_matrix_built_entry_by_entry():
    rng = np.random.default_rng(1)
    n = 23
    r, c, M = random_directed(rng, n, 0.2)
    A1 = M | np.eye(n, dtype=bool)
    d = A1.sum(axis=1)
    Ahat = np.zeros((n, n))
    for i in range(n):
        for j in range(n):
            if A1[i, j]:
                Ahat[i, j] = 1.0 / math.sqrt(float(d[i]) * float(d[j]))
    X = rng.standard_normal((n, 4)).astype(np.float32)
    Z, B = oracle.aggregate_transposed(n, r, c, X)
    want = np.zeros((n, 4))
    for j in range(n):
        for i in range(n):
            want[j] += Ahat[i, j] * X[i].astype(np.float64)
    assert np.max(np.abs(Z - want)) < 1e-13


def test_symmetric_pattern_equals_the_forward_operator_and_input_form_does_not_matter():
    rng = np.random.default_rng(2)
    n = 60
    M = np.triu(rng.random((n, n)) < 0.1, 1)
    M = M | M.T
    r, c = [a.astype(np.int32) for a in np.nonzero(M)]
    X = rng.standard_normal((n, 5)).astype(np.float32)
    _, yd, bound, _ = oracle.aggregate(n, r, c, X)
    Z, B = oracle.aggregate_transposed(n, r, c, X)
    assert np.max(np.abs(Z - yd)) < 1e-13 and np.max(np.abs(B - bound)) < 1e-13
    # duplicates, diagonal entries and the order of the pairs are ignored, as in the forward oracle
    perm = rng.permutation(r.size)
    r2 = np.concatenate([r[perm], r[:5], np.arange(3, dtype=np.int32)])
    c2 = np.concatenate([c[perm], c[:5], np.arange(3, dtype=np.int32)])
    Z2, _ = oracle.aggregate_transposed(n, r2, c2, X)
    assert np.max(np.abs(Z2 - Z)) < 1e-13
