"""Pins of the CPU oracle's aggregation against what the mathematics fixes (no GPU).

Everything expected here is built without the oracle: dense matrices written out in numpy long
double from the definition A^ = D^-1/2 (A + I) D^-1/2 (Eq. 1 aggregates over N(v) united with {v}),
closed forms, hand-worked fixtures and invariants.
"""
import itertools
import os

import numpy as np
import pytest

import oracle

LD = np.longdouble


def dense_ahat(n, rows, cols):
    """Dense A^ in long double from a directed edge list (duplicates / diagonal ignored)."""
    A = np.zeros((n, n), dtype=LD)
    for i, j in zip(rows, cols):
        if i != j:
            A[i, j] = 1
    A += np.eye(n, dtype=LD)
    d = A.sum(axis=1)
    s = 1 / np.sqrt(d)
    return s[:, None] * A * s[None, :]


def rand_graph(rng, n, p, symmetric=True):
    M = rng.random((n, n)) < p
    if symmetric:
        M = np.triu(M, 1)
        M = M | M.T
    np.fill_diagonal(M, False)
    r, c = np.nonzero(M)
    return r.astype(np.int32), c.astype(np.int32)


def check_dense(n, rows, cols, X):
    Y, Yd, B, _ = oracle.aggregate(n, rows, cols, X)
    Ah = dense_ahat(n, rows, cols)
    ref = Ah @ X.astype(LD)
    bound = np.abs(Ah) @ np.abs(X.astype(LD))
    scale = np.maximum(bound.astype(np.float64), 1e-300)
    assert np.all(np.abs(Yd - ref.astype(np.float64)) <= 1e-14 * scale)
    assert np.all(np.abs(B - bound.astype(np.float64)) <= 1e-14 * scale)
    assert np.array_equal(Y, Yd.astype(np.float32))


def test_exhaustive_directed_graphs_up_to_4_nodes():
    rng = np.random.default_rng(0)
    for n in (1, 2, 3, 4):
        pairs = [(i, j) for i in range(n) for j in range(n) if i != j]
        X = rng.uniform(-1, 1, size=(n, 3)).astype(np.float32)
        for mask in range(1 << len(pairs)):
            sel = [p for b, p in enumerate(pairs) if mask >> b & 1]
            rows = np.array([p[0] for p in sel], dtype=np.int32)
            cols = np.array([p[1] for p in sel], dtype=np.int32)
            check_dense(n, rows, cols, X)


@pytest.mark.parametrize("seed", range(12))
def test_random_graphs_up_to_64_nodes_match_dense(seed):
    rng = np.random.default_rng(100 + seed)
    n = int(rng.integers(5, 65))
    rows, cols = rand_graph(rng, n, rng.uniform(0.02, 0.6), symmetric=bool(seed % 2))
    F = int(rng.integers(1, 20))
    X = rng.uniform(-1, 1, size=(n, F)).astype(np.float32)
    check_dense(n, rows, cols, X)


@pytest.mark.parametrize("name", ["path3_ahat.txt", "star5_ahat.txt"])
def test_hand_worked_fixtures(golden_dir, name):
    Ah = np.loadtxt(os.path.join(golden_dir, name))
    n = Ah.shape[0]
    if name.startswith("path3"):
        und = [(0, 1), (1, 2)]
    else:
        und = [(0, l) for l in range(1, n)]
    rows = np.array([a for a, b in und] + [b for a, b in und], dtype=np.int32)
    cols = np.array([b for a, b in und] + [a for a, b in und], dtype=np.int32)
    X = np.eye(n, dtype=np.float32)  # Y = A^ itself
    _, Yd, B, _ = oracle.aggregate(n, rows, cols, X)
    assert np.allclose(Yd, Ah, rtol=0, atol=1e-15)
    assert np.allclose(B, np.abs(Ah), rtol=0, atol=1e-15)


def test_complete_graph_gives_column_means():
    n, F = 9, 5
    rng = np.random.default_rng(3)
    rows, cols = np.nonzero(~np.eye(n, dtype=bool))
    X = rng.uniform(-1, 1, size=(n, F)).astype(np.float32)
    _, Yd, _, _ = oracle.aggregate(n, rows, cols, X)
    mean = X.astype(np.float64).mean(axis=0)
    assert np.allclose(Yd, np.broadcast_to(mean, (n, F)), rtol=0, atol=1e-15)


def test_isolated_nodes_and_empty_graph_copy_features():
    n, F = 7, 4
    rng = np.random.default_rng(4)
    X = rng.uniform(-1, 1, size=(n, F)).astype(np.float32)
    Y, Yd, B, _ = oracle.aggregate(n, np.zeros(0, np.int32), np.zeros(0, np.int32), X)
    assert np.array_equal(Y, X) and np.array_equal(Yd, X.astype(np.float64))
    assert np.array_equal(B, np.abs(X).astype(np.float64))
    # one edge 0-1; nodes 2.. stay isolated
    Y, _, _, _ = oracle.aggregate(n, np.array([0, 1], np.int32), np.array([1, 0], np.int32), X)
    assert np.array_equal(Y[2:], X[2:])
    assert np.allclose(Y[0], 0.5 * (X[0].astype(np.float64) + X[1]), atol=1e-7)


def test_star_closed_form():
    n, F = 33, 6
    rng = np.random.default_rng(5)
    X = rng.uniform(-1, 1, size=(n, F)).astype(np.float32)
    leaves = np.arange(1, n, dtype=np.int32)
    rows = np.concatenate([np.zeros(n - 1, np.int32), leaves])
    cols = np.concatenate([leaves, np.zeros(n - 1, np.int32)])
    _, Yd, _, _ = oracle.aggregate(n, rows, cols, X)
    Xd = X.astype(np.float64)
    centre = Xd[0] / n + Xd[1:].sum(axis=0) / np.sqrt(2.0 * n)
    leaf = Xd[1:] / 2 + Xd[0] / np.sqrt(2.0 * n)
    assert np.allclose(Yd[0], centre, rtol=0, atol=1e-14)
    assert np.allclose(Yd[1:], leaf, rtol=0, atol=1e-14)


def test_regular_graph_row_sums_are_one():
    n = 50  # cycle: every d_i = 3, so A^ 1 = 1
    i = np.arange(n, dtype=np.int32)
    rows = np.concatenate([i, (i + 1) % n]).astype(np.int32)
    cols = np.concatenate([(i + 1) % n, i]).astype(np.int32)
    _, Yd, _, _ = oracle.aggregate(n, rows, cols, np.ones((n, 2), np.float32))
    assert np.allclose(Yd, 1.0, rtol=0, atol=1e-15)


@pytest.mark.parametrize("symmetric", [True, False])
def test_sqrt_degree_vector_is_fixed_and_row_sums_match_degrees(symmetric):
    """(A + I) 1 = d, hence A^ sqrt(d) = sqrt(d); and (A^ 1)_i = d_i^-1/2 sum_j d_j^-1/2."""
    rng = np.random.default_rng(6)
    n = 300
    rows, cols = rand_graph(rng, n, 0.03, symmetric)
    nbrs = [set() for _ in range(n)]
    for i, j in zip(rows.tolist(), cols.tolist()):
        nbrs[i].add(j)
    d = np.array([len(s) + 1 for s in nbrs], dtype=np.float64)
    x = np.sqrt(d).astype(np.float32)
    X = np.stack([x, np.ones(n, np.float32)], axis=1)
    _, Yd, _, _ = oracle.aggregate(n, rows, cols, X)
    # column 0: fixed vector (x is sqrt(d) rounded to float, so allow that rounding)
    assert np.allclose(Yd[:, 0], np.sqrt(d), rtol=2e-7, atol=0)
    # column 1: row sums from the degrees, computed here with python sets
    expect = np.array([(sum(d[j] ** -0.5 for j in nbrs[i]) + d[i] ** -0.5) * d[i] ** -0.5
                       for i in range(n)])
    assert np.allclose(Yd[:, 1], expect, rtol=1e-13, atol=0)


def test_symmetry_and_linearity():
    rng = np.random.default_rng(7)
    n, F = 200, 8
    rows, cols = rand_graph(rng, n, 0.05, True)
    X1 = rng.uniform(-1, 1, size=(n, F)).astype(np.float32)
    X2 = rng.uniform(-1, 1, size=(n, F)).astype(np.float32)
    ones = np.ones((n, 1), np.float32)
    _, Y1, _, _ = oracle.aggregate(n, rows, cols, X1)
    _, Y2, _, _ = oracle.aggregate(n, rows, cols, X2)
    _, R, _, _ = oracle.aggregate(n, rows, cols, ones)
    # 1^T A^ X = (A^ 1)^T X for symmetric A
    assert np.allclose(Y1.sum(axis=0), (R * X1.astype(np.float64)).sum(axis=0), atol=1e-12)
    # linearity (2*X1 and X1 + X2/4 are formed exactly enough in float for a 1e-6 check)
    Xc = (2 * X1.astype(np.float64) + 0.25 * X2.astype(np.float64)).astype(np.float32)
    _, Yc, _, _ = oracle.aggregate(n, rows, cols, Xc)
    assert np.allclose(Yc, 2 * Y1 + 0.25 * Y2, atol=1e-6)


def test_input_order_duplicates_and_diagonal_do_not_matter():
    rng = np.random.default_rng(8)
    n, F = 40, 3
    rows, cols = rand_graph(rng, n, 0.2, False)
    X = rng.uniform(-1, 1, size=(n, F)).astype(np.float32)
    _, Yd, B, _ = oracle.aggregate(n, rows, cols, X)
    perm = rng.permutation(rows.size)
    r2 = np.concatenate([rows[perm], rows[:7], np.arange(5, dtype=np.int32)])
    c2 = np.concatenate([cols[perm], cols[:7], np.arange(5, dtype=np.int32)])
    _, Yd2, B2, _ = oracle.aggregate(n, r2, c2, X)
    assert np.array_equal(Yd, Yd2) and np.array_equal(B, B2)


def test_threads_and_strided_input_give_identical_results():
    rng = np.random.default_rng(9)
    n, F = 500, 7
    rows, cols = rand_graph(rng, n, 0.02, True)
    wide = rng.uniform(-1, 1, size=(n, 3 * F)).astype(np.float32)
    X = wide[:, F:2 * F]  # row stride 3F: the middle snapshot of a coalescent operand
    Y1, Yd1, B1, used1 = oracle.aggregate(n, rows, cols, X, threads=1)
    Y4, Yd4, B4, used4 = oracle.aggregate(n, rows, cols, X, threads=4)
    Yc, _, _, _ = oracle.aggregate(n, rows, cols, np.ascontiguousarray(X))
    assert used1 == 1 and used4 == 4
    assert np.array_equal(Yd1, Yd4) and np.array_equal(B1, B4) and np.array_equal(Y1, Yc)


def test_bad_arguments_are_rejected():
    X = np.zeros((3, 2), np.float32)
    with pytest.raises(ValueError):
        oracle.aggregate(3, np.array([0], np.int32), np.array([3], np.int32), X)
    with pytest.raises(ValueError):
        oracle.aggregate(3, np.array([-1], np.int32), np.array([0], np.int32), X)
