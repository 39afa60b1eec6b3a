"""The synthetic generator: canonical CSR output, sizes, symmetry, determinism, overlap rate."""
import numpy as np
import pytest

import synth


def canon_check(n, rowptr, col, edges):
    assert rowptr.dtype == np.int32 and col.dtype == np.int32
    assert rowptr[0] == 0 and rowptr[-1] == 2 * edges == col.size
    assert col.min() >= 0 and col.max() < n
    rows = np.repeat(np.arange(n), np.diff(rowptr))
    assert not np.any(rows == col), "no diagonal"
    key = rows.astype(np.int64) * n + col
    assert np.all(np.diff(key) > 0), "sorted by (row, col), no duplicates"
    rkey = np.sort(col.astype(np.int64) * n + rows)
    assert np.array_equal(key, rkey), "both directions present"


@pytest.mark.parametrize("name", ["tiny", "small"])
def test_chung_lu_configs(name):
    cfg = synth.CONFIGS[name]
    s = synth.make(cfg)
    assert len(s) == cfg.snapshots
    for t in range(cfg.snapshots):
        canon_check(cfg.n, s.rowptr[t], s.col[t], cfg.edges)
    sets = [set(zip(*(a.tolist() for a in s.coo(t)))) for t in range(cfg.k)]
    frac = len(set.intersection(*sets)) / len(sets[0])
    assert abs(frac - (1 - cfg.churn) ** (cfg.k - 1)) < 0.02
    step = len(sets[0] - sets[1]) / len(sets[0])
    assert abs(step - cfg.churn) < 0.01
    deg = np.diff(s.rowptr[0])
    assert deg.max() > 8 * deg.mean(), "power-law tail"
    assert deg.max() <= 2 * np.sqrt(2 * cfg.edges) + 10


def test_rmat_small_instance_and_determinism():
    a = synth.graphs(3000, 20000, 3, 0.02, "rmat", (0.57, 0.19, 0.19), seed=9)
    b = synth.graphs(3000, 20000, 3, 0.02, "rmat", (0.57, 0.19, 0.19), seed=9)
    c = synth.graphs(3000, 20000, 3, 0.02, "rmat", (0.57, 0.19, 0.19), seed=10)
    for t in range(3):
        canon_check(3000, a.rowptr[t], a.col[t], 20000)
        assert np.array_equal(a.col[t], b.col[t]) and np.array_equal(a.rowptr[t], b.rowptr[t])
    assert not np.array_equal(a.col[0], c.col[0])


def test_features_are_uniform_counter_based_and_per_snapshot():
    x0 = synth.features(5, 0, 1000, 16)
    x0b = synth.features(5, 0, 1000, 16)
    x1 = synth.features(5, 1, 1000, 16)
    assert np.array_equal(x0, x0b) and not np.array_equal(x0, x1)
    assert x0.dtype == np.float32 and x0.min() >= -1 and x0.max() < 1
    assert abs(x0.mean()) < 0.03 and abs(x0.std() - 3 ** -0.5) < 0.02
    # every value is m * 2^-23 - 1 for an integer m
    m = (x0.astype(np.float64) + 1) * 2 ** 23
    assert np.array_equal(m, np.round(m))


def test_invalid_arguments():
    with pytest.raises(ValueError):
        synth.graphs(10, 1000, 1, 0.0, "chung-lu", (2.5, 8.0), 0)  # more edges than the graph holds
