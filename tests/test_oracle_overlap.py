"""Pins of the CPU oracle's overlap / exclusive decomposition (no GPU).

Section 4.1-4.2: the snapshots of a group are regrouped as one overlap part shared by all of them
plus one exclusive part each.  Expected values come from python sets, not from the oracle.
"""
import numpy as np
import pytest

import oracle
import synth


def csr_to_set(n, csr):
    rowptr, col = csr
    assert rowptr.shape == (n + 1,) and rowptr[0] == 0 and rowptr[-1] == col.size
    assert np.all(np.diff(rowptr) >= 0)
    out = set()
    for i in range(n):
        seg = col[rowptr[i]:rowptr[i + 1]]
        assert np.all(np.diff(seg) > 0), "columns must be strictly ascending within a row"
        out.update((i, int(j)) for j in seg)
    return out


def rand_edges(rng, n, m):
    r = rng.integers(0, n, size=m).astype(np.int32)
    c = rng.integers(0, n, size=m).astype(np.int32)
    return r, c


def py_sets(lists):
    return [{(int(i), int(j)) for i, j in zip(r, c) if i != j} for r, c in lists]


@pytest.mark.parametrize("seed", range(10))
def test_matches_set_intersection_on_small_random_graphs(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 65))
    k = int(rng.integers(1, 7))
    base = rand_edges(rng, n, int(rng.integers(0, 6 * n + 1)))
    lists = []
    for _ in range(k):
        extra = rand_edges(rng, n, int(rng.integers(0, n + 1)))
        keep = rng.random(base[0].size) < 0.8
        lists.append((np.concatenate([base[0][keep], extra[0]]),
                      np.concatenate([base[1][keep], extra[1]])))
    common, excl = oracle.overlap(n, lists)
    sets = py_sets(lists)
    want_common = set.intersection(*sets)
    assert csr_to_set(n, common) == want_common
    for t in range(k):
        assert csr_to_set(n, excl[t]) == sets[t] - want_common


def test_partition_invariants_on_synthetic_frames():
    cfg = synth.CONFIGS["tiny"]
    snaps = synth.make(cfg)
    lists = [snaps.coo(t) for t in range(cfg.k)]
    common, excl = oracle.overlap(cfg.n, lists)
    C = csr_to_set(cfg.n, common)
    sets = py_sets(lists)
    D = [csr_to_set(cfg.n, e) for e in excl]
    for t in range(cfg.k):
        assert C.isdisjoint(D[t])
        assert C | D[t] == sets[t]
        assert len(C) + len(D[t]) == len(sets[t])
    assert set.intersection(*D) == set()  # the overlap is maximal
    # undirected input => both parts stay symmetric
    assert C == {(j, i) for i, j in C}


def test_special_cases():
    rng = np.random.default_rng(11)
    n = 30
    a = rand_edges(rng, n, 120)
    sa = py_sets([a])[0]
    # k = 1: everything is overlap
    common, excl = oracle.overlap(n, [a])
    assert csr_to_set(n, common) == sa and excl[0][1].size == 0
    # identical snapshots: no exclusive edges
    common, excl = oracle.overlap(n, [a, a, a])
    assert csr_to_set(n, common) == sa and all(e[1].size == 0 for e in excl)
    # pairwise disjoint snapshots: empty overlap, exclusive = whole snapshot
    b = (a[0], (a[1] + 1) % n)
    sb = py_sets([b])[0] - sa
    rb = np.array([i for i, j in sb], np.int32)
    cb = np.array([j for i, j in sb], np.int32)
    common, excl = oracle.overlap(n, [a, (rb, cb)])
    assert common[1].size == 0
    assert csr_to_set(n, excl[0]) == sa and csr_to_set(n, excl[1]) == sb
    # empty graph / no nodes
    common, excl = oracle.overlap(0, [(np.zeros(0, np.int32), np.zeros(0, np.int32))])
    assert common[0].tolist() == [0] and common[1].size == 0


def test_out_of_range_is_rejected():
    with pytest.raises(ValueError):
        oracle.overlap(3, [(np.array([0], np.int32), np.array([5], np.int32))])
