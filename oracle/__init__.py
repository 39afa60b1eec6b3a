"""ctypes front end of the CPU oracle (``pipad_oracle.cpp``).  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's CPU-baseline leg may import this package; the
HIP library never does, and this package never imports the HIP library.  Inputs are edge lists
(directed ``(row, col)`` pairs, host numpy arrays); see the C++ file for what each call computes and
which passages of the paper it follows (Eq. 1 with the symmetric GCN normalisation; the overlap /
exclusive regrouping of Sections 4.1-4.2).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pipad_oracle.cpp")
_LIB = os.path.join(_HERE, "libpipad_oracle.so")
_lib = None


def build(force: bool = True) -> str:
    """Compile the oracle with g++ (always when force, else only if the library is absent)."""
    if force or not os.path.exists(_LIB):
        cmd = ["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-pthread", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        lib = ctypes.CDLL(_LIB)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
        lib.pipad_oracle_overlap_create.restype = vp
        lib.pipad_oracle_overlap_create.argtypes = [i32, i32, vp, vp, vp]
        lib.pipad_oracle_overlap_destroy.restype = None
        lib.pipad_oracle_overlap_destroy.argtypes = [vp]
        lib.pipad_oracle_overlap_nnz.restype = i64
        lib.pipad_oracle_overlap_nnz.argtypes = [vp, i32]
        lib.pipad_oracle_overlap_csr.restype = ctypes.c_int
        lib.pipad_oracle_overlap_csr.argtypes = [vp, i32, vp, vp]
        lib.pipad_oracle_aggregate.restype = ctypes.c_int
        lib.pipad_oracle_aggregate.argtypes = [i32, i64, vp, vp, i32, vp, i64, vp, i64, vp, vp, i32]
        lib.pipad_oracle_hardware_threads.restype = ctypes.c_int
        lib.pipad_oracle_hardware_threads.argtypes = []
        _lib = lib
    return _lib


def hardware_threads() -> int:
    return int(_load().pipad_oracle_hardware_threads())


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


Csr = Tuple[np.ndarray, np.ndarray]  # (rowptr int32[n+1], col int32[nnz])


def overlap(n: int, edge_lists: Sequence[Tuple[np.ndarray, np.ndarray]]) -> Tuple[Csr, List[Csr]]:
    """Splits k snapshots (edge lists) into the overlap CSR and k exclusive CSRs."""
    lib = _load()
    k = len(edge_lists)
    rows = [_i32(r) for r, _ in edge_lists]
    cols = [_i32(c) for _, c in edge_lists]
    for r, c in zip(rows, cols):
        if r.shape != c.shape or r.ndim != 1:
            raise ValueError("rows and cols must be 1-D arrays of equal length")
    nnz = np.array([r.size for r in rows], dtype=np.int64)
    rp = (ctypes.c_void_p * k)(*[r.ctypes.data for r in rows])
    cp = (ctypes.c_void_p * k)(*[c.ctypes.data for c in cols])
    h = lib.pipad_oracle_overlap_create(n, k, nnz.ctypes.data, ctypes.addressof(rp),
                                        ctypes.addressof(cp))
    if not h:
        raise ValueError("oracle rejected the snapshots (index out of range or bad sizes)")
    try:
        parts = []
        for t in range(-1, k):
            m = lib.pipad_oracle_overlap_nnz(h, t)
            rowptr = np.empty(n + 1, dtype=np.int32)
            col = np.empty(m, dtype=np.int32)
            if lib.pipad_oracle_overlap_csr(h, t, rowptr.ctypes.data, col.ctypes.data) != 0:
                raise RuntimeError("pipad_oracle_overlap_csr failed")
            parts.append((rowptr, col))
    finally:
        lib.pipad_oracle_overlap_destroy(h)
    return parts[0], parts[1:]


def aggregate(n: int, rows, cols, X: np.ndarray, threads: int = 1, want_bound: bool = True,
              want_double: bool = True):
    """Y = D^-1/2 (A+I) D^-1/2 X for one snapshot given as an edge list.

    Returns ``(Y float32[n,F], Yd float64[n,F] | None, B float64[n,F] | None, threads_used)`` where
    ``B = |A^| |X|`` element-wise is the scale of the parity tolerance."""
    lib = _load()
    rows, cols = _i32(rows), _i32(cols)
    if X.dtype != np.float32 or X.ndim != 2 or X.strides[1] != 4 or X.strides[0] % 4:
        raise ValueError("X must be a float32 matrix with unit column stride")
    if X.shape[0] != n:
        raise ValueError("X must have n rows")
    F = X.shape[1]
    ldx = X.strides[0] // 4 if n > 1 else max(F, X.strides[0] // 4)
    Y = np.empty((n, F), dtype=np.float32)
    Yd = np.empty((n, F), dtype=np.float64) if want_double else None
    B = np.empty((n, F), dtype=np.float64) if want_bound else None
    used = lib.pipad_oracle_aggregate(
        n, rows.size, rows.ctypes.data, cols.ctypes.data, F, X.ctypes.data, ldx,
        Y.ctypes.data, F, Yd.ctypes.data if want_double else None,
        B.ctypes.data if want_bound else None, threads)
    if used < 1:
        raise ValueError("oracle rejected the arguments")
    return Y, Yd, B, used


def aggregate_update(n: int, rows, cols, X: np.ndarray, W: np.ndarray,
                     bias: Optional[np.ndarray] = None, threads: int = 1):
    """One GCN layer of one snapshot as Eq. 1 composes it: the update (a fully connected layer
    with weights W[F, Fo] and optional bias[Fo], Section 2.1) applied to the aggregation result,
    H = (D^-1/2 (A+I) D^-1/2 X) W + bias, in float64 from the float32 inputs.

    Returns ``(H float64[n, Fo], B2 float64[n, Fo])`` with ``B2 = (|A^| |X|) |W| + |bias|``, the
    scale of the parity tolerance.  The aggregation is :func:`aggregate`; the product is numpy's
    float64 matmul (a library primitive used as one step)."""
    if W.ndim != 2 or W.shape[0] != X.shape[1]:
        raise ValueError("W must be [F, Fo]")
    _, yd, bound, _ = aggregate(n, rows, cols, X, threads=threads)
    w64 = W.astype(np.float64)
    H = yd @ w64
    B2 = bound @ np.abs(w64)
    if bias is not None:
        b64 = np.asarray(bias, dtype=np.float64).reshape(1, -1)
        if b64.shape[1] != W.shape[1]:
            raise ValueError("bias must have Fo entries")
        H = H + b64
        B2 = B2 + np.abs(b64)
    return H, B2


def aggregate_transposed(n: int, rows, cols, X: np.ndarray):
    """Z = (D^-1/2 (A+I) D^-1/2)^T X for one snapshot given as an edge list: what the backward pass
    of the aggregation multiplies by (the transposed operator, needed as such only for directed
    patterns).  D holds the row sums of A + I, exactly as in :func:`aggregate`: transposing moves the
    entries, not the normalisation.  Written out from the definition in float64:
    Z[j] += X[i] / sqrt(d_i d_j) for every pair (i, j) of A + I.

    Returns ``(Zd float64[n, F], B float64[n, F])`` with B the same sum over absolute values."""
    rows, cols = _i32(rows), _i32(cols)
    if X.shape[0] != n:
        raise ValueError("X must have n rows")
    keep = rows != cols
    pairs = np.unique(np.stack([rows[keep].astype(np.int64), cols[keep].astype(np.int64)], axis=1),
                      axis=0) if keep.any() else np.zeros((0, 2), dtype=np.int64)
    diag = np.arange(n, dtype=np.int64)
    r = np.concatenate([pairs[:, 0], diag])
    c = np.concatenate([pairs[:, 1], diag])
    d = np.bincount(r, minlength=n).astype(np.float64)
    w = 1.0 / np.sqrt(d[r] * d[c])
    x64 = X.astype(np.float64)
    Zd = np.zeros((n, X.shape[1]), dtype=np.float64)
    B = np.zeros_like(Zd)
    np.add.at(Zd, c, w[:, None] * x64[r])
    np.add.at(B, c, w[:, None] * np.abs(x64[r]))
    return Zd, B
