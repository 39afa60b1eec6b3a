"""Seeded synthetic frames: the only module shared by the CPU oracle's tests and the HIP path's tests.

It holds none of the method's arithmetic (no normalisation, no intersection, no aggregation): it
draws random graph snapshots and random features, nothing else.  The graphs stand in for the
paper's Table 1 datasets, which are not available: power-law graphs whose topology changes by a
small fraction between adjacent snapshots (Section 3.1, "Topology overlap": about 10 % on average),
processed in groups of 2-8 snapshots (Section 4.3).

Native part: ``pipad_synth.cpp`` -> ``libpipad_synth.so`` (g++, OpenMP), loaded with ctypes.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pipad_synth.cpp")
_LIB = os.path.join(_HERE, "libpipad_synth.so")
_lib = None


def build(force: bool = True) -> str:
    """Compile the generator with g++ (always when force, else only if the library is absent)."""
    if force or not os.path.exists(_LIB):
        cmd = ["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-fopenmp", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        lib = ctypes.CDLL(_LIB)
        lib.pipad_synth_graphs.restype = ctypes.c_int
        lib.pipad_synth_graphs.argtypes = [
            ctypes.c_int, ctypes.c_int32, ctypes.c_int64, ctypes.c_int32, ctypes.c_int64,
            ctypes.c_double, ctypes.c_double, ctypes.c_double, ctypes.c_uint64,
            ctypes.c_void_p, ctypes.c_void_p]
        lib.pipad_synth_features.restype = None
        lib.pipad_synth_features.argtypes = [
            ctypes.c_uint64, ctypes.c_int32, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p]
        _lib = lib
    return _lib


@dataclass(frozen=True)
class Config:
    """One synthetic workload.  ``edges`` is the number of undirected edges of every snapshot."""
    name: str
    n: int
    snapshots: int
    k: int
    model: str            # "chung-lu" | "rmat"
    params: Tuple[float, ...]
    edges: int
    churn: float
    feat: int
    seed: int

    @property
    def frames(self) -> int:
        """Number of frames when the window of k snapshots slides by one (Section 3.3)."""
        return self.snapshots - self.k + 1


# The five workloads this build is measured on (sizes, models and seeds are fixed by the task).
CONFIGS = {
    "tiny": Config("tiny", 2_000, 4, 4, "chung-lu", (2.5, 8.0), 8_000, 0.05, 16, 0),
    "small": Config("small", 20_000, 16, 4, "chung-lu", (2.2, 12.0), 120_000, 0.10, 32, 1),
    "medium": Config("medium", 200_000, 16, 8, "chung-lu", (2.1, 16.0), 1_600_000, 0.03, 64, 2),
    "large": Config("large", 1_000_000, 8, 8, "rmat", (0.57, 0.19, 0.19), 10_000_000, 0.01, 64, 3),
    "low-overlap": Config("low-overlap", 500_000, 8, 8, "chung-lu", (2.3, 20.0), 5_000_000, 0.40,
                          128, 4),
}


@dataclass
class Snapshots:
    """n_snap canonical CSR snapshots (undirected, both directions stored, ascending columns,
    no duplicates, no diagonal).  ``rowptr[t]`` is int32[n+1], ``col[t]`` is int32[2*edges]."""
    n: int
    rowptr: List[np.ndarray] = field(default_factory=list)
    col: List[np.ndarray] = field(default_factory=list)

    def __len__(self) -> int:
        return len(self.rowptr)

    def coo(self, t: int) -> Tuple[np.ndarray, np.ndarray]:
        """Directed (row, col) pairs of snapshot t (plain expansion of the row pointer)."""
        rp = self.rowptr[t]
        rows = np.repeat(np.arange(self.n, dtype=np.int32), np.diff(rp))
        return rows, self.col[t]


def graphs(n: int, edges: int, snapshots: int, churn: float, model: str,
           params: Tuple[float, ...], seed: int) -> Snapshots:
    """Draws ``snapshots`` graphs: the first from the model, each later one by removing
    round(churn*edges) uniformly chosen undirected edges and adding as many fresh ones."""
    lib = _load()
    rowptr = np.empty((snapshots, n + 1), dtype=np.int32)
    col = np.empty((snapshots, 2 * edges), dtype=np.int32)
    p = tuple(params) + (0.0,) * (3 - len(params))
    m = {"chung-lu": 0, "rmat": 1}[model]
    rc = lib.pipad_synth_graphs(m, n, edges, snapshots, int(round(churn * edges)),
                                p[0], p[1], p[2], seed, rowptr.ctypes.data, col.ctypes.data)
    if rc != 0:
        raise ValueError(f"pipad_synth_graphs rejected its arguments (rc={rc})")
    return Snapshots(n, [rowptr[t] for t in range(snapshots)], [col[t] for t in range(snapshots)])


def features(seed: int, t: int, n: int, feat: int, out: np.ndarray | None = None) -> np.ndarray:
    """X_t: float32[n, feat], iid uniform on [-1, 1), re-drawn for every snapshot index t."""
    lib = _load()
    if out is None:
        out = np.empty((n, feat), dtype=np.float32)
    assert out.dtype == np.float32 and out.flags.c_contiguous and out.size == n * feat
    lib.pipad_synth_features(seed, t, 0, n * feat, out.ctypes.data)
    return out


def make(cfg: Config | str) -> Snapshots:
    """All snapshots of a named workload."""
    if isinstance(cfg, str):
        cfg = CONFIGS[cfg]
    return graphs(cfg.n, cfg.edges, cfg.snapshots, cfg.churn, cfg.model, cfg.params, cfg.seed)
