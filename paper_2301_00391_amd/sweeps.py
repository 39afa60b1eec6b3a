"""Sensitivity sweeps of the frame-parallel aggregation on synthetic frames (needs a GPU).

Analogues of the paper's offline analysis of its parallel GNN (Section 4.4, Fig. 9: speedup of
S_per in {2, 4, 8} snapshots per partition over one-snapshot execution, against overlap rate and
against the feature dimension) and of its dimension-sensitivity test (Section 5.3, Fig. 11b),
on the synthetic generator instead of the paper's datasets.

  python -m paper_2301_00391_amd.sweeps overlap   # churn x k table
  python -m paper_2301_00391_amd.sweeps features  # F x k table

Every cell times ``pipad_frame_aggregate`` of one frame of k snapshots and, as the baseline, the
same k snapshots aggregated one at a time (k frames of a single snapshot each, whose overlap part
is the whole snapshot).  Output: a markdown table on stdout.
"""
from __future__ import annotations

import sys

import numpy as np
import torch

import synth
import paper_2301_00391_amd as pipad


def _time(fn, reps=5):
    fn()
    torch.cuda.synchronize()
    a = torch.cuda.Event(enable_timing=True)
    b = torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / reps


def _frame_times(snaps, k, feat, dev):
    n = snaps.n
    gs = [(torch.from_numpy(snaps.rowptr[t]).to(dev), torch.from_numpy(snaps.col[t]).to(dev))
          for t in range(k)]
    frame = pipad.frame_build_overlap(gs)
    singles = [pipad.frame_build_overlap([g]) for g in gs]
    layout_wide = False  # k separate matrices: the layout the slice-per-XCD kernel prefers
    xw = torch.rand((n, k, feat), device=dev) * 2 - 1
    if layout_wide:
        x, y = xw, torch.empty_like(xw)
        xs = [xw[:, t:t + 1, :] for t in range(k)]
        ys = [y[:, t:t + 1, :] for t in range(k)]
    else:
        x = [xw[:, t, :].contiguous() for t in range(k)]
        y = [torch.empty_like(v) for v in x]
        xs = [[v] for v in x]
        ys = [[v] for v in y]
    t_frame = _time(lambda: pipad.frame_aggregate(frame, x, y))

    def one_by_one():
        for t in range(k):
            pipad.frame_aggregate(singles[t], xs[t], ys[t])

    t_single = _time(one_by_one)
    nnz_c = int(frame.common()[1].numel())
    rate = nnz_c / float(np.mean([snaps.col[t].size for t in range(k)]))
    for f in singles:
        f.close()
    frame.close()
    return t_frame, t_single, rate


def overlap_sweep(dev):
    n, edges, feat = 200_000, 1_600_000, 64
    print(f"Chung-Lu gamma 2.1, N = {n}, {edges} undirected edges per snapshot, F = {feat}; "
          "cell = frame ms / one-at-a-time ms (speedup); OR = overlap rate |C| / mean |E_t|\n")
    print("| churn per step | " + " | ".join(f"k = {k}" for k in (2, 4, 8)) + " |")
    print("|---|---|---|---|")
    for churn in (0.01, 0.03, 0.10, 0.20, 0.40):
        snaps = synth.graphs(n, edges, 8, churn, "chung-lu", (2.1, 16.0), seed=2)
        cells = []
        for k in (2, 4, 8):
            tf, ts, rate = _frame_times(snaps, k, feat, dev)
            cells.append(f"OR {rate:.2f}: {tf:.3f} / {ts:.3f} ({ts / tf:.2f}x)")
        print(f"| {churn:.0%} | " + " | ".join(cells) + " |", flush=True)


def feature_sweep(dev):
    n, edges, churn = 200_000, 1_600_000, 0.03
    snaps = synth.graphs(n, edges, 8, churn, "chung-lu", (2.1, 16.0), seed=2)
    print(f"Chung-Lu gamma 2.1, N = {n}, {edges} undirected edges per snapshot, churn {churn:.0%}; "
          "cell = frame ms / one-at-a-time ms (speedup)\n")
    print("| F | " + " | ".join(f"k = {k}" for k in (2, 4, 8)) + " |")
    print("|---|---|---|---|")
    for feat in (2, 6, 16, 32, 64, 128):
        cells = []
        for k in (2, 4, 8):
            tf, ts, _ = _frame_times(snaps, k, feat, dev)
            cells.append(f"{tf:.3f} / {ts:.3f} ({ts / tf:.2f}x)")
        print(f"| {feat} | " + " | ".join(cells) + " |", flush=True)


def main(argv):
    if not torch.cuda.is_available():
        print("sweeps need a GPU", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    which = argv[1] if len(argv) > 1 else "overlap"
    if which == "overlap":
        overlap_sweep(dev)
    elif which == "features":
        feature_sweep(dev)
    else:
        print(__doc__, file=sys.stderr)
        return 2
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
