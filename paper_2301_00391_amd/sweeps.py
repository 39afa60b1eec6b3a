"""Sensitivity sweeps of the frame-parallel aggregation on synthetic frames (needs a GPU).

Analogues of the paper's offline analysis of its parallel GNN (Section 4.4, Fig. 9: speedup of
S_per in {2, 4, 8} snapshots per partition over one-snapshot execution, against overlap rate and
against the feature dimension) and of its dimension-sensitivity test (Section 5.3, Fig. 11b),
on the synthetic generator instead of the paper's datasets.

  python -m paper_2301_00391_amd.sweeps overlap   # churn x k table
  python -m paper_2301_00391_amd.sweeps features  # F x k table
  python -m paper_2301_00391_amd.sweeps sliding   # cost per new snapshot when the frame slides by one
  python -m paper_2301_00391_amd.sweeps workloads # the benchmark frames: one frame vs one snapshot at a time
  python -m paper_2301_00391_amd.sweeps smallf    # F = 2 / 6 / 16: the coalescent kernel vs per-snapshot slices

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


def _frame_times(snaps, k, feat, dev, with_concatenated=False):
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
    # the physically concatenated (coalescent) operand: where the small-F kernel applies
    t_concat = None
    if with_concatenated:
        yw = torch.empty_like(xw)
        t_concat = _time(lambda: pipad.frame_aggregate(frame, xw, yw))
    nnz_c = int(frame.common()[1].numel())
    rate = nnz_c / float(np.mean([snaps.col[t].size for t in range(k)]))
    for f in singles:
        f.close()
    frame.close()
    if with_concatenated:
        return t_frame, t_single, rate, t_concat
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
          "cell = frame ms on k separate matrices [/ frame ms on the concatenated operand] / "
          "one-at-a-time ms (speedup of the better frame)\n")
    print("| F | " + " | ".join(f"k = {k}" for k in (2, 4, 8)) + " |")
    print("|---|---|---|---|")
    for feat in (2, 6, 16, 32, 64, 128):
        cells = []
        for k in (2, 4, 8):
            if feat < 32:
                tf, ts, _, tc = _frame_times(snaps, k, feat, dev, with_concatenated=True)
                cells.append(f"{tf:.3f} / {tc:.3f} / {ts:.3f} ({ts / min(tf, tc):.2f}x)")
            else:
                tf, ts, _ = _frame_times(snaps, k, feat, dev)
                cells.append(f"{tf:.3f} / {ts:.3f} ({ts / tf:.2f}x)")
        print(f"| {feat} | " + " | ".join(cells) + " |", flush=True)


def sliding_sweep(dev):
    """Frames that slide by one snapshot (Section 3.3) share k - 1 snapshots with their
    predecessor.  The aggregation of the raw input features depends on the snapshot alone, so its
    result can be kept across frames (the paper's inter-frame reuse, Section 4.3); layers whose
    input depends on the weights need the whole frame again.  Three ways to pay per new snapshot:
    the whole frame again; only the entering snapshot, as a frame of its own; or - when the
    snapshots are known in advance, as in training - disjoint groups of k snapshots aggregated as
    frames once, cost divided by k."""
    print("cost per new snapshot in ms (build_overlap + aggregate), stride-1 frames\n")
    print("| workload | whole frame again | entering snapshot alone | disjoint groups of k, per snapshot |")
    print("|---|---|---|---|")
    for name in ("small", "medium"):
        cfg = synth.CONFIGS[name]
        n, k, feat = cfg.n, cfg.k, cfg.feat
        snaps = synth.graphs(n, cfg.edges, cfg.snapshots, cfg.churn, cfg.model, cfg.params, cfg.seed)
        gs = [(torch.from_numpy(snaps.rowptr[t]).to(dev), torch.from_numpy(snaps.col[t]).to(dev))
              for t in range(cfg.snapshots)]
        xs = [torch.rand((n, feat), device=dev) * 2 - 1 for _ in range(cfg.snapshots)]
        ys = [torch.empty_like(x) for x in xs]

        def whole():
            for f in range(cfg.frames):
                fr = pipad.frame_build_overlap(gs[f:f + k])
                pipad.frame_aggregate(fr, xs[f:f + k], ys[f:f + k])

        def entering():
            for f in range(cfg.frames):
                t = f + k - 1
                fr = pipad.frame_build_overlap(gs[t:t + 1])
                pipad.frame_aggregate(fr, xs[t:t + 1], ys[t:t + 1])

        def groups():
            for g in range(cfg.snapshots // k):
                fr = pipad.frame_build_overlap(gs[g * k:(g + 1) * k])
                pipad.frame_aggregate(fr, xs[g * k:(g + 1) * k], ys[g * k:(g + 1) * k])

        t_whole = _time(whole, 3) / cfg.frames
        t_enter = _time(entering, 3) / cfg.frames
        t_group = _time(groups, 3) / (cfg.snapshots // k * k)
        print(f"| {name} (N = {n}, k = {k}, F = {feat}, {cfg.frames} frames) | {t_whole:.3f} | "
              f"{t_enter:.3f} | {t_group:.3f} |", flush=True)


def workload_sweep(dev):
    """The benchmark workloads in the benchmark layout: one frame of k snapshots against the same
    snapshots handled one at a time (k frames of one snapshot, whose overlap part is the whole
    snapshot), for the extraction and for the aggregation."""
    print("ms per frame; aggregation in the benchmark layout (rows of X padded to an odd number of "
          "128-byte lines)\n")
    print("| workload | extraction: frame | extraction: k single snapshots | aggregation: frame | "
          "aggregation: one at a time |")
    print("|---|---|---|---|---|")
    for name in ("medium", "large", "low-overlap"):
        cfg = synth.CONFIGS[name]
        n, k, feat = cfg.n, cfg.k, cfg.feat
        snaps = synth.graphs(n, cfg.edges, k, cfg.churn, cfg.model, cfg.params, cfg.seed)
        gs = [(torch.from_numpy(snaps.rowptr[t]).to(dev), torch.from_numpy(snaps.col[t]).to(dev))
              for t in range(k)]
        stride = pipad.padded_row_stride(feat)
        xb = [torch.rand((n, stride), device=dev) * 2 - 1 for _ in range(k)]
        xs = [b[:, :feat] for b in xb]
        ys = [torch.empty((n, feat), device=dev) for _ in range(k)]
        frame = pipad.frame_build_overlap(gs)
        singles = [pipad.frame_build_overlap([g]) for g in gs]

        def one_by_one():
            for t in range(k):
                pipad.frame_aggregate(singles[t], [xs[t]], [ys[t]])

        t_frame = _time(lambda: pipad.frame_aggregate(frame, xs, ys))
        t_single = _time(one_by_one)
        b_frame = _time(lambda: pipad.frame_build_overlap(gs), 3)
        b_single = _time(lambda: [pipad.frame_build_overlap([g]) for g in gs], 3)
        print(f"| {name} (N = {n}, k = {k}, F = {feat}) | {b_frame:.2f} | {b_single:.2f} | "
              f"{t_frame:.3f} | {t_single:.3f} |", flush=True)
        for f in singles:
            f.close()
        frame.close()
        del xb, xs, ys, gs


def small_f_sweep(dev):
    """The paper's own feature widths (F = 2, 6, 16, Section 5.1) on the benchmark graphs:
    the coalescent kernel (one gather per overlap entry for several snapshots' rows, concatenated
    operand) against the per-snapshot slices on the same operand and on k separate matrices."""
    print("aggregation ms per frame\n")
    print("| graph | F | concatenated operand, coalescent kernel | concatenated operand, slices | "
          "k separate matrices, slices | what the automatic policy picks on the concatenated operand |")
    print("|---|---|---|---|---|---|")
    for name in ("large", "medium", "low-overlap", "small"):
        cfg = synth.CONFIGS[name]
        n, k = cfg.n, cfg.k
        snaps = synth.graphs(n, cfg.edges, k, cfg.churn, cfg.model, cfg.params, cfg.seed)
        gs = [(torch.from_numpy(snaps.rowptr[t]).to(dev), torch.from_numpy(snaps.col[t]).to(dev))
              for t in range(k)]
        frame = pipad.frame_build_overlap(gs)
        for feat in (2, 6, 16):
            xw = torch.rand((n, k, feat), device=dev) * 2 - 1
            yw = torch.empty_like(xw)
            xl = [xw[:, t, :].contiguous() for t in range(k)]
            yl = [torch.empty_like(x) for x in xl]
            pipad.set_option("agg_coalescent", 2)
            t_co = _time(lambda: pipad.frame_aggregate(frame, xw, yw))
            pipad.set_option("agg_coalescent", 0)
            t_ws = _time(lambda: pipad.frame_aggregate(frame, xw, yw))
            t_ls = _time(lambda: pipad.frame_aggregate(frame, xl, yl))
            pipad.set_option("agg_coalescent", 1)
            t_auto = _time(lambda: pipad.frame_aggregate(frame, xw, yw))
            print(f"| {name} | {feat} | {t_co:.3f} | {t_ws:.3f} | {t_ls:.3f} | {t_auto:.3f} |", flush=True)
        frame.close()


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
    elif which == "sliding":
        sliding_sweep(dev)
    elif which == "workloads":
        workload_sweep(dev)
    elif which == "smallf":
        small_f_sweep(dev)
    else:
        print(__doc__, file=sys.stderr)
        return 2
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
