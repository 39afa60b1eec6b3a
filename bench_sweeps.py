"""Sensitivity sweeps of the frame-parallel aggregation on synthetic frames (needs a GPU).

Analogues of the paper's offline analysis of its parallel GNN (Section 4.4, Fig. 9: speedup of
S_per in {2, 4, 8} snapshots per partition over one-snapshot execution, against overlap rate and
against the feature dimension) and of its dimension-sensitivity test (Section 5.3, Fig. 11b),
on the synthetic generator instead of the paper's datasets.

  python bench.py --sweep overlap    # churn x k table
  python bench.py --sweep features   # F x k table
  python bench.py --sweep sliding    # cost per new snapshot when the frame slides by one
  python bench.py --sweep workloads  # the benchmark frames: one frame vs one snapshot at a time
  python bench.py --sweep smallf     # F = 2 / 6 / 16: the coalescent kernel vs per-snapshot slices
  python bench.py --sweep rows       # row-length classes: thresholds of the three kinds of work items
  python bench.py --sweep labels     # the large frame with its nodes relabelled (locality sensitivity)
  python bench.py --sweep oracle     # the CPU oracle on one thread and on all threads
  python bench.py --sweep partitions # a group of 8 snapshots as 8 / S_per frames of S_per: the tuner's table

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
    # k separate matrices (the layout the per-snapshot slices prefer)
    xw = torch.rand((n, k, feat), device=dev) * 2 - 1
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
    print("cost per new snapshot in ms, stride-1 frames: build_overlap + aggregate for the first three "
          "columns; extraction only for the last two\n")
    print("| workload | whole frame again | whole extraction, aggregation of the entering snapshot "
          "(pipad_frame_aggregate_subset) | entering snapshot alone as a frame of one | "
          "disjoint groups of k, per snapshot | extraction of the whole frame | "
          "lower bound of an incremental extraction |")
    print("|---|---|---|---|---|---|---|")
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

        def subset():
            for f in range(cfg.frames):
                fr = pipad.frame_build_overlap(gs[f:f + k])
                pipad.frame_aggregate_subset(fr, [k - 1], [None] * (k - 1) + [xs[f + k - 1]],
                                             [None] * (k - 1) + [ys[f + k - 1]])

        def entering():
            for f in range(cfg.frames):
                t = f + k - 1
                fr = pipad.frame_build_overlap(gs[t:t + 1])
                pipad.frame_aggregate(fr, xs[t:t + 1], ys[t:t + 1])

        def groups():
            for g in range(cfg.snapshots // k):
                fr = pipad.frame_build_overlap(gs[g * k:(g + 1) * k])
                pipad.frame_aggregate(fr, xs[g * k:(g + 1) * k], ys[g * k:(g + 1) * k])

        # An incremental extraction (Section 3.3 reuse applied to the topology): the k - 1 kept
        # snapshots share M = C + R, R = the entries missing only from the leaving snapshot, and
        # the next frame follows from one split of M against the entering snapshot.  Its first two
        # steps can be run with the existing call: (1) R and the exclusive parts without R =
        # extraction over the k - 1 kept exclusive parts; (2) the split of M (here: C, a few
        # entries fewer) against the entering snapshot = extraction of a frame of two.  The merges
        # that turn the pieces back into canonical parts come on top, so this is a lower bound.
        def build_only():
            for f in range(cfg.frames):
                pipad.frame_build_overlap(gs[f:f + k])

        frames0 = [pipad.frame_build_overlap(gs[f:f + k]) for f in range(cfg.frames - 1)]
        parts = [([fr.delta(t) for t in range(1, k)], fr.common()) for fr in frames0]

        def incremental():
            for f, (deltas, common) in enumerate(parts):
                pipad.frame_build_overlap(deltas)
                pipad.frame_build_overlap([common, gs[f + k]])

        t_whole = _time(whole, 3) / cfg.frames
        t_subset = _time(subset, 3) / cfg.frames
        t_enter = _time(entering, 3) / cfg.frames
        t_group = _time(groups, 3) / (cfg.snapshots // k * k)
        t_build = _time(build_only, 3) / cfg.frames
        t_incr = _time(incremental, 3) / len(parts)
        print(f"| {name} (N = {n}, k = {k}, F = {feat}, {cfg.frames} frames) | {t_whole:.3f} | "
              f"{t_subset:.3f} | {t_enter:.3f} | {t_group:.3f} | {t_build:.3f} | {t_incr:.3f} |", flush=True)
        for fr in frames0:
            fr.close()


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
        # a frame keeps the options it was built with: one frame per setting of agg_coalescent
        frames = {}
        for mode in (2, 0, 1):
            pipad.set_option("agg_coalescent", mode)
            frames[mode] = pipad.frame_build_overlap(gs)
        for feat in (2, 6, 16):
            xw = torch.rand((n, k, feat), device=dev) * 2 - 1
            yw = torch.empty_like(xw)
            xl = [xw[:, t, :].contiguous() for t in range(k)]
            yl = [torch.empty_like(x) for x in xl]
            t_co = _time(lambda: pipad.frame_aggregate(frames[2], xw, yw))
            t_ws = _time(lambda: pipad.frame_aggregate(frames[0], xw, yw))
            t_ls = _time(lambda: pipad.frame_aggregate(frames[0], xl, yl))
            t_auto = _time(lambda: pipad.frame_aggregate(frames[1], xw, yw))
            print(f"| {name} | {feat} | {t_co:.3f} | {t_ws:.3f} | {t_ls:.3f} | {t_auto:.3f} |", flush=True)
        for fr in frames.values():
            fr.close()


def row_class_sweep(dev):
    """Load balance by row length (the job of the paper's sliced CSR, Section 4.1 / 5.4): the
    thresholds between the three kinds of work items on the large frame."""
    cfg = synth.CONFIGS["large"]
    n, k, feat = cfg.n, cfg.k, cfg.feat
    snaps = synth.graphs(n, cfg.edges, k, cfg.churn, cfg.model, cfg.params, cfg.seed)
    gs = [(torch.from_numpy(snaps.rowptr[t]).to(dev), torch.from_numpy(snaps.col[t]).to(dev))
          for t in range(k)]
    stride = pipad.padded_row_stride(feat)
    xb = [torch.rand((n, stride), device=dev) * 2 - 1 for _ in range(k)]
    xs = [b[:, :feat] for b in xb]
    ys = [torch.empty((n, feat), device=dev) for _ in range(k)]
    defaults = {key: pipad.get_option(key) for key in
                ("short_max", "mid_max", "hub_threshold", "hub_segment", "sub_classes")}
    print("large frame (N = 1M R-MAT, k = 8, F = 64), ms per call\n")
    print("| short_max | mid_max | hub_threshold = hub_segment | sub_classes | extraction | aggregation |")
    print("|---|---|---|---|---|---|")
    rows = [dict(), dict(short_max=32), dict(short_max=128), dict(mid_max=256), dict(mid_max=1024),
            dict(mid_max=2048), dict(hub_threshold=8192, hub_segment=8192),
            dict(hub_threshold=1 << 30, hub_segment=1 << 30), dict(sub_classes=2), dict(sub_classes=4),
            dict(mid_max=1 << 30)]
    for change in rows:
        opts = dict(defaults, **change)
        for key, val in opts.items():
            pipad.set_option(key, val)
        t_build = _time(lambda: pipad.frame_build_overlap(gs), 3)
        frame = pipad.frame_build_overlap(gs)
        t_agg = _time(lambda: pipad.frame_aggregate(frame, xs, ys))
        frame.close()
        seg = "never cut" if opts["hub_threshold"] >= 1 << 30 else str(opts["hub_threshold"])
        mid = "all rows whole (no column classes)" if opts["mid_max"] >= 1 << 30 else str(opts["mid_max"])
        print(f"| {opts['short_max']} | {mid} | {seg} | {opts['sub_classes']} | {t_build:.3f} | {t_agg:.3f} |",
              flush=True)
    for key, val in defaults.items():
        pipad.set_option(key, val)


def label_sweep(dev):
    """Locality sensitivity: the large frame with its nodes relabelled (graph and features permuted
    together, so the result is the same up to the permutation)."""
    cfg = synth.CONFIGS["large"]
    n, k, feat = cfg.n, cfg.k, cfg.feat
    snaps = synth.graphs(n, cfg.edges, k, cfg.churn, cfg.model, cfg.params, cfg.seed)
    deg = np.diff(snaps.rowptr[0])
    rng = np.random.default_rng(0)
    perms = {"natural ids (R-MAT: popularity tied to the id's bits)": None,
             "random ids": rng.permutation(n).astype(np.int64),
             "ids sorted by degree (hubs first)": np.argsort(np.argsort(-deg, kind="stable"), kind="stable"),
             # neighbours in memory stay neighbours; only the order inside every 256 ids changes
             "ids sorted by degree within aligned blocks of 256":
                 np.argsort(np.lexsort((-deg, np.arange(n) // 256)), kind="stable"),
             "ids sorted by degree within aligned blocks of 4096":
                 np.argsort(np.lexsort((-deg, np.arange(n) // 4096)), kind="stable")}
    stride = pipad.padded_row_stride(feat)
    print("large frame (N = 1M R-MAT, k = 8, F = 64), aggregation ms per call\n")
    print("| node labels | rows of X padded (stride 96 floats) | rows of X dense (stride 64) |")
    print("|---|---|---|")
    for label, new_id in perms.items():
        gs = []
        for t in range(k):
            rp, col = snaps.rowptr[t], snaps.col[t]
            if new_id is not None:  # entry (i, j) -> (new_id[i], new_id[j]), rows and columns re-sorted
                rows = np.repeat(np.arange(n, dtype=np.int64), np.diff(rp))
                r2, c2 = new_id[rows], new_id[col]
                order = np.lexsort((c2, r2))
                rp = np.concatenate([[0], np.cumsum(np.bincount(r2, minlength=n))]).astype(np.int32)
                col = c2[order].astype(np.int32)
            gs.append((torch.from_numpy(np.ascontiguousarray(rp)).to(dev),
                       torch.from_numpy(np.ascontiguousarray(col)).to(dev)))
        frame = pipad.frame_build_overlap(gs)
        cells = []
        for st in (stride, feat):
            xb = [torch.rand((n, st), device=dev) * 2 - 1 for _ in range(k)]
            xs = [b[:, :feat] for b in xb]
            ys = [torch.empty((n, feat), device=dev) for _ in range(k)]
            cells.append(_time(lambda: pipad.frame_aggregate(frame, xs, ys)))
            del xb, xs, ys
        frame.close()
        print(f"| {label} | {cells[0]:.3f} | {cells[1]:.3f} |", flush=True)


def partition_sweep(dev):
    """The decision the paper's tuner takes (Section 4.4): how many snapshots S_per of a group
    share one overlap part.  A group of 8 snapshots is processed as 8 / S_per frames of S_per
    snapshots each; one cell = aggregation ms for the 8 snapshots [+ extraction ms for them],
    the best S_per of the row marked."""
    n, edges = 200_000, 1_600_000
    print(f"Chung-Lu gamma 2.1, N = {n}, {edges} undirected edges per snapshot, 8 snapshots; cell = "
          "aggregation ms + extraction ms for all 8 snapshots (concatenated operand for F < 32)\n")
    print("| churn per step | F | " + " | ".join(f"S_per = {sp}" for sp in (1, 2, 4, 8)) + " | best by aggregation | best with extraction |")
    print("|---|---|---|---|---|---|---|---|")
    for churn in (0.01, 0.10, 0.40):
        snaps = synth.graphs(n, edges, 8, churn, "chung-lu", (2.1, 16.0), seed=2)
        gs = [(torch.from_numpy(snaps.rowptr[t]).to(dev), torch.from_numpy(snaps.col[t]).to(dev))
              for t in range(8)]
        for feat in (2, 16, 64):
            cells, agg, tot = [], [], []
            for sp in (1, 2, 4, 8):
                groups = [gs[i:i + sp] for i in range(0, 8, sp)]
                t_build = min(_time(lambda: [pipad.frame_build_overlap(g).close() for g in groups], reps=1)
                              for _ in range(3))
                frames = [pipad.frame_build_overlap(g) for g in groups]
                if feat < 32:
                    xs = [torch.rand((n, sp, feat), device=dev) * 2 - 1 for _ in groups]
                else:
                    xs = [[torch.rand((n, feat), device=dev) * 2 - 1 for _ in range(sp)] for _ in groups]
                ys = [torch.empty_like(x) if feat < 32 else [torch.empty_like(v) for v in x] for x in xs]

                def run():
                    for f, x, y in zip(frames, xs, ys):
                        pipad.frame_aggregate(f, x, y)
                t_agg = _time(run)
                for f in frames:
                    f.close()
                cells.append(f"{t_agg:.3f} + {t_build:.3f}")
                agg.append(t_agg)
                tot.append(t_agg + t_build)
                del xs, ys
            sps = (1, 2, 4, 8)
            print(f"| {churn:.0%} | {feat} | " + " | ".join(cells) +
                  f" | {sps[int(np.argmin(agg))]} | {sps[int(np.argmin(tot))]} |", flush=True)


def oracle_sweep(dev):
    """The CPU oracle (plain per-snapshot aggregation in double, never tuned) on this host: one
    thread and all hardware threads, one snapshot of every benchmark frame."""
    import time

    import oracle
    print("CPU oracle, one snapshot, seconds and edge*feat updates per second\n")
    print("| workload | threads | seconds | updates/s |")
    print("|---|---|---|---|")
    for name in ("medium", "large", "low-overlap"):
        cfg = synth.CONFIGS[name]
        snaps = synth.graphs(cfg.n, cfg.edges, 1, cfg.churn, cfg.model, cfg.params, cfg.seed)
        rows, cols = snaps.coo(0)
        x = synth.features(cfg.seed, 0, cfg.n, cfg.feat)
        upd = cfg.feat * (cols.size + cfg.n)
        for threads in (1, oracle.hardware_threads()):
            t0 = time.perf_counter()
            _, _, _, used = oracle.aggregate(cfg.n, rows, cols, x, threads=threads,
                                             want_bound=False, want_double=False)
            dt = time.perf_counter() - t0
            print(f"| {name} | {used} | {dt:.2f} | {upd / dt:.3g} |", flush=True)


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
    elif which == "rows":
        row_class_sweep(dev)
    elif which == "labels":
        label_sweep(dev)
    elif which == "oracle":
        oracle_sweep(dev)
    elif which == "partitions":
        partition_sweep(dev)
    else:
        print(__doc__, file=sys.stderr)
        return 2
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
