#!/usr/bin/env python3
"""Benchmark of the frame-parallel GCN aggregation hot path on one MI355X.

One *step* = one pass of the whole hot path over one frame of k snapshots that is already resident
in HBM: ``pipad_frame_build_overlap`` (overlap + exclusive CSRs, D^-1/2) followed by
``pipad_frame_aggregate`` (Y_t = A^_t X_t for all t).  Prints ONE JSON line.

  value      edge.feature updates per second over whole steps (U = F * sum_t (nnz_t + N) per frame)
  roofline   the aggregation kernels against the HBM roofline: algorithmic ("minimal") bytes of one
             aggregate call divided by its duration measured with HIP events on its stream
  cpu_baseline  the CPU oracle timed on this host on a bounded sample of the same frame

Usage: python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload large] [--epochs E] [--cold]
(--epochs E > 1 runs E aggregations per overlap extraction, the way training reuses one frame's
decomposition every epoch; the default 1 keeps the whole path in every step.)

Workloads with more snapshots than a frame holds (small, medium) slide the frame by one snapshot
per step and wrap around (Section 3.3), so the timed steps visit the frames in order.  --cold
writes 1 GiB of scratch between steps (outside the HIP-event brackets), so that no step finds the
previous one's data in the caches; its ms_per_step is the sum of the event-bracketed parts.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E peak
CALIBRATION_BYTES = 1 << 30  # what --calibrate-counters copies (k_stream_copy)


def kernel_sources_sha() -> str:
    """Fingerprint of the HIP sources and headers the library is built from."""
    import hashlib
    h = hashlib.sha256()
    for d in (os.path.join(ROOT, "paper_2301_00391_amd", "csrc"), os.path.join(ROOT, "include")):
        for name in sorted(os.listdir(d)):
            if name.endswith((".hip", ".h")):
                h.update(name.encode())
                h.update(open(os.path.join(d, name), "rb").read())
    return h.hexdigest()[:16]


def traffic_profile_path(workload: str) -> str:
    return os.path.join(ROOT, "profiles", f"k_aggregate_{workload}_l2_miss_traffic.txt")


def measured_traffic(workload: str):
    """Bytes one aggregate call moves between the L2s and the memory side (fabric traffic: HBM or
    the memory-side cache), from the committed rocprofv3 counter summary of this workload:
    FETCH_SIZE / WRITE_SIZE in KiB per dispatch, each scaled by what the same counter reads for a
    plain copy kernel of known size.  Returns (bytes or None, fingerprint of the kernel sources the
    summary was taken with or None): the bytes are only reported when the summary was taken with
    the kernel sources of this tree."""
    path = traffic_profile_path(workload)
    if not os.path.exists(path):
        return None, None
    vals, sha = {}, None
    for line in open(path):
        if line.startswith("kernel_sources_sha:"):
            sha = line.split(":", 1)[1].strip()
        elif ":" in line and not line.startswith("#"):
            key, _, val = line.partition(":")
            try:
                vals[key.strip()] = float(val.split()[0])
            except (ValueError, IndexError):
                pass
    if sha != kernel_sources_sha():
        return None, sha
    try:
        return int((vals["fetch_size_kib"] * vals["fetch_scale"] +
                    vals["write_size_kib"] * vals["write_scale"]) * 1024), sha
    except KeyError:
        return None, sha


def write_traffic_profile(workload: str, dirs, bench_line: dict) -> None:
    """--profile-summary: turns the rocprofv3 CSV output of four runs of this script (kernel trace,
    FETCH_SIZE, WRITE_SIZE, L2 hits/misses; see the command lines it writes into the files) into
    the two short summaries kept under profiles/ for this workload."""
    import csv
    import glob
    import re

    def find(d, name):
        hits = glob.glob(os.path.join(d, "**", name), recursive=True)
        if not hits:
            raise SystemExit(f"no {name} under {d}")
        return hits[0]

    def kname(n):
        m = re.search(r"(k_[a-z_]+)", n)
        return m.group(1) if m else n[:40]

    kt, pf, pw, pl = dirs
    fo = bench_line["config"].get("fused_update_cols", 0)
    args = f"--workload {workload} --steps {bench_line['steps']} --warmup {bench_line['warmup']}"
    if fo:
        args += f" --update {fo}"
    counter_args = args + " --no-cpu --calibrate-counters"  # the counter runs skip the CPU leg
    if "cpu_baseline" not in bench_line:
        args += " --no-cpu"
    tag = f"{workload}_update" if fo else workload
    agg_kernels = ("k_aggregate_update", "k_split_finish") if fo else ("k_aggregate", "k_split_finish")
    head = (f"# bench.py, workload {workload} (N={bench_line['config']['n']}, k={bench_line['config']['k']}, "
            f"F={bench_line['config']['F']}), one MI355X, kernel sources {kernel_sources_sha()}\n")
    rows = list(csv.DictReader(open(find(kt, "bench_kernel_stats.csv"))))
    out = [head.rstrip(),
           f"# command (from the repository root): export TMPDIR=/tmp && rocprofv3 --kernel-trace --stats -d <out> -o bench "
           f"--output-format csv -- python3 bench.py {args}",
           f"# bench.py in the same run: ms_per_step {bench_line['ms_per_step']:.3f}, aggregate_ms (HIP events) "
           f"{bench_line['aggregate_ms']:.3f}, build_overlap_ms {bench_line['build_overlap_ms']:.3f}", "",
           f"{'kernel':28s} {'calls':>6s} {'avg_us':>10s} {'min_us':>10s} {'max_us':>10s} {'total_ms':>10s} {'pct':>6s}"]
    agg_us = 0.0
    for r in rows:
        n = kname(r["Name"])
        if not n.startswith("k_"):
            continue
        out.append(f"{n:28s} {r['Calls']:>6s} {float(r['AverageNs'])/1e3:10.1f} {float(r['MinNs'])/1e3:10.1f} "
                   f"{float(r['MaxNs'])/1e3:10.1f} {float(r['TotalDurationNs'])/1e6:10.2f} {float(r['Percentage']):6.2f}")
        if n in agg_kernels:
            agg_us += float(r["AverageNs"]) / 1e3
    out += ["", f"{agg_kernels[0]} + k_split_finish average per call: {agg_us/1e3:.3f} ms  (HIP-event bracket of "
                f"pipad_frame_aggregate in the same run: {bench_line['aggregate_ms']:.3f} ms)"]
    open(os.path.join(ROOT, "profiles", f"bench_{tag}_kernel_trace.txt"), "w").write("\n".join(out) + "\n")

    def mean_counter(d, counter, kernels=agg_kernels):
        tot = {}
        for r in csv.DictReader(open(find(d, "bench_counter_collection.csv"))):
            n = kname(r["Kernel_Name"])
            if r["Counter_Name"] == counter and n in kernels:
                tot.setdefault(n, []).append(float(r["Counter_Value"]))
        return sum(sum(v) / len(v) for v in tot.values()), max((len(v) for v in tot.values()), default=0)

    f, nf = mean_counter(pf, "FETCH_SIZE")
    w, _ = mean_counter(pw, "WRITE_SIZE")
    hit, _ = mean_counter(pl, "TCC_HIT_sum")
    miss, _ = mean_counter(pl, "TCC_MISS_sum")
    # the same counters on the copy kernel of known size that --calibrate-counters ran in those runs
    cal_kib = CALIBRATION_BYTES / 1024
    cf, ncf = mean_counter(pf, "FETCH_SIZE", ("k_stream_copy",))
    cw, ncw = mean_counter(pw, "WRITE_SIZE", ("k_stream_copy",))
    if not ncf or not ncw:
        raise SystemExit("the counter runs hold no k_stream_copy dispatch: run them with --calibrate-counters")
    fscale, wscale = cal_kib / cf, cal_kib / cw
    tb = (f * fscale + w * wscale) * 1024
    algo = bench_line["roofline"]["algorithmic_bytes"]
    t = [head.rstrip(),
         "# Traffic between the L2s and the memory side (the fabric: served by HBM or by the 256 MB memory-side",
         f"# cache) of one {'pipad_frame_aggregate_update' if fo else 'pipad_frame_aggregate'} call = {agg_kernels[0]} + "
         "k_split_finish; rocprofv3 counters, KiB per dispatch.",
         f"# commands (from the repository root, one run each): export TMPDIR=/tmp && rocprofv3 --pmc FETCH_SIZE -d <out> -o bench "
         f"--output-format csv -- python3 bench.py {counter_args}",
         "#                              ... --pmc WRITE_SIZE ...  |  ... --pmc TCC_HIT_sum TCC_MISS_sum TCC_REQ_sum ...",
         "# summary written by: python3 bench.py --profile-summary <kernel-trace dir> <FETCH dir> <WRITE dir> <L2 dir> "
         f"--workload {workload}  (bench line of the kernel-trace run on stdin)",
         f"# calibration, in the same runs (--calibrate-counters: k_stream_copy, a plain 16-byte-per-lane copy of "
         f"{cal_kib:.0f} KiB",
         f"#   to a separate buffer): FETCH_SIZE read {cf:.0f} KiB for the {cal_kib:.0f} KiB it reads -> scale {fscale:.3f};",
         f"#   WRITE_SIZE read {cw:.0f} KiB for the {cal_kib:.0f} KiB it writes -> scale {wscale:.3f}",
         f"# mean over {nf} dispatches:",
         f"kernel_sources_sha: {kernel_sources_sha()}",
         f"fetch_size_kib: {f:.0f}", f"write_size_kib: {w:.0f}", f"fetch_scale: {fscale:.4f}", f"write_scale: {wscale:.4f}",
         f"l2_hits_per_call: {hit:.4g}", f"l2_misses_per_call: {miss:.4g}",
         f"l2_hit_rate: {hit / max(hit + miss, 1):.3f}",
         f"# => {tb/1e9:.2f} GB per call between L2 and memory side; algorithmic (minimal) bytes of the call "
         f"{algo/1e9:.2f} GB; ratio {tb/algo:.2f}",
         f"# => at aggregate_ms {bench_line['aggregate_ms']:.3f}: {tb/bench_line['aggregate_ms']/1e6:.0f} GB/s of fabric traffic"]
    open(traffic_profile_path(tag), "w").write("\n".join(t) + "\n")
    print("\n".join(out) + "\n\n" + "\n".join(t))


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def _timed(torch, fn, reps):
    """Mean milliseconds of fn() over reps launches on the current stream (one warm-up first)."""
    fn()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        fn()
    b.record()
    b.synchronize()
    return a.elapsed_time(b) / reps


def measure_ceilings(pipad, torch, full: bool):
    """What the memory system of this GPU delivers for the two kinds of traffic the aggregation
    consists of (kernels of include/pipad_ceilings.h): a streaming read, and gathers of feature
    rows in the aggregation kernel's access shape from working sets that fit one L2, the
    memory-side cache, or only HBM.  Returns a dict; ``full`` adds the whole sweep."""
    import ctypes
    lib = pipad.load_library()
    dev = torch.device("cuda:0")
    st = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    sink = torch.empty(lib.pipad_ceiling_sink_floats(), dtype=torch.float32, device=dev)
    res = {}
    src = torch.ones(1 << 29, dtype=torch.float32, device=dev)  # 2 GiB
    ms = _timed(torch, lambda: lib.pipad_ceiling_stream_read(src.data_ptr(), src.numel() * 4,
                                                             sink.data_ptr(), st), 10)
    res["stream_read_GBps"] = src.numel() * 4 / ms / 1e6
    if full:
        dst = torch.empty(1 << 28, dtype=torch.float32, device=dev)  # 1 GiB
        ms = _timed(torch, lambda: lib.pipad_ceiling_stream_copy(src.data_ptr(), dst.data_ptr(),
                                                                 dst.numel() * 4, st), 10)
        res["stream_copy_GBps"] = 2 * dst.numel() * 4 / ms / 1e6  # read + written
        del dst
    count = 1 << 24
    gen = torch.Generator(device="cpu").manual_seed(7)

    def gather(row_floats, stride, ws_bytes, classes):
        rows = max(1, ws_bytes // (stride * 4))
        table = src[: rows * stride]
        if classes:  # section x of the index only touches the x-th eighth of the table
            per = count // classes
            base = (torch.arange(classes).repeat_interleave(per) * (rows // classes))
            idx = (torch.randint(0, max(1, rows // classes), (count,), generator=gen) + base)
        else:
            idx = torch.randint(0, rows, (count,), generator=gen)
        idx = idx.to(torch.int32).to(dev)
        rc = []
        ms = _timed(torch, lambda: rc.append(lib.pipad_ceiling_gather(
            table.data_ptr(), rows, row_floats, stride, idx.data_ptr(), count, classes,
            sink.data_ptr(), st)), 5)
        assert all(r == 0 for r in rc), rc
        return count * row_floats * 4 / ms / 1e6  # GB/s of gathered bytes

    MiB = 1 << 20
    # the three numbers the roofline block uses: 256-byte rows from an L2-, a MALL- and an HBM-sized set
    res["gather_256B_L2_GBps"] = gather(64, 64, 2 * MiB, 0)
    res["gather_256B_MALL_GBps"] = gather(64, 64, 64 * MiB, 0)
    res["gather_256B_HBM_GBps"] = gather(64, 64, 2048 * MiB - 4096, 0)
    if full:
        sweep = []
        for row_floats, stride in ((64, 64), (64, 96), (32, 32)):
            for ws in (1, 2, 3, 4, 6, 8, 12, 16, 24, 32, 64, 128, 256, 1024, 2047):
                for classes in (0, 8):
                    sweep.append({"row_bytes": row_floats * 4, "stride_bytes": stride * 4,
                                  "working_set_MiB": ws, "xcd_classes": classes,
                                  "GBps": gather(row_floats, stride, ws * MiB, classes)})
        res["sweep"] = sweep
    return res


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="large")
    ap.add_argument("--epochs", type=int, default=1, help="aggregations per overlap extraction")
    ap.add_argument("--layout", default="list", choices=["wide", "list"],
                    help="wide: one [N, k, F] coalescent operand; list: k separate [N, F] matrices")
    ap.add_argument("--opt", action="append", default=[], metavar="KEY=VALUE",
                    help="library option set before the frames are built (pipad_set_option), "
                         "e.g. --opt short_max=16 --opt slice_cols=32")
    ap.add_argument("--row-stride", default="auto", choices=["auto", "dense"],
                    help="rows of X: padded to an odd number of 128-byte lines (auto) or F floats")
    ap.add_argument("--update", type=int, default=0, metavar="FO",
                    help="time pipad_frame_aggregate_update (the GCN layer with FO output columns: "
                         "aggregation + fully connected update) instead of the aggregation alone")
    ap.add_argument("--cold", action="store_true", help="flush the caches between steps")
    ap.add_argument("--profile-summary", nargs=4, metavar="DIR",
                    help="no GPU needed: write profiles/bench_<workload>_kernel_trace.txt and "
                         "profiles/k_aggregate_<workload>_l2_miss_traffic.txt from four rocprofv3 output "
                         "directories (kernel trace, FETCH_SIZE, WRITE_SIZE, TCC hit/miss) of this "
                         "script; the bench line of the kernel-trace run is read from stdin")
    ap.add_argument("--calibrate-counters", action="store_true",
                    help="before the timed steps, run the plain copy kernel of include/pipad_ceilings.h "
                         "three times (1 GiB each): a profiler's traffic counters are scaled by what "
                         "they read for it")
    ap.add_argument("--sweep", default=None,
                    choices=["overlap", "features", "sliding", "workloads", "smallf", "rows", "labels", "oracle",
                             "partitions"],
                    help="print one of the sensitivity tables (bench_sweeps.py) instead of the bench line")
    ap.add_argument("--ceilings", action="store_true",
                    help="only measure the streaming and gather ceilings of this GPU (full sweep) "
                         "and print them as one JSON line")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle leg")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="skip the short measurement of the streaming and gather ceilings")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--cpu-threads", type=int, default=0, help="oracle threads (0 = all)")
    args = ap.parse_args()
    if args.profile_summary:
        line = json.loads(sys.stdin.read().strip().splitlines()[-1])
        write_traffic_profile(args.workload, args.profile_summary, line)
        return 0
    if args.sweep:
        import bench_sweeps
        import paper_2301_00391_amd as pipad
        for item in args.opt:  # defaults the sweep's frames are built with (where it sets none itself)
            key, _, val = item.partition("=")
            pipad.set_option(key, int(val))
        return bench_sweeps.main(["bench_sweeps", args.sweep])
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no sharding, no collectives); "
              "use --gpus 1", file=sys.stderr)
        return 2

    import torch

    import synth
    import paper_2301_00391_amd as pipad

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 3
    pipad.load_library()
    if args.ceilings:
        res = measure_ceilings(pipad, torch, full=True)
        log("| row bytes | stride | working set MiB | XCD classes | gathered GB/s |")
        log("|---|---|---|---|---|")
        for r in res["sweep"]:
            log(f"| {r['row_bytes']} | {r['stride_bytes']} | {r['working_set_MiB']} | "
                f"{r['xcd_classes']} | {r['GBps']:.0f} |")
        print(json.dumps(res), flush=True)
        return 0
    options = {}
    for item in args.opt:
        key, _, val = item.partition("=")
        pipad.set_option(key, int(val))
        options[key] = int(val)
    dev = torch.device("cuda:0")
    cfg = synth.CONFIGS[args.workload]
    n, k, F = cfg.n, cfg.k, cfg.feat

    t0 = time.time()
    S, nframes = cfg.snapshots, cfg.frames
    snaps = synth.graphs(n, cfg.edges, S, cfg.churn, cfg.model, cfg.params, cfg.seed)
    log(f"[bench] generated {S} snapshots of {args.workload} in {time.time() - t0:.1f}s")
    t0 = time.time()
    gsnaps = [(torch.from_numpy(snaps.rowptr[t]).to(dev), torch.from_numpy(snaps.col[t]).to(dev))
              for t in range(S)]
    xh0 = None  # host copy of snapshot 0's features, for the CPU leg
    # HBM layout of X: k separate row-major matrices; by default a row starts every odd number of
    # 128-byte lines (the padding is never read), which spreads the gathered rows over the channels
    x_stride = pipad.padded_row_stride(F) if args.row_stride == "auto" else F
    if args.layout == "wide":
        x_stride = k * F
    if args.layout == "wide":
        # one [N, k, F] operand per frame would hold every snapshot k times: the concatenated
        # layout is timed on frame 0 only
        nframes = 1
        xw = torch.empty((n, k, F), dtype=torch.float32, device=dev)
        for t in range(k):
            xt = synth.features(cfg.seed, t, n, F)
            xh0 = xt if t == 0 else xh0
            xw[:, t, :] = torch.from_numpy(xt).to(dev)
        Xs, Ys = None, None
        Yw = torch.empty_like(xw)
    else:
        Xs = []
        for t in range(S):
            xt = synth.features(cfg.seed, t, n, F)
            xh0 = xt if t == 0 else xh0
            buf = torch.zeros((n, x_stride), dtype=torch.float32, device=dev)
            buf[:, :F] = torch.from_numpy(xt).to(dev)
            Xs.append(buf[:, :F])
        Ys = [torch.empty((n, F), dtype=torch.float32, device=dev) for _ in range(k)]
    Fo = args.update
    if Fo:
        if args.layout == "wide":
            print("bench.py: --update is timed on the list layout", file=sys.stderr)
            return 2
        gen = torch.Generator(device="cpu").manual_seed(cfg.seed)
        Wt = (torch.randn((F, Fo), generator=gen) / F ** 0.5).to(dev)
        bt = torch.randn(Fo, generator=gen).to(dev)
        Hs = [torch.empty((n, Fo), dtype=torch.float32, device=dev) for _ in range(k)]
    scratch = torch.empty(1 << 28, dtype=torch.float32, device=dev) if args.cold else None
    if args.calibrate_counters:
        import ctypes
        lib = pipad.load_library()
        a = torch.ones(CALIBRATION_BYTES // 4, dtype=torch.float32, device=dev)
        b = torch.empty_like(a)
        for _ in range(3):
            rc = lib.pipad_ceiling_stream_copy(a.data_ptr(), b.data_ptr(), CALIBRATION_BYTES,
                                               ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
            assert rc == 0, rc
        torch.cuda.synchronize()
        del a, b
    torch.cuda.synchronize()
    log(f"[bench] features and upload in {time.time() - t0:.1f}s")

    nnz_s = [int(snaps.col[t].size) for t in range(S)]

    def frame_inputs(f):
        if args.layout == "wide":
            return gsnaps[:k], xw, Yw
        return gsnaps[f:f + k], Xs[f:f + k], Ys

    stream = torch.cuda.current_stream()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True),
           torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]

    def step(f, events=None):
        g, X, Y = frame_inputs(f)
        if scratch is not None:
            scratch.fill_(1.0)
        if events:
            events[0].record(stream)
        frame = pipad.frame_build_overlap(g)
        if events:
            events[1].record(stream)
        for _ in range(args.epochs):
            if Fo:
                pipad.frame_aggregate_update(frame, X, Wt, bt, H=Hs)
            else:
                pipad.frame_aggregate(frame, X, Y)
        if events:
            events[2].record(stream)
        return frame

    # untimed pass over every frame: sizes of the decompositions (for the algorithmic bytes) and
    # first-touch effects; then the requested warm-up steps
    b_min, upd, nnz_c_f, nnz_d_f = [], [], [], []
    for f in range(nframes):
        frame = step(f)
        nnz_c = int(frame.common()[1].numel())
        nnz_d = [int(frame.delta(t)[1].numel()) for t in range(k)]
        nnz_c_f.append(nnz_c)
        nnz_d_f.append(nnz_d)
        # algorithmic bytes of one aggregate call: X read once, Y written once, every column index
        # of the overlap and exclusive parts once, the row pointers, D^-1/2
        # (with the fused update: H written instead of Y, W and the bias read once)
        out_cols = Fo if Fo else F
        b_min.append(4 * k * n * (F + out_cols) + 4 * (nnz_c + sum(nnz_d)) + 4 * (k + 1) * (n + 1) +
                     4 * k * n + (4 * (F + 1) * Fo if Fo else 0))
        upd.append(F * sum(nnz_s[f + t] + n for t in range(k)))  # per aggregate call
    for w in range(args.warmup):
        frame = step((w - args.warmup) % nframes)
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for s in range(args.steps):
        frame = step(s % nframes, ev[s])
    torch.cuda.synchronize()
    t_end = time.perf_counter()
    build_all = np.array([e[0].elapsed_time(e[1]) for e in ev])
    agg_all = np.array([e[1].elapsed_time(e[2]) for e in ev]) / args.epochs
    build_ms, agg_ms = float(build_all.mean()), float(agg_all.mean())
    if args.cold:
        ms_per_step = build_ms + agg_ms * args.epochs
    else:
        ms_per_step = (t_end - t_start) * 1e3 / args.steps
    visited = [s % nframes for s in range(args.steps)]
    updates = float(np.mean([upd[f] for f in visited]))
    bytes_min = float(np.mean([b_min[f] for f in visited]))
    entries_in = float(np.mean([sum(nnz_s[f:f + k]) for f in visited]))
    achieved = bytes_min / (agg_ms * 1e-3) / 1e9
    value = updates * args.epochs / (ms_per_step * 1e-3)
    nnz_c, nnz_d = nnz_c_f[0], nnz_d_f[0]
    nnz_t = nnz_s[:k]
    # the committed counter summary belongs to the default configuration of the workload
    plain = not (Fo or options or args.row_stride != "auto" or args.layout != "list" or args.epochs != 1)
    traffic, traffic_sha = measured_traffic(args.workload) if plain else (None, None)

    out = {
        "metric": "frame-aggregation edge*feat updates/s (build_overlap + aggregate per frame, k=%d)" % k,
        "value": value,
        "unit": "edge*feat updates/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": args.workload, "n": n, "k": k, "F": F, "model": None,
                   "generator": cfg.model, "edges_per_snapshot": cfg.edges, "churn": cfg.churn,
                   "seed": cfg.seed, "layout": args.layout, "x_row_stride_floats": x_stride,
                   "epochs_per_build": args.epochs, "options": options,
                   "frames": nframes, "fused_update_cols": Fo, "cache": "cold" if args.cold else "as left by the previous step",
                   "nnz_common": nnz_c, "nnz_exclusive": nnz_d,
                   "overlap_rate": nnz_c / (sum(nnz_t) / k)},
        "frames_per_s": 1e3 / ms_per_step,
        "build_overlap_ms": build_ms,
        "build_overlap_ms_median": float(np.median(build_all)),
        "build_input_entries_per_s": entries_in / (build_ms * 1e-3),
        "aggregate_ms": agg_ms,
        "aggregate_ms_median": float(np.median(agg_all)),
        "aggregate_updates_per_s": updates / (agg_ms * 1e-3),
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic,
                     "traffic_kind": "bytes between the L2s and the memory side (HBM or memory-side cache) "
                                     "per aggregate call, from " + os.path.relpath(traffic_profile_path(args.workload), ROOT),
                     "traffic_kernel_sources": traffic_sha, "kernel_sources": kernel_sources_sha(),
                     "kernel": ("pipad_frame_aggregate_update (k_aggregate_update + k_split_finish)" if Fo
                                else "pipad_frame_aggregate (k_aggregate + k_split_finish)"),
                     "algorithmic_bytes": int(bytes_min),
                     # the row gathers themselves: every edge.feat update pulls 4 bytes through the
                     # vector memory path even when the caches serve them all
                     "gather_bytes": int(4 * updates)},
        "paper_context": "PiPAD reports 1.22x-9.57x end-to-end training speedup on a V100 (no absolute "
                         "number for this path)",
    }
    del out["config"]["model"]
    if not args.no_ceilings:
        # what this GPU delivers, measured now with the kernels of include/pipad_ceilings.h: the
        # attainable time of one aggregate call is bounded by its algorithmic bytes at the
        # streaming rate AND by its gathered bytes at the rate of row gathers that all hit the L2
        ceil = measure_ceilings(pipad, torch, full=False)
        roof = out["roofline"]
        roof["stream_read_GBps"] = ceil["stream_read_GBps"]
        roof["gather_peak"] = ceil["gather_256B_L2_GBps"]
        roof["gather_peak_kind"] = "256-byte row gathers, working set resident in one L2, GB/s"
        roof["gather_MALL_GBps"] = ceil["gather_256B_MALL_GBps"]
        roof["gather_HBM_GBps"] = ceil["gather_256B_HBM_GBps"]
        roof["attainable_ms"] = max(bytes_min / ceil["stream_read_GBps"],
                                    4 * updates / ceil["gather_256B_L2_GBps"]) / 1e6
        roof["frac_of_attainable"] = roof["attainable_ms"] / agg_ms

    if not args.no_cpu:
        import oracle
        threads = args.cpu_threads if args.cpu_threads > 0 else oracle.hardware_threads()
        # the last timed step worked on frame `last`: its snapshot 0 is snapshot `last` of the run
        last = visited[-1]
        y_gpu = (Hs[0] if Fo else Yw[:, 0, :] if args.layout == "wide" else Ys[0]).cpu().numpy()
        w_host = Wt.cpu().numpy() if Fo else None
        b_host = bt.cpu().numpy() if Fo else None
        budget = 1e-5 + ((F + 2) * 2.0 ** -24 if Fo else 0.0)
        done, cpu_s, worst = 0, 0.0, 0.0
        for j in range(k):
            t = last + j
            rows, cols = snaps.coo(t)
            xt = xh0 if t == 0 else synth.features(cfg.seed, t, n, F)
            t1 = time.perf_counter()
            if Fo:
                yd, bound = oracle.aggregate_update(n, rows, cols, xt, w_host, b_host, threads=threads)
                used = threads
            else:
                # timed as the plain aggregation: float32 result only
                _, _, _, used = oracle.aggregate(n, rows, cols, xt, threads=threads,
                                                 want_bound=False, want_double=False)
            cpu_s += time.perf_counter() - t1
            done += 1
            if j == 0:  # the sample doubles as an end-to-end parity check of that snapshot (untimed)
                if not Fo:
                    _, yd, bound, _ = oracle.aggregate(n, rows, cols, xt, threads=threads)
                err = np.abs(y_gpu.astype(np.float64) - yd)
                worst = float(np.max(err / np.maximum(bound, 1e-300)))
            if cpu_s >= args.cpu_seconds:
                break
        cpu_updates = F * sum(nnz_s[last + j] + n for j in range(done))
        out["cpu_baseline"] = {"value": cpu_updates / cpu_s, "unit": "edge*feat updates/s",
                               "cores": used, "kind": "oracle",
                               "sample": f"per-snapshot aggregation of snapshots {last}..{last + done - 1} "
                                         f"of the same workload ({cpu_s:.1f} s of oracle time; the oracle "
                                         "works from an edge list, so its time includes sorting and "
                                         "de-duplicating the pairs of every snapshot)"}
        out["parity_first_snapshot_worst_err_over_bound"] = worst
        out["parity_ok"] = bool(worst <= budget)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
