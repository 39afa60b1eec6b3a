"""bench.py --profile-summary on hand-made rocprofv3 CSVs: the two summaries it writes, the counter
scales it derives from the copy kernel of known size, and that bench.py only trusts a summary taken
with the kernel sources of the tree."""
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402

WORKLOAD = "selftest"  # not a benchmark workload: the files are removed again


def write_csv(path, header, rows):
    os.makedirs(os.path.dirname(path), exist_ok=True)
    with open(path, "w") as f:
        f.write(",".join(header) + "\n")
        for r in rows:
            f.write(",".join(f'"{v}"' for v in r) + "\n")


def test_profile_summary_round_trip(tmp_path):
    agg = "void pipad::(anonymous namespace)::k_aggregate<4, true, 4>(pipad::(anonymous namespace)::AggArgs)"
    fin = "void pipad::(anonymous namespace)::k_split_finish<4, false>(pipad::(anonymous namespace)::AggArgs)"
    cpy = "pipad::(anonymous namespace)::k_stream_copy(HIP_vector_type<float, 4u> const*, HIP_vector_type<float, 4u>*, unsigned long)"
    kt, pf, pw, pl = (str(tmp_path / d) for d in ("kt", "pf", "pw", "pl"))
    write_csv(os.path.join(kt, "x", "bench_kernel_stats.csv"),
              ["Name", "Calls", "TotalDurationNs", "AverageNs", "Percentage", "MinNs", "MaxNs", "StdDev"],
              [[agg, 4, 16000000, 4000000, 80.0, 3900000, 4100000, 1.0],
               [fin, 4, 200000, 50000, 1.0, 49000, 51000, 1.0]])
    cal_kib = bench.CALIBRATION_BYTES // 1024
    head = ["Kernel_Name", "Counter_Name", "Counter_Value"]
    write_csv(os.path.join(pf, "x", "bench_counter_collection.csv"), head,
              [[agg, "FETCH_SIZE", 1000000], [agg, "FETCH_SIZE", 3000000], [fin, "FETCH_SIZE", 1000],
               [cpy, "FETCH_SIZE", cal_kib // 2]])          # the counter reads half of what is read
    write_csv(os.path.join(pw, "x", "bench_counter_collection.csv"), head,
              [[agg, "WRITE_SIZE", 500000], [fin, "WRITE_SIZE", 500], [cpy, "WRITE_SIZE", cal_kib]])
    write_csv(os.path.join(pl, "x", "bench_counter_collection.csv"), head,
              [[agg, "TCC_HIT_sum", 300], [agg, "TCC_MISS_sum", 100], [agg, "TCC_REQ_sum", 400]])
    line = {"steps": 5, "warmup": 1, "ms_per_step": 6.0, "aggregate_ms": 4.05, "build_overlap_ms": 1.5,
            "config": {"n": 10, "k": 8, "F": 64, "fused_update_cols": 0},
            "roofline": {"algorithmic_bytes": 4_000_000_000}}
    made = [os.path.join(ROOT, "profiles", f"bench_{WORKLOAD}_kernel_trace.txt"),
            bench.traffic_profile_path(WORKLOAD)]
    try:
        out = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--profile-summary", kt, pf, pw, pl,
                              "--workload", WORKLOAD], input=json.dumps(line), text=True,
                             capture_output=True, check=True).stdout
        assert "k_aggregate + k_split_finish average per call: 4.050 ms" in out
        text = open(made[1]).read()
        assert "fetch_scale: 2.0000" in text and "write_scale: 1.0000" in text
        assert "l2_hit_rate: 0.750" in text
        # (2,000,000 + 1,000) KiB fetched x 2 + 500,500 KiB written
        want = int(((2001000 * 2.0) + 500500 * 1.0) * 1024)
        got, sha = bench.measured_traffic(WORKLOAD)
        assert sha == bench.kernel_sources_sha() and abs(got - want) <= 1024
        # a summary taken with other kernel sources is not reported
        open(made[1], "w").write(text.replace(f"kernel_sources_sha: {sha}", "kernel_sources_sha: 0123456789abcdef"))
        assert bench.measured_traffic(WORKLOAD) == (None, "0123456789abcdef")
    finally:
        for path in made:
            if os.path.exists(path):
                os.remove(path)


def test_profile_summary_needs_the_calibration_kernel(tmp_path):
    agg = "k_aggregate<4, true, 4>"
    kt, pf, pw, pl = (str(tmp_path / d) for d in ("kt", "pf", "pw", "pl"))
    write_csv(os.path.join(kt, "bench_kernel_stats.csv"),
              ["Name", "Calls", "TotalDurationNs", "AverageNs", "Percentage", "MinNs", "MaxNs", "StdDev"],
              [[agg, 1, 1, 1, 1.0, 1, 1, 0.0]])
    head = ["Kernel_Name", "Counter_Name", "Counter_Value"]
    for d, c in ((pf, "FETCH_SIZE"), (pw, "WRITE_SIZE"), (pl, "TCC_HIT_sum")):
        write_csv(os.path.join(d, "bench_counter_collection.csv"), head, [[agg, c, 1]])
    line = {"steps": 1, "warmup": 0, "ms_per_step": 1.0, "aggregate_ms": 1.0, "build_overlap_ms": 1.0,
            "config": {"n": 1, "k": 1, "F": 1, "fused_update_cols": 0}, "roofline": {"algorithmic_bytes": 1}}
    made = [os.path.join(ROOT, "profiles", f"bench_{WORKLOAD}_kernel_trace.txt"), bench.traffic_profile_path(WORKLOAD)]
    try:
        r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--profile-summary", kt, pf, pw, pl,
                            "--workload", WORKLOAD], input=json.dumps(line), text=True, capture_output=True)
        assert r.returncode != 0 and "calibrate-counters" in r.stderr
        assert not os.path.exists(made[1])
    finally:
        for path in made:
            if os.path.exists(path):
                os.remove(path)
