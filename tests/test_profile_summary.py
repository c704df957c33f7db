"""Host logic of the profile summariser: from the CSV files rocprofv3 writes (here: three hand-made ones of a few
rows) to the tables under profiles/ and the line bench.py reads the GEMM's measured HBM traffic from."""
import os

from paper_2303_06318_amd import profile_summary

GEMM = "void moe::gemm_bf16_kernel<false, true, 0>(moe::GemmDesc)"
COPY = "__amd_rocclr_copyBuffer"


def write(path, header, rows):
    os.makedirs(os.path.dirname(path), exist_ok=True)
    with open(path, "w") as f:
        f.write(",".join('"%s"' % h for h in header) + "\n")
        for r in rows:
            f.write(",".join('"%s"' % v for v in r) + "\n")


def test_summary_tables_and_traffic_line(tmp_path):
    S = tmp_path / "session"
    write(str(S / "kt" / "kt_kernel_stats.csv"),
          ["Name", "Calls", "TotalDurationNs", "AverageNs", "Percentage", "MinNs", "MaxNs", "StdDev"],
          [[GEMM, 4, 2000000, 500000, 90.0, 480000, 520000, 1.0], ["moe::dispatch_kernel(int)", 2, 80000, 40000, 10.0, 39000, 41000, 1.0]])
    cols = ["Kernel_Name", "Grid_Size", "Counter_Name", "Counter_Value"]
    # the 1 GiB copy reads back as 524288 KiB fetched (the counter counts half) and 1048576 KiB written
    write(str(S / "fetch" / "f_counter_collection.csv"), cols,
          [[COPY, 1 << 20, "FETCH_SIZE", 524288], [COPY, 64, "FETCH_SIZE", 1], [GEMM, 65536, "FETCH_SIZE", 400000],
           [GEMM, 65536, "FETCH_SIZE", 420000]])
    write(str(S / "write" / "w_counter_collection.csv"), cols,
          [[COPY, 1 << 20, "WRITE_SIZE", 1048576], [GEMM, 65536, "WRITE_SIZE", 131072], [GEMM, 65536, "WRITE_SIZE", 131072]])
    out = tmp_path / "profiles"
    os.makedirs(out)
    (out / "gemm_traffic.txt").write_text("# header\nworkload=other bytes_per_launch=1 commit=x summary=y\n"
                                          "workload=wl bytes_per_launch=2 commit=old summary=z\n")
    rc = profile_summary.main([str(S), "--workload", "wl", "--commit", "abc1234", "--profiles-dir", str(out)])
    assert rc == 0
    md = (out / "layer_wl.md").read_text()
    assert "abc1234" in md and "rocprofv3 --kernel-trace --stats" in md
    assert "| `%s` | 4 | 500.0 | 480.0 | 520.0 | 90.00 |" % GEMM in md
    assert "scaled by 2.000 (fetch) and 1.000 (write)" in md
    # (410000 KiB x 2 + 131072 KiB) x 1024 B = 0.974 GB per launch, over 500 us
    want = (410000 * 2 + 131072) * 1024
    assert "%.3f GB" % (want / 1e9) in md and "500.0 | %.0f" % (want / 500.0 / 1e3) in md
    # no counters without their directory: the MFMA section is absent, and so is its command
    assert "MfmaUtil" not in md
    lines = (out / "gemm_traffic.txt").read_text().splitlines()
    assert "workload=other bytes_per_launch=1 commit=x summary=y" in lines          # other workloads' lines stay
    assert not any("commit=old" in l for l in lines)                                    # this workload's line is replaced
    assert "workload=wl bytes_per_launch=%d commit=abc1234 summary=layer_wl.md" % want in lines


def test_bench_reads_the_committed_traffic_line():
    """bench.py takes roofline.traffic from the committed profiles/gemm_traffic.txt: the headline workload has a line,
    with the commit it was measured at, and the figure lies between the algorithmic bytes of a launch and three
    times as much; a workload without a line gives None (the field is then null)."""
    import bench
    v, commit = bench.measured_gemm_traffic("cfg5_6p7b_tp4_fwdbwd")
    assert commit and len(commit) >= 7
    algorithmic = 16 * 4096 * 4096 * 2 + 16384 * (4096 + 4096) * 2
    assert algorithmic <= v <= 3 * algorithmic
    assert bench.measured_gemm_traffic("no_such_workload") == (None, None)
