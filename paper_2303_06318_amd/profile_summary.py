"""Turn the raw rocprofv3 output of ONE profiling session into the short summaries under profiles/.

A session is a scratch directory (raw profiler output, never committed) with these sub-directories, each written by
one rocprofv3 run of the committed bench.py (the commands are repeated at the top of the summary this writes):

    kt/     --kernel-trace --stats                       kt_kernel_stats.csv, bench.log   (the only one required)
    fetch/  --pmc FETCH_SIZE   (bench.py --copy-calibration)   f_counter_collection.csv
    write/  --pmc WRITE_SIZE   (bench.py --copy-calibration)   w_counter_collection.csv
    mfma/   --pmc MfmaUtil SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE   m_counter_collection.csv   (optional)

Writes profiles/<name>.md (tables) and updates the line of this workload in profiles/gemm_traffic.txt, the
file bench.py reads roofline.traffic from.  Nothing here runs on the GPU.

    python -m paper_2303_06318_amd.profile_summary <session dir> --workload cfg5_6p7b_tp4_fwdbwd --commit <hash>
"""
from __future__ import annotations

import argparse
import collections
import csv
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
COPY_BYTES = 1 << 30           # bench.py --copy-calibration copies 1 GiB with the runtime's copy kernel

GEMM_NAMES = {
    "<false, true, 1>": "forward GEMM1 + GeLU, GeLU' (A k-contiguous, B n-contiguous)",
    "<false, true, 0>": "forward GEMM2 (A k-contiguous, B n-contiguous)",
    "<false, false, 2>": "dH x GeLU' (both k-contiguous)",
    "<false, false, 0>": "dD (both k-contiguous)",
    "<true, true, 0>": "weight gradients (both output-contiguous), 2 launches per step",
}


def kernel_stats(path):
    rows = list(csv.DictReader(open(path)))
    rows.sort(key=lambda r: -float(r["TotalDurationNs"]))
    return rows


def counters(path):
    """kernel name (+ grid for the copy kernel) -> counter -> list of values, one per dispatch."""
    d = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(path)):
        key = r["Kernel_Name"]
        if "copyBuffer" in key:
            key += " grid=" + r["Grid_Size"]
        d[key][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return d


def mean(v):
    return sum(v) / len(v)


def bench_line(log):
    for line in open(log):
        if line.startswith("{") and '"metric"' in line:
            return json.loads(line)
    return None


def gemm_key(name):
    for k in GEMM_NAMES:
        if "gemm_bf16_kernel" + k in name:
            return k
    return None


def main(argv=None) -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("session")
    ap.add_argument("--workload", required=True)
    ap.add_argument("--commit", required=True, help="the commit the profiled tree was built from")
    ap.add_argument("--out", default=None, help="summary file name under profiles/ (default: layer_<workload>.md)")
    ap.add_argument("--profiles-dir", default=os.path.join(ROOT, "profiles"), help="where the summaries are written")
    ap.add_argument("--bench-args", default="", help="further bench.py arguments the session's runs were made with (e.g. --fused)")
    args = ap.parse_args(argv)
    S = args.session
    wl_args = args.workload + (" " + args.bench_args.strip() if args.bench_args.strip() else "")
    out_md = os.path.join(args.profiles_dir, args.out or "layer_%s.md" % args.workload)
    L = []
    L.append("# rocprofv3 summaries: whole layer step, workload %s\n" % wl_args)
    L.append("Measured at commit %s; every section comes from one run of the committed bench.py, all runs in one session on one box." % args.commit)
    L.append("Commands (from /tmp with TMPDIR=/tmp; R = repository root, S = the session's scratch output directory):\n")
    L.append("    export MOE_TED_SERIAL=1   # kernel trace only: every GEMM on the caller's stream, so durations are those of kernels that have the chip to themselves")
    L.append("    rocprofv3 --kernel-trace --stats -d $S/kt -o kt --output-format csv -- python3 $R/bench.py --workload %s --steps 10 --warmup 3 --no-cpu-baseline --no-isolated" % wl_args)
    L.append("    unset MOE_TED_SERIAL")
    if os.path.isdir(os.path.join(S, "fetch")):
        L.append("    rocprofv3 --pmc FETCH_SIZE -d $S/fetch -o f --output-format csv -- python3 $R/bench.py --workload %s --steps 2 --warmup 1 --no-cpu-baseline --no-isolated --copy-calibration" % wl_args)
    if os.path.isdir(os.path.join(S, "write")):
        L.append("    rocprofv3 --pmc WRITE_SIZE -d $S/write -o w --output-format csv -- python3 $R/bench.py --workload %s --steps 2 --warmup 1 --no-cpu-baseline --no-isolated --copy-calibration" % wl_args)
    if os.path.isdir(os.path.join(S, "mfma")):
        L.append("    rocprofv3 --pmc MfmaUtil SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE -d $S/mfma -o m --output-format csv -- python3 $R/bench.py --workload %s --steps 2 --warmup 1 --no-cpu-baseline --no-isolated" % wl_args)
    L.append("    python3 -m paper_2303_06318_amd.profile_summary $S --workload %s --commit %s%s%s\n" % (
        args.workload, args.commit, " --bench-args='%s'" % args.bench_args.strip() if args.bench_args.strip() else "",
        " --out %s" % args.out if args.out else ""))

    # ---- 1. kernel trace
    stats = kernel_stats(os.path.join(S, "kt", "kt_kernel_stats.csv"))
    L.append("## 1. Kernel trace (13 steps: 3 warm-up + 10 timed; microseconds)\n")
    L.append("| kernel | calls | avg us | min us | max us | % of GPU time |")
    L.append("|---|---|---|---|---|---|")
    g_tot = g_n = 0
    for r in stats:
        L.append("| `%s` | %s | %.1f | %.1f | %.1f | %.2f |" % (r["Name"][:96], r["Calls"], float(r["AverageNs"]) / 1e3,
                                                            float(r["MinNs"]) / 1e3, float(r["MaxNs"]) / 1e3, float(r["Percentage"])))
        if "gemm_bf16_kernel" in r["Name"]:
            g_tot += float(r["TotalDurationNs"])
            g_n += int(r["Calls"])
    b = None
    blog = os.path.join(S, "kt", "bench.log")
    if os.path.exists(blog):
        b = bench_line(blog)
    if g_n:
        L.append("\nAll `gemm_bf16_kernel` instantiations: %d launches, average %.1f us per launch (template arguments: A "
                 "output-contiguous, B n-contiguous, epilogue 0 store / 1 GeLU / 2 times saved GeLU')." % (g_n, g_tot / g_n / 1e3))
    if b:
        rf = b["roofline"]
        L.append("bench.py in the same run (events on the launch stream around the FFN entry points, which also contain the "
                 "plan launches): avg_launch_ms = %s -> %s %s = %.1f %% of %s; ms_per_step = %s (median %s), %s tokens/s." % (
                     rf["avg_launch_ms"], rf["achieved"], rf["unit"], 100 * rf["frac"], rf["peak"], b["ms_per_step"],
                     b.get("ms_per_step_median"), b["value"]))
        L.append("phase_ms = %s" % json.dumps(b["phase_ms"]))
        L.append("routing alone: %s" % json.dumps(b.get("route")))

    # ---- 2. HBM traffic
    fpath, wpath = os.path.join(S, "fetch", "f_counter_collection.csv"), os.path.join(S, "write", "w_counter_collection.csv")
    traffic_avg = None
    if os.path.exists(fpath) and os.path.exists(wpath):
        F, W = counters(fpath), counters(wpath)
        # calibration: the dispatch of the copy kernel with the largest grid moved COPY_BYTES each way
        def calib(D, cname):
            best = None
            for k, v in D.items():
                if "copyBuffer" in k and cname in v:
                    m = max(v[cname])
                    best = m if best is None or m > best else best
            return best
        cf, cw = calib(F, "FETCH_SIZE"), calib(W, "WRITE_SIZE")
        sf = COPY_BYTES / 1024.0 / cf if cf else 1.0
        sw = COPY_BYTES / 1024.0 / cw if cw else 1.0
        L.append("\n## 2. HBM traffic per launch (FETCH_SIZE / WRITE_SIZE in KiB per dispatch, two runs)\n")
        L.append("Calibration: the plain 1 GiB device copy reads FETCH_SIZE = %.0f KiB and WRITE_SIZE = %.0f KiB for 1048576 KiB "
                 "each way, so the counters are scaled by %.3f (fetch) and %.3f (write).\n" % (cf or 0, cw or 0, sf, sw))
        L.append("Last two columns: the kernel's average duration in the kernel trace of section 1 and the counter bytes "
                 "over that duration (as a fraction of 8 TB/s).\n")
        L.append("| kernel | dispatches | FETCH_SIZE KiB | WRITE_SIZE KiB | scaled HBM bytes per launch | avg us | counter GB/s |")
        L.append("|---|---|---|---|---|---|---|")
        dur = {r["Name"]: float(r["AverageNs"]) / 1e3 for r in stats}
        tot_bytes = tot_n = 0
        for k in sorted(F, key=lambda k: -mean(F[k].get("FETCH_SIZE", [0]))):
            if "copyBuffer" in k or "FETCH_SIZE" not in F[k] or k not in W:
                continue
            f, w = mean(F[k]["FETCH_SIZE"]), mean(W[k]["WRITE_SIZE"])
            by = (f * sf + w * sw) * 1024.0
            label = GEMM_NAMES.get(gemm_key(k) or "", None)
            us = dur.get(k)
            rate = "%.1f | %.0f (%.2f)" % (us, by / us / 1e3, by / us / 1e3 / 8000.0) if us else " | "
            L.append("| `%s`%s | %d | %.0f | %.0f | %.3f GB | %s |" % (k[:70], " -- " + label if label else "", len(F[k]["FETCH_SIZE"]), f, w,
                                                                   by / 1e9, rate))
            if "gemm_bf16_kernel" in k:
                n = len(F[k]["FETCH_SIZE"])
                tot_bytes += by * n
                tot_n += n
        if tot_n:
            traffic_avg = tot_bytes / tot_n
            L.append("\nAverage over all GEMM launches of a step: %.3f GB per launch (what bench.py reports as roofline.traffic)." % (traffic_avg / 1e9))

    # ---- 3. MFMA utilisation
    mpath = os.path.join(S, "mfma", "m_counter_collection.csv")
    if os.path.exists(mpath):
        M = counters(mpath)
        L.append("\n## 3. Matrix-core utilisation and LDS (per launch)\n")
        L.append("| GEMM instantiation | MfmaUtil % | SQ_LDS_IDX_ACTIVE | SQ_LDS_BANK_CONFLICT |")
        L.append("|---|---|---|---|")
        for k, v in M.items():
            gk = gemm_key(k)
            if gk:
                L.append("| %s | %.1f | %.0f | %.0f |" % (GEMM_NAMES[gk], mean(v.get("MfmaUtil", [0])), mean(v.get("SQ_LDS_IDX_ACTIVE", [0])),
                                                      mean(v.get("SQ_LDS_BANK_CONFLICT", [0]))))
    open(out_md, "w").write("\n".join(L) + "\n")
    print("wrote", out_md)

    if traffic_avg is not None:
        tpath = os.path.join(args.profiles_dir, "gemm_traffic.txt")
        lines = []
        if os.path.exists(tpath):
            lines = [l.rstrip("\n") for l in open(tpath) if not (l.strip() and not l.startswith("#") and ("workload=%s " % args.workload) in l + " ")]
        if not any(l.startswith("#") for l in lines):
            lines.insert(0, "# HBM bytes per grouped-GEMM launch (average over the launches of a step), from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE scaled by a")
            lines.insert(1, "# plain copy of known size; written by paper_2303_06318_amd/profile_summary.py, read by bench.py (roofline.traffic).")
        lines.append("workload=%s bytes_per_launch=%.0f commit=%s summary=%s" % (args.workload, traffic_avg, args.commit, os.path.basename(out_md)))
        open(tpath, "w").write("\n".join(lines) + "\n")
        print("updated", tpath)
    return 0


if __name__ == "__main__":
    sys.exit(main())
