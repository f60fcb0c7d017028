"""Turns rocprofv3 output of a bench.py run into the short summaries kept under profiles/.

    python -m paper_2411_05787_amd.profile_summary trace <workload> <layers> <stats.csv> <bench.json> [<kernel_trace.csv>]
    python -m paper_2411_05787_amd.profile_summary pmc   <workload> <layers> <fetch.csv> <write.csv> <copy_bytes>

`trace` writes profiles/bench_<workload>_kernel_trace.txt from the --kernel-trace --stats csv (and, when
the per-dispatch trace is given, the average over the launches of the roofline measurement, which are
the last ones of the first kernel of a full step).  `pmc` writes profiles/bench_<workload>_pmc.{txt,json}
from the two --pmc passes (FETCH_SIZE, WRITE_SIZE), scaled by what the same counters read for the copy
kernel of known size that every bench.py run launches; bench.py reads the json for `roofline.traffic`.
The git commit the profiled tree was built from is recorded in both.
"""
from __future__ import annotations

import collections
import re
import csv
import json
import os
import statistics as st
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# attn_split_kernel<G, NW, EMIT, TWO_SEG, LAZY, TAGGED, TRIG>: the first kernel of a full step, and the partial step without the trigger inside
FULL_KERNEL = r"attn_split_kernel<\d+, 4, true, false, false, false, false>"
PARTIAL_KERNEL = r"attn_split_kernel<\d+, 4, false, true, false, (true|false), false>"
LEGEND = [
    ("attn_split_kernel<G, 4, true, false, false, false, false>", "streams C_f once and emits raw scores: first kernel of rk_full_attn (weights returned) and rk_full_attn_select; rk_full_attn_scores launches it alone (the roofline measurement)"),
    ("attn_split_kernel<G, 4, true, false, false, true, false>", "the same with the output merged inside (tagged partial results, merge by slices): the one kernel of rk_full_attn_deferred for groups of up to 4 heads"),
    ("attn_split_kernel<G, 4, false, true, false, true, false>", "rk_partial_attn: one launch, tagged partial results, merged by slices (every workgroup its share) or by the last workgroup"),
    ("attn_split_kernel<G, 4, false, true, false, false, false>", "rk_partial_attn, groups of more than 4 heads in launches over many (sequence, KV head) pairs, and rk_partial_attn_static: one launch, ticketed merge"),
    ("attn_split_kernel<G, 4, false, true, false, *, true>", "rk_partial_attn_triggered: the partial step of a trigger test step, with the query-similarity test inside"),
    ("attn_split_kernel<G, 4, false, false, false, true, false>", "rk_full_attn without weights over short rows: one launch, merged inside"),
    ("merge_normalise_kernel", "output merge of rk_full_attn / rk_full_attn_deferred (+ weights in place for rk_full_attn)"),
    ("finish_pool_kernel<G, TILE>", "second kernel of rk_full_attn_select: merge, weights, group max, max-pool, histogram"),
    ("pool_batched_kernel<G>", "pooling tiles of the finishing kernel for all layers in one launch (rk_refresh_batched)"),
    ("select_kernel / select_batched_kernel", "top-K: per call / for all layers in one launch"),
    ("gather_rows_kernel / gather_rows_batched_kernel", "rk_gather_small_kv: per call / for all layers in one launch"),
    ("pool_hist_kernel", "first kernel of rk_topk_select"),
    ("query_sim_kernel", "rk_query_sim"),
    ("score_split_kernel<G>, window_*_kernel, h2o_*_kernel", "rk_score_select, rk_window_select, rk_h2o_step (per-call measurements only)"),
]


def commit_id() -> str:
    try:
        head = subprocess.run(["git", "-C", ROOT, "rev-parse", "--short=12", "HEAD"], capture_output=True, text=True).stdout.strip()
        dirty = subprocess.run(["git", "-C", ROOT, "status", "--porcelain", "--", "paper_2411_05787_amd/csrc", "bench.py"],
                               capture_output=True, text=True).stdout.strip()
        return head + ("+local changes" if dirty else "")
    except Exception:
        return "unknown"


def short(name: str) -> str:
    return name.split("(")[0].replace("void ", "")


def kernel_trace(workload, layers, stats_csv, bench_json, dispatch_csv=None):
    rows = list(csv.DictReader(open(stats_csv)))
    cmd = "rocprofv3 --kernel-trace --stats -d gpurun_out/prof_%s -o bench --output-format csv -- python3 bench.py --workload %s --no-cpu-baseline --no-other-workloads" % (workload, workload)
    out = ["rocprofv3 kernel-trace summary: bench.py, workload %s, %s layers (the workload's own count)" % (workload, layers),
           "tree: commit %s" % commit_id(), "",
           "command (run from /tmp with TMPDIR=/tmp on the MI355X box):", "  " + cmd, "",
           "bench.py JSON line of the same run:", "  " + open(bench_json).read().strip(), "",
           "%-72s %8s %10s %10s %10s %10s" % ("kernel (library kernels only)", "calls", "avg_us", "min_us", "max_us", "total_ms")]
    for r in rows:
        if "rk::" not in r["Name"]:
            continue
        out.append("%-72s %8s %10.2f %10.2f %10.2f %10.2f" % (short(r["Name"]), r["Calls"], float(r["AverageNs"]) / 1e3,
                                                              float(r["MinNs"]) / 1e3, float(r["MaxNs"]) / 1e3,
                                                              float(r["TotalDurationNs"]) / 1e6))
    if dispatch_csv:
        per = collections.defaultdict(list)
        for r in csv.DictReader(open(dispatch_csv)):
            per[short(r["Kernel_Name"])].append((int(r["Start_Timestamp"]), (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3))
        bench = json.loads(open(bench_json).read().strip().splitlines()[-1])
        for key, block in ((FULL_KERNEL, "roofline"), (PARTIAL_KERNEL, "roofline_partial")):
            n = int(bench[block]["launches"])
            for k, v in per.items():
                if re.search(key, k):
                    v.sort()
                    if block == "roofline":
                        last = [d for _, d in v[-n:]]          # the roofline graph replays are the last launches of this kernel
                        out += ["", "last %d dispatches of %s (the timed replays of the roofline graph):" % (len(last), k),
                                "  avg %.2f us, min %.2f, max %.2f   (bench line: %s us per launch by events)" % (
                                    sum(last) / len(last), min(last), max(last), bench[block]["avg_launch_us"])]
                    else:
                        d = [x for _, x in v]
                        out += ["", "%s: all %d dispatches avg %.2f us, median %.2f (bench line: %s us per launch by events)" % (
                            k, len(d), sum(d) / len(d), st.median(d), bench[block]["avg_launch_us"])]
    out += ["", "which kernel is what (G = query heads per KV head):"] + ["  %-52s %s" % (a, b) for a, b in LEGEND]
    path = os.path.join(ROOT, "profiles", "bench_%s_kernel_trace.txt" % workload)
    open(path, "w").write("\n".join(out) + "\n")
    print("wrote", path)


def pmc(workload, layers, fetch_csv, write_csv, copy_bytes):
    def load(path, cname):
        d = collections.defaultdict(list)
        for r in csv.DictReader(open(path)):
            if r["Counter_Name"] == cname:
                d[short(r["Kernel_Name"])].append(float(r["Counter_Value"]))
        return d
    f, w = load(fetch_csv, "FETCH_SIZE"), load(write_csv, "WRITE_SIZE")
    cf, cw = st.median(f["rk::calibration_copy_kernel"]), st.median(w["rk::calibration_copy_kernel"])
    fs, wsc = copy_bytes / 1024 / cf, copy_bytes / 1024 / cw
    base = "python3 bench.py --workload %s --steps 12 --warmup 2 --no-cpu-baseline --no-other-workloads" % workload
    out = ["rocprofv3 --pmc summary: HBM bytes per dispatch of the library kernels in bench.py, workload %s, %s layers" % (workload, layers),
           "tree: commit %s" % commit_id(), "",
           "commands (run from /tmp with TMPDIR=/tmp; one counter per run):",
           "  rocprofv3 --pmc FETCH_SIZE -d gpurun_out/pmc_fetch_%s -o f --output-format csv -- %s" % (workload, base),
           "  rocprofv3 --pmc WRITE_SIZE -d gpurun_out/pmc_write_%s -o w --output-format csv -- %s" % (workload, base), "",
           "calibration: rk::calibration_copy_kernel copies %d bytes (reads them once, writes them once)." % copy_bytes,
           "  FETCH_SIZE reads %.1f KiB for it -> scale %.4f;  WRITE_SIZE reads %.1f KiB -> scale %.4f" % (cf, fs, cw, wsc), "",
           "%-60s %6s %14s %14s %12s %12s" % ("kernel (median over its dispatches)", "n", "FETCH_SIZE KiB", "WRITE_SIZE KiB", "read MB", "written MB")]
    js = {"workload": workload, "layers": int(layers), "commit": commit_id(), "fetch_scale": fs, "write_scale": wsc, "copy_bytes": copy_bytes}
    for k in f:
        if "rk::" not in k:
            continue
        a, b = st.median(f[k]), st.median(w.get(k, [0.0]))
        out.append("%-60s %6d %14.1f %14.1f %12.2f %12.2f" % (k[-60:], len(f[k]), a, b, a * 1024 * fs / 1e6, b * 1024 * wsc / 1e6))
        if re.search(FULL_KERNEL, k):
            js["attn_split"] = {"kernel": k, "fetch_kib": a, "write_kib": b}
        if re.search(PARTIAL_KERNEL, k) and len(f[k]) > js.get("partial_attn", {}).get("dispatches", 0):
            # (both hand-overs can be in one run: the comparison policies' short caches take the tagged one; the bench's own
            # partial steps are the form with the most dispatches)
            js["partial_attn"] = {"kernel": k, "fetch_kib": a, "write_kib": b, "dispatches": len(f[k])}
    out += ["", "(a kernel launched with several shapes in one run, e.g. the first kernel of a full step over the policy runs'",
            " short caches, shows the median shape; the bench's own shape dominates the dispatch counts above)"]
    open(os.path.join(ROOT, "profiles", "bench_%s_pmc.txt" % workload), "w").write("\n".join(out) + "\n")
    json.dump(js, open(os.path.join(ROOT, "profiles", "bench_%s_pmc.json" % workload), "w"), indent=1)
    print("wrote profiles/bench_%s_pmc.{txt,json}" % workload)


if __name__ == "__main__":
    what = sys.argv[1]
    if what == "trace":
        kernel_trace(sys.argv[2], sys.argv[3], sys.argv[4], sys.argv[5], sys.argv[6] if len(sys.argv) > 6 else None)
    elif what == "pmc":
        pmc(sys.argv[2], sys.argv[3], sys.argv[4], sys.argv[5], int(sys.argv[6]))
    else:
        raise SystemExit(__doc__)
