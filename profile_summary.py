#!/usr/bin/env python3
"""Turns the rocprofv3 output of four (or five) runs of bench.py on one workload into the short text summaries under profiles/
and into the entry of profiles/hbm_traffic.json that bench.py reads for `roofline.traffic`.

The four runs (each from /tmp on the MI355X machine, `export TMPDIR=/tmp` first; R = the repository, O = an output folder,
W = the workload arguments, e.g. `--workload vgg16_fc` or `--workload vgg16_conv4 --conv-split batch`):

  rocprofv3 --kernel-trace --stats --output-format csv -d O/kt -o run -- python3 R/bench.py W --steps 20 --warmup 3 \\
      --headline-only --no-cpu-baseline --launch-log O/launches.json
  rocprofv3 --pmc FETCH_SIZE --output-format csv -d O/fetch -o run -- python3 R/bench.py W --steps 2 --warmup 1 \\
      --no-graph --headline-only --no-cpu-baseline
  rocprofv3 --pmc WRITE_SIZE --output-format csv -d O/write -o run -- python3 R/bench.py W (same arguments)
  rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CU_CYCLES --output-format csv -d O/mfma -o run -- python3 R/bench.py W (same)
  (optional) rocprofv3 --pmc SQ_WAVE_CYCLES SQ_WAIT_ANY SQ_WAIT_INST_ANY SQ_WAIT_INST_LDS SQ_ACTIVE_INST_LDS SQ_ACTIVE_INST_VMEM \\
      --output-format csv -d O/sq -o run -- python3 R/bench.py W (same)

then, anywhere:   python3 profile_summary.py O

How dispatches are told apart: bench.py launches the same kernels in the same order every step, and after its last step
53 retiles of the workload's largest tensor.  launches.json lists the launches of one step in order (kernel class, shape,
algorithmic bytes and flops, as the library's own profiling hooks record them); the library's dispatches in a profiler
file, in dispatch order, are therefore steps x that list followed by the 53 retiles.  The retiles copy a known number of
bytes, which calibrates the two traffic counters.
"""
import csv
import glob
import json
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
PROFILES = os.path.join(ROOT, "profiles")
N_RETILE = 53                # 3 warm-up + 50 timed retile launches at the end of bench.py
PEAK_TFLOPS, PEAK_GBS = 2500.0, 8000.0


def one(pattern):
    hits = sorted(glob.glob(pattern, recursive=True))
    if not hits:
        raise SystemExit("no file matches %s" % pattern)
    return hits[0]


def library_dispatches(path, order_key):
    """rows of the library's own kernels (namespace tt), in dispatch order"""
    rows = [r for r in csv.DictReader(open(path)) if "tt::" in r["Kernel_Name"]]
    rows.sort(key=lambda r: int(r[order_key]))
    return rows


# kernels the library launches inside another launch's profiling record (the filter flip in front of the convolution
# data gradient): their time and counters are added to the dispatch that follows
HELPERS = ("filter_flip",)


def per_launch(rows, n, value):
    """average of value(row) per position in the step, over all steps; the trailing retiles separately"""
    folded, carry = [], 0.0
    for r in rows:
        if any(h in r["Kernel_Name"] for h in HELPERS):
            carry += value(r)
            continue
        folded.append((r, value(r) + carry))
        carry = 0.0
    values = {id(r): v for r, v in folded}
    rows = [r for r, _ in folded]
    value = lambda r: values[id(r)]
    body, tail = rows[:-N_RETILE], rows[-N_RETILE:]
    if len(body) % n:
        raise SystemExit("%d library dispatches before the retiles: no multiple of the %d launches of a step" % (len(body), n))
    steps = len(body) // n
    out = []
    for i in range(n):
        vals = [value(body[s * n + i]) for s in range(steps)]
        out.append(sum(vals) / len(vals))
    names = [body[i]["Kernel_Name"] for i in range(n)]
    rt = [value(r) for r in tail]
    return out, names, sum(rt) / len(rt), steps


def short(name):
    return name.replace("tt::(anonymous namespace)::", "").replace("void ", "").replace("tt::", "")[:84]


def counters(path, n):
    """{counter: (per-launch averages, retile average)} of one --pmc run"""
    rows = library_dispatches(path, "Dispatch_Id")
    by_counter = {}
    for r in rows:
        by_counter.setdefault(r["Counter_Name"], []).append(r)
    out = {}
    for c, rs in by_counter.items():
        vals, _, rt, _ = per_launch(rs, n, lambda r: float(r["Counter_Value"]))
        out[c] = (vals, rt)
    return out


def main():
    if len(sys.argv) != 2:
        raise SystemExit(__doc__)
    O = sys.argv[1]
    log = json.load(open(os.path.join(O, "launches.json")))
    wl, launches = log["workload"], log["launches"]
    n = len(launches)
    os.makedirs(PROFILES, exist_ok=True)

    def key(rec):
        return "%s count=%d %dx%dx%d" % (rec["kernel"], rec["count"], rec["d0"], rec["d1"], rec["d2"])

    # ---- kernel trace
    kt = library_dispatches(one(os.path.join(O, "kt", "**", "*kernel_trace.csv")), "Start_Timestamp")
    dur, names, rt_us, steps = per_launch(kt, n, lambda r: (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    with open(os.path.join(PROFILES, "%s_step_kernel_trace.txt" % wl), "w") as f:
        f.write("# rocprofv3 --kernel-trace --stats of one benchmark run of workload %s (command: see profile_summary.py);\n"
                "# average duration of every launch of a step over %d steps (warm-up, graph replays and the eager pass),\n"
                "# in launch order; rates from the launch's algorithmic bytes and flops.\n" % (wl, steps))
        f.write("%-3s %-44s %-84s %10s %9s %9s\n" % ("#", "launch", "kernel", "avg_us", "TFLOP/s", "GB/s"))
        for i, rec in enumerate(launches):
            tf = rec["flops"] / (dur[i] * 1e-6) / 1e12 if rec["flops"] else 0.0
            gb = rec["bytes"] / (dur[i] * 1e-6) / 1e9
            f.write("%-3d %-44s %-84s %10.2f %9.1f %9.0f\n" % (i, key(rec), short(names[i]), dur[i], tf, gb))
        f.write("# step total %.1f us in %d launches; retile of the largest tensor %.2f us\n" % (sum(dur), n, rt_us))
        stats = one(os.path.join(O, "kt", "**", "*kernel_stats.csv"))
        f.write("\n# per kernel template over the whole run (rocprofv3 --stats)\n%-100s %7s %12s %10s %6s\n" % (
            "kernel", "calls", "total_us", "avg_us", "pct"))
        for r in csv.DictReader(open(stats)):
            if "tt::" in r["Name"]:
                f.write("%-100s %7s %12.1f %10.2f %6s\n" % (short(r["Name"])[:100], r["Calls"], float(r["TotalDurationNs"]) / 1e3,
                                                            float(r["AverageNs"]) / 1e3, r["Percentage"]))

    # ---- HBM traffic
    fetch = counters(one(os.path.join(O, "fetch", "**", "*counter_collection.csv")), n)["FETCH_SIZE"]
    write = counters(one(os.path.join(O, "write", "**", "*counter_collection.csv")), n)["WRITE_SIZE"]
    # the retile reads and writes rows x cols x element bytes: take them from the retile's own record at the end of the log
    rt_bytes = float(log["retile_bytes_each_way"])
    fs, ws = rt_bytes / 1024.0 / fetch[1], rt_bytes / 1024.0 / write[1]
    table = {}
    with open(os.path.join(PROFILES, "%s_step_hbm_traffic_pmc.txt" % wl), "w") as f:
        f.write("# HBM traffic per launch of workload %s from two rocprofv3 --pmc runs (FETCH_SIZE, then WRITE_SIZE; eager\n"
                "# launches; commands: see profile_summary.py).  Calibration: a retile of the largest tensor copies %.0f KiB each\n"
                "# way and reads FETCH_SIZE = %.1f, WRITE_SIZE = %.1f per dispatch: FETCH_SIZE x %.5f and WRITE_SIZE x %.5f give KiB.\n"
                % (wl, rt_bytes / 1024.0, fetch[1], write[1], fs, ws))
        f.write("%-3s %-44s %12s %12s %10s %10s %12s %8s\n" % ("#", "launch", "FETCH_SIZE", "WRITE_SIZE", "read_MB", "write_MB",
                                                               "algorithm_MB", "ratio"))
        for i, rec in enumerate(launches):
            rb, wb = fetch[0][i] * fs * 1024.0, write[0][i] * ws * 1024.0
            f.write("%-3d %-44s %12.1f %12.1f %10.2f %10.2f %12.2f %8.3f\n" % (
                i, key(rec), fetch[0][i], write[0][i], rb / 1e6, wb / 1e6, rec["bytes"] / 1e6, (rb + wb) / max(rec["bytes"], 1)))
            e = table.setdefault(key(rec), {"read_bytes": 0.0, "write_bytes": 0.0, "algorithmic_bytes": rec["bytes"], "launches": 0})
            e["read_bytes"] += rb
            e["write_bytes"] += wb
            e["launches"] += 1
    for e in table.values():            # launches of one shape within a step: their average
        e["read_bytes"] = round(e["read_bytes"] / e["launches"])
        e["write_bytes"] = round(e["write_bytes"] / e["launches"])
    tf = os.path.join(PROFILES, "hbm_traffic.json")
    try:
        whole = json.load(open(tf))
    except (OSError, ValueError):
        whole = {}
    whole[wl] = {"source": "%s_step_hbm_traffic_pmc.txt" % wl, "fetch_scale_KiB": fs, "write_scale_KiB": ws, "launches": table}
    with open(tf, "w") as fh:
        json.dump(whole, fh, indent=1, sort_keys=True)
        fh.write("\n")

    # ---- matrix-unit busy time
    mp = glob.glob(os.path.join(O, "mfma", "**", "*counter_collection.csv"), recursive=True)
    if mp:
        c = counters(mp[0], n)
        busy, cu = c["SQ_VALU_MFMA_BUSY_CYCLES"][0], c["SQ_BUSY_CU_CYCLES"][0]
        with open(os.path.join(PROFILES, "%s_step_mfma_busy_pmc.txt" % wl), "w") as f:
            f.write("# Matrix-unit utilisation per launch of workload %s (rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CU_CYCLES;\n"
                    "# command: see profile_summary.py).  busy = MFMA busy cycles summed over the SIMDs / (4 SIMDs x busy CU cycles):\n"
                    "# the share of the time a CU works on the launch during which its matrix units execute.  of_peak = the\n"
                    "# launch's flops over its duration in the kernel trace against %d TFLOP/s.\n" % (wl, int(PEAK_TFLOPS)))
            f.write("%-3s %-44s %16s %16s %8s %9s %8s\n" % ("#", "launch", "MFMA_BUSY_CYCLES", "BUSY_CU_CYCLES", "busy", "TFLOP/s", "of_peak"))
            for i, rec in enumerate(launches):
                if not rec["flops"]:
                    continue
                tfl = rec["flops"] / (dur[i] * 1e-6) / 1e12
                f.write("%-3d %-44s %16.0f %16.0f %8.3f %9.1f %8.3f\n" % (i, key(rec), busy[i], cu[i], busy[i] / (4.0 * cu[i]) if cu[i] else 0.0,
                                                                       tfl, tfl / PEAK_TFLOPS))
    # ---- where the waves' cycles go (optional fifth run)
    sp = glob.glob(os.path.join(O, "sq", "**", "*counter_collection.csv"), recursive=True)
    if sp:
        c = counters(sp[0], n)
        names_sq = ["SQ_WAVE_CYCLES", "SQ_WAIT_ANY", "SQ_WAIT_INST_ANY", "SQ_WAIT_INST_LDS", "SQ_ACTIVE_INST_LDS", "SQ_ACTIVE_INST_VMEM"]
        with open(os.path.join(PROFILES, "%s_step_wave_cycles_pmc.txt" % wl), "w") as f:
            f.write("# Where the waves' cycles go per launch of workload %s (rocprofv3 --pmc %s;\n"
                    "# command: see profile_summary.py).  Shares of SQ_WAVE_CYCLES (cycles waves spend resident): waiting at a wait\n"
                    "# count or barrier (WAIT_ANY), waiting for an instruction to be issued (WAIT_INST_ANY), of which for an LDS\n"
                    "# instruction (WAIT_INST_LDS); cycles an LDS / a vector-memory instruction is being issued.\n" % (wl, " ".join(names_sq)))
            f.write("%-3s %-44s %14s %10s %14s %14s %12s %12s\n" % ("#", "launch", "WAVE_CYCLES", "WAIT_ANY", "WAIT_INST_ANY", "WAIT_INST_LDS",
                                                                    "ACTIVE_LDS", "ACTIVE_VMEM"))
            for i, rec in enumerate(launches):
                wc = c["SQ_WAVE_CYCLES"][0][i] or 1.0
                f.write("%-3d %-44s %14.0f %10.3f %14.3f %14.3f %12.3f %12.3f\n" % (
                    i, key(rec), wc, c["SQ_WAIT_ANY"][0][i] / wc, c["SQ_WAIT_INST_ANY"][0][i] / wc, c["SQ_WAIT_INST_LDS"][0][i] / wc,
                    c["SQ_ACTIVE_INST_LDS"][0][i] / wc, c["SQ_ACTIVE_INST_VMEM"][0][i] / wc))
    print("wrote profiles for", wl)


if __name__ == "__main__":
    main()
