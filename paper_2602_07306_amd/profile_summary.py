"""Turns raw rocprofv3 output into the short summaries kept under profiles/.

    python -m paper_2602_07306_amd.profile_summary kernels <dir with *kernel_stats.csv> --command "<full command>"
        [--bench-json FILE] > profiles/<kernel>_<workload>.txt
    python -m paper_2602_07306_amd.profile_summary traffic --fetch <dir of the FETCH_SIZE pass>
        --write <dir of the WRITE_SIZE pass> --kernel <substring of the kernel name> --algorithmic-bytes N
        --command "<command of the FETCH_SIZE pass>" --command "<command of the WRITE_SIZE pass>" [--note TEXT]
        > profiles/<kernel>_<workload>_traffic.json
    python -m paper_2602_07306_amd.profile_summary mfma <dir of the counter pass> --command "<full command>"
        [--kernel SUBSTRING ...] > profiles/<workload>_mfma_counters.json

`mfma` reads a pass over SQ_INSTS_VALU_MFMA_MOPS_BF16, SQ_VALU_MFMA_BUSY_CYCLES and GRBM_GUI_ACTIVE and reports, per
kernel, the matrix FLOPs executed and the share of the matrix pipes' cycles that were busy.

`traffic` scales both counters (KiB per dispatch) by what the same counter reads for the plain copy kernel of known
size that `bench.py --copy-calibration` runs in the same process (hbm_copy_kernel over 1 GiB: 1 GiB read, 1 GiB
written), and reports HBM-side bytes per launch of the named kernel.
"""
import argparse
import collections
import csv
import glob
import json
import os
import sys

CALIB_KERNEL = "hbm_copy_kernel"
CALIB_BYTES = 1 << 30


def find(root, pattern):
    files = glob.glob(os.path.join(root, "**", pattern), recursive=True)
    if not files:
        raise SystemExit("no %s under %s" % (pattern, root))
    return files


def kernels(args):
    rows = []
    for f in find(args.dir, "*kernel_stats.csv"):
        rows += list(csv.DictReader(open(f)))
    rows.sort(key=lambda r: -float(r["TotalDurationNs"]))
    out = ["rocprofv3 --kernel-trace --stats summary (MI355X, gfx950)", "command: %s" % args.command, "",
           "%-100s %8s %14s %12s %7s" % ("kernel", "calls", "total_ms", "avg_us", "pct")]
    for r in rows[:args.top]:
        out.append("%-100s %8s %14.3f %12.2f %7s" % (r["Name"][:100], r["Calls"], float(r["TotalDurationNs"]) / 1e6,
                                                    float(r["AverageNs"]) / 1e3, r["Percentage"]))
    if args.bench_json:
        out += ["", "bench.py JSON line of the same run:", open(args.bench_json).read().strip()]
    print("\n".join(out))


def counter_means(root, counter):
    """{kernel name: (dispatches, mean counter value)} of one --pmc pass."""
    acc = collections.defaultdict(lambda: [0, 0.0])
    for f in find(root, "*counter_collection.csv"):
        for r in csv.DictReader(open(f)):
            if r["Counter_Name"] == counter:
                a = acc[r["Kernel_Name"]]
                a[0] += 1
                a[1] += float(r["Counter_Value"])
    return {k: (n, s / n) for k, (n, s) in acc.items()}


def pick(means, needle, min_value=0.0):
    hits = {k: v for k, v in means.items() if needle in k and v[1] >= min_value}
    if not hits:
        raise SystemExit("no kernel matching %r in the counter pass" % needle)
    return max(hits.items(), key=lambda kv: kv[1][0] * kv[1][1])   # the variant that moved the most bytes


def traffic(args):
    rec = {"kernel": None, "commands": args.command, "raw_per_launch_KiB": {}, "calibration_kernel": CALIB_KERNEL,
           "calibration_raw_KiB": {}, "scale": {}, "dispatches": {}}
    total = 0.0
    for counter, root in (("FETCH_SIZE", args.fetch), ("WRITE_SIZE", args.write)):
        means = counter_means(root, counter)
        name, (n, mean) = pick(means, args.kernel)
        _, (_, cal) = pick(means, CALIB_KERNEL)
        scale = (CALIB_BYTES / 1024.0) / cal          # the copy reads and writes CALIB_BYTES
        rec["kernel"] = name[:160]
        rec["raw_per_launch_KiB"][counter] = mean
        rec["calibration_raw_KiB"][counter] = cal
        rec["scale"][counter] = scale
        rec["dispatches"][counter] = n
        rec[counter.split("_")[0].lower() + "_bytes_per_launch"] = mean * 1024.0 * scale
        total += mean * 1024.0 * scale
    rec["traffic_bytes_per_launch"] = total
    rec["algorithmic_bytes_per_launch"] = args.algorithmic_bytes
    rec["ratio"] = total / args.algorithmic_bytes if args.algorithmic_bytes else None
    if args.note:
        rec["note"] = args.note
    print(json.dumps(rec, indent=1))


def mfma(args):
    mops = counter_means(args.dir, "SQ_INSTS_VALU_MFMA_MOPS_BF16")
    busy = counter_means(args.dir, "SQ_VALU_MFMA_BUSY_CYCLES")
    active = counter_means(args.dir, "GRBM_GUI_ACTIVE")
    rec = {"command": args.command,
           "reading": "Per launch, mean over launches. SQ_INSTS_VALU_MFMA_MOPS_BF16 counts 512 FLOPs per unit; "
                      "SQ_VALU_MFMA_BUSY_CYCLES sums the busy cycles of the 1024 MFMA pipes (4 SIMDs x 256 CUs); "
                      "GRBM_GUI_ACTIVE sums the active cycles of the 8 XCDs, so one eighth of it is the kernel's duration "
                      "in shader clocks. mfma_pipe_busy = busy / (1024 x duration). Counter runs serialise kernels; "
                      "durations are a few per cent longer than in the timed run.",
           "kernels": {}}
    names = [k for k in mops if mops[k][1] > 0 and (not args.kernel or any(n in k for n in args.kernel))]
    names.sort(key=lambda k: -mops[k][0] * mops[k][1])
    for k in names[:args.top]:
        clocks = active[k][1] / 8.0
        rec["kernels"][k[:120]] = {"launches": mops[k][0], "mfma_flops_executed": mops[k][1] * 512.0,
                                   "mfma_busy_cycles": busy[k][1], "duration_shader_clocks": clocks,
                                   "mfma_pipe_busy": busy[k][1] / (1024.0 * clocks)}
    print(json.dumps(rec, indent=1))


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="mode", required=True)
    k = sub.add_parser("kernels")
    k.add_argument("dir")
    k.add_argument("--command", required=True)
    k.add_argument("--bench-json")
    k.add_argument("--top", type=int, default=18)
    t = sub.add_parser("traffic")
    t.add_argument("--fetch", required=True)
    t.add_argument("--write", required=True)
    t.add_argument("--kernel", required=True)
    t.add_argument("--algorithmic-bytes", type=float, required=True)
    t.add_argument("--command", action="append", required=True)
    t.add_argument("--note")
    m = sub.add_parser("mfma")
    m.add_argument("dir")
    m.add_argument("--command", required=True)
    m.add_argument("--kernel", action="append")
    m.add_argument("--top", type=int, default=6)
    args = ap.parse_args()
    {"kernels": kernels, "traffic": traffic, "mfma": mfma}[args.mode](args)


if __name__ == "__main__":
    main()
