#!/usr/bin/env python3
"""Turns rocprofv3 CSV output into the short text summaries kept under profiles/.

Usage (after the rocprofv3 runs named in each summary's header; from /tmp on the GPU machine with TMPDIR=/tmp):
  python profile_summary.py stats   <dir with *_kernel_stats.csv>        --title "..." --command "..." > profiles/<name>.txt
  python profile_summary.py counters <dir with *_counter_collection.csv> --title "..." --command "..." > profiles/<name>.txt
  python profile_summary.py traffic --fetch <dir> --write <dir> --dominant <kernel substring> --command "..." > profiles/<name>.txt

`traffic` scales FETCH_SIZE / WRITE_SIZE (KiB per dispatch) by what the same counters read for the calibration kernel
of known size that `bench.py --copy-calibration` launches (an elementwise add reading 1 GiB and writing 1 GiB), and ends
with one JSON line that bench.py reports as roofline.traffic, stamped with the library commit the run used.
"""
import argparse
import collections
import csv
import glob
import json
import os
import re
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))


def short(name):
    name = re.sub(r"^void ", "", name).replace("surgeon::", "").replace("(anonymous namespace)::", "")
    name = re.sub(r"\(.*$", "", name)
    return name[:96]


def find(directory, suffix):
    hits = sorted(glob.glob(os.path.join(directory, "**", "*" + suffix), recursive=True))
    if not hits:
        sys.exit("no *%s under %s" % (suffix, directory))
    return hits[0]


def library_commit():
    try:
        return json.load(open(os.path.join(ROOT, "paper_2503_20354_amd", "build_info.json")))
    except Exception:
        return {"commit": "unknown", "dirty": None}


def header(args):
    print(args.title)
    print("command (from /tmp on the GPU box, TMPDIR=/tmp):")
    for line in args.command.split(" && "):
        print("  " + line)
    print("library: %s" % json.dumps(library_commit()))


def cmd_stats(args):
    header(args)
    rows = list(csv.DictReader(open(find(args.dir, "kernel_stats.csv"))))
    total = sum(float(r["TotalDurationNs"]) for r in rows)
    print("%-98s %7s %11s %10s %6s" % ("kernel", "calls", "total ms", "avg us", "%"))
    for r in sorted(rows, key=lambda r: -float(r["TotalDurationNs"]))[:args.top]:
        t = float(r["TotalDurationNs"])
        print("%-98s %7d %11.3f %10.1f %6.1f" % (short(r["Name"]), int(r["Calls"]), t / 1e6, float(r["AverageNs"]) / 1e3,
                                                  100.0 * t / total))
    print("all kernels: %.3f ms" % (total / 1e6))


def per_kernel_counters(path, only=None):
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    dur = collections.defaultdict(dict)
    for r in csv.DictReader(open(path)):
        n = short(r["Kernel_Name"])
        if only and only not in n:
            continue
        acc[n][r["Counter_Name"]].append(float(r["Counter_Value"]))
        dur[n][r["Dispatch_Id"]] = (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3
    return acc, dur


def cmd_counters(args):
    header(args)
    acc, dur = per_kernel_counters(find(args.dir, "counter_collection.csv"))
    order = sorted((n for n in acc if args.only in n), key=lambda n: -sum(dur[n].values()))[:args.top]
    for n in order:
        d = list(dur[n].values())
        print("%s  dispatches=%d avg_us=%.1f" % (n, len(d), sum(d) / len(d)))
        c = {k: sum(v) / len(v) for k, v in acc[n].items()}
        for k in sorted(c):
            print("    %-30s mean per dispatch %.4g" % (k, c[k]))
        # derived: matrix-pipeline utilisation = MFMA busy cycles / (SIMD cycles of the dispatch); the busy counters are
        # summed over the chip's 1024 SIMDs, SQ_BUSY_CYCLES over its 32 shader engines x XCDs
        if "SQ_VALU_MFMA_BUSY_CYCLES" in c and "SQ_BUSY_CYCLES" in c and c["SQ_BUSY_CYCLES"] > 0:
            cycles = c["SQ_BUSY_CYCLES"] / 32.0
            print("    -> matrix pipeline busy %.1f %% of SIMD cycles (cycles per dispatch %.0f)" %
                  (100.0 * c["SQ_VALU_MFMA_BUSY_CYCLES"] / (cycles * 1024.0), cycles))
        if "SQ_INSTS_VALU" in c and "SQ_WAVES" in c and c["SQ_WAVES"] > 0:
            print("    -> per wavefront: %.0f vector, %.0f scalar, %.0f LDS instructions" %
                  (c["SQ_INSTS_VALU"] / c["SQ_WAVES"], c.get("SQ_INSTS_SALU", 0.0) / c["SQ_WAVES"],
                   c.get("SQ_INSTS_LDS", 0.0) / c["SQ_WAVES"]))
        if "SQ_ACTIVE_INST_VALU" in c and "SQ_BUSY_CYCLES" in c and c["SQ_BUSY_CYCLES"] > 0:
            # SQ_ACTIVE_INST_* count in units of four cycles per SIMD (one per issued wave64 instruction on gfx950)
            cycles = c["SQ_BUSY_CYCLES"] / 32.0
            print("    -> vector ALU busy %.1f %% of SIMD cycles" % (100.0 * 4.0 * c["SQ_ACTIVE_INST_VALU"] / (cycles * 1024.0)))
            if "SQ_ACTIVE_INST_LDS" in c:
                print("    -> LDS busy %.1f %% of compute-unit cycles" % (100.0 * 4.0 * c["SQ_ACTIVE_INST_LDS"] / (cycles * 256.0)))
        if "SQ_INSTS_VALU" in c and "SQ_INSTS_MFMA" in c and c["SQ_INSTS_MFMA"] > 0:
            print("    -> vector instructions per matrix instruction %.2f" %
                  ((c["SQ_INSTS_VALU"] - c["SQ_INSTS_MFMA"]) / c["SQ_INSTS_MFMA"]))


def cmd_traffic(args):
    header(args)
    out = {}
    factors = {}
    for which, directory in (("FETCH_SIZE", args.fetch), ("WRITE_SIZE", args.write)):
        acc, dur = per_kernel_counters(find(directory, "counter_collection.csv"))
        cal = [n for n in acc if "elementwise" in n or "vectorized" in n]
        if not cal:
            sys.exit("calibration kernel not found in " + directory)
        cal_kib = max(max(acc[n][which]) for n in cal if which in acc[n])
        factors[which] = (1 << 20) / cal_kib  # the calibration kernel moves exactly 1 GiB = 2^20 KiB in each direction
        print("%s read %.0f KiB for the 1 GiB calibration kernel -> factor %.3f" % (which, cal_kib, factors[which]))
        for n in acc:
            if which in acc[n]:
                out.setdefault(n, {})[which] = factors[which] * 1024.0 * sum(acc[n][which]) / len(acc[n][which])
                out[n]["n"] = len(acc[n][which])
                out[n]["us"] = sum(dur[n].values()) / len(dur[n])
    print("%-98s %6s %9s %12s %12s %9s" % ("kernel", "calls", "avg us", "fetch B", "write B", "TB/s"))
    dominant = None
    for n in sorted(out, key=lambda n: -out[n]["us"] * out[n]["n"])[:args.top]:
        f, w = out[n].get("FETCH_SIZE", 0.0), out[n].get("WRITE_SIZE", 0.0)
        print("%-98s %6d %9.1f %12.4g %12.4g %9.2f" % (n, out[n]["n"], out[n]["us"], f, w, (f + w) / out[n]["us"] / 1e6))
        if args.dominant and args.dominant in n and dominant is None:
            dominant = f + w
    print("machine-readable (bench.py reports it as roofline.traffic):")
    print(json.dumps({"dw_hbm_bytes_per_launch": dominant, "dominant_kernel": args.dominant, "fetch_factor": factors["FETCH_SIZE"],
                      "write_factor": factors["WRITE_SIZE"], "library_commit": library_commit().get("commit")}))


def main():
    ap = argparse.ArgumentParser()
    sub = ap.add_subparsers(dest="what", required=True)
    for name in ("stats", "counters"):
        p = sub.add_parser(name)
        p.add_argument("dir")
        p.add_argument("--title", default="rocprofv3 summary")
        p.add_argument("--command", default="")
        p.add_argument("--top", type=int, default=14)
        p.add_argument("--only", default="", help="counters: kernels whose name contains this text")
    p = sub.add_parser("traffic")
    p.add_argument("--fetch", required=True)
    p.add_argument("--write", required=True)
    p.add_argument("--dominant", default="dw_conv_kernel")
    p.add_argument("--title", default="rocprofv3 HBM traffic")
    p.add_argument("--command", default="")
    p.add_argument("--top", type=int, default=14)
    args = ap.parse_args()
    {"stats": cmd_stats, "counters": cmd_counters, "traffic": cmd_traffic}[args.what](args)


if __name__ == "__main__":
    main()
