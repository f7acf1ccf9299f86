"""Turn rocprofv3 CSV output into the short text summaries kept under profiles/.

    python -m paper_2605_06534_amd.profile_summary --workload decoder32b_tp8 --density 0.02 \\
        --stats <dir of a `--kernel-trace --stats` run> --fetch <dir of a `--pmc FETCH_SIZE` run> \\
        --write <dir of a `--pmc WRITE_SIZE` run> [--lds <dir of a `--pmc SQ_LDS_BANK_CONFLICT SQ_LDS_ACTIVE ...` run>] \\
        --command "<the profiled command>" --out-prefix profiles/encode_apply_decoder32b_tp8

writes <prefix>_kernel_stats.txt and <prefix>_hbm_traffic.txt.  The traffic file carries one
`TRAFFIC key=value ...` line per library kernel, which bench.py reads for `roofline.traffic`:
FETCH_SIZE / WRITE_SIZE are KiB per dispatch (summed over the counter's instances, averaged over
the dispatches of the kernel), and each is scaled by what the same counter reads for the copy probe
(bw_copy_kernel moves exactly 1 GiB each way per dispatch in bench.py), found in the same run.
"""
import argparse
import collections
import csv
import glob
import hashlib
import os
import re
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
COPY_KIB = float(1 << 20)        # the copy probe reads and writes 1 GiB per dispatch


def kernels_sha256():
    h = hashlib.sha256()
    for f in ("kernels.hip", "rose_internal.h"):
        with open(os.path.join(ROOT, "paper_2605_06534_amd", "csrc", f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def short(name):
    """'void rose::encode_kernel<0, 0, 0>(rose::EncodeArgs)' -> 'encode_kernel<0,0,0>'"""
    m = re.search(r"rose::([A-Za-z0-9_]+(?:<[^>]*>)?)\s*\(", name)
    return m.group(1).replace(" ", "") if m else None


def counters(directory):
    """-> {kernel: {counter: (mean per dispatch, dispatches)}} for the library's kernels"""
    per = collections.defaultdict(lambda: collections.defaultdict(lambda: collections.defaultdict(float)))
    for f in glob.glob(os.path.join(directory, "**", "*counter_collection.csv"), recursive=True):
        for r in csv.DictReader(open(f)):
            k = short(r["Kernel_Name"])
            if k:
                per[k][r["Counter_Name"]][r["Dispatch_Id"]] += float(r["Counter_Value"])
    return {k: {c: (sum(d.values()) / len(d), len(d)) for c, d in cs.items()} for k, cs in per.items()}


def stats(directory):
    rows = []
    for f in glob.glob(os.path.join(directory, "**", "*kernel_stats.csv"), recursive=True):
        for r in csv.DictReader(open(f)):
            k = short(r["Name"])
            if k:
                rows.append((k, int(r["Calls"]), float(r["AverageNs"]), float(r["MinNs"]), float(r["MaxNs"])))
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", required=True)
    ap.add_argument("--density", default="recipe")
    ap.add_argument("--stats")
    ap.add_argument("--fetch")
    ap.add_argument("--write")
    ap.add_argument("--lds")
    ap.add_argument("--command", default="python3 bench.py")
    ap.add_argument("--bench-json", help="the JSON line bench.py printed in the --stats run, to quote beside it")
    ap.add_argument("--out-prefix", required=True)
    a = ap.parse_args()
    sha = kernels_sha256()
    dens = a.density if a.density == "recipe" else "%g" % float(a.density)
    pre = "cd /tmp && export TMPDIR=/tmp && rocprofv3 %s --output-format csv -d <out> -- " + a.command

    if a.stats:
        with open(a.out_prefix + "_kernel_stats.txt", "w") as f:
            f.write("rocprofv3 kernel summary: %s, density %s (kernel sources %s)\n" % (a.workload, dens, sha))
            f.write("command: " + pre % "--kernel-trace --stats" + "\n")
            f.write("%-34s %8s %14s %14s %14s\n" % ("kernel", "calls", "avg_ns", "min_ns", "max_ns"))
            for k, calls, avg, mn, mx in sorted(stats(a.stats), key=lambda r: -r[1] * r[2]):
                f.write("%-34s %8d %14.0f %14.0f %14.0f\n" % (k, calls, avg, mn, mx))
            if a.bench_json and os.path.exists(a.bench_json):
                line = [l for l in open(a.bench_json) if l.startswith("{")]
                if line:
                    import json
                    j = json.loads(line[-1])
                    r, d = j["roofline"], j["detail"]
                    f.write("bench.py in the same run (HIP events): encode %.4f ms per launch, apply %.4f ms per step, "
                            "step %.4f ms, nnz %d\n" % (d["t_encode_ms"], d["t_apply_ms"], j["ms_per_step"], j["config"]["nnz"]))
                    f.write("encode algorithmic bytes per launch %d -> %.1f GB/s = %.4f of 8 TB/s\n"
                            % (r["algorithmic_bytes"], r["achieved"], r["frac"]))
                    if "decoder7b_tp4" in d:
                        for key, e in d["decoder7b_tp4"].items():
                            f.write("  then decoder7b_tp4 at %g: encode %.4f ms (%.4f of peak), apply %.4f ms\n"
                                    % (e["density"], e["t_encode_ms"], e["encode_frac_of_peak"], e["t_apply_ms"]))

    if a.fetch and a.write:
        cf, cw = counters(a.fetch), counters(a.write)
        if "bw_copy_kernel" not in cf or "bw_copy_kernel" not in cw:
            sys.exit("the copy probe is not in the counter runs: no calibration")
        fs = COPY_KIB / cf["bw_copy_kernel"]["FETCH_SIZE"][0]
        wsc = COPY_KIB / cw["bw_copy_kernel"]["WRITE_SIZE"][0]
        with open(a.out_prefix + "_hbm_traffic.txt", "w") as f:
            f.write("rocprofv3 HBM traffic counters: %s, density %s (kernel sources %s)\n" % (a.workload, dens, sha))
            f.write("commands (one counter per run):\n  " + pre % "--pmc FETCH_SIZE" + "\n  " + pre % "--pmc WRITE_SIZE" + "\n")
            f.write("calibration: bw_copy_kernel moves 1,048,576 KiB each way per dispatch; FETCH_SIZE reads %.0f -> scale %.3f; "
                    "WRITE_SIZE reads %.0f -> scale %.3f\n" % (cf["bw_copy_kernel"]["FETCH_SIZE"][0], fs,
                                                              cw["bw_copy_kernel"]["WRITE_SIZE"][0], wsc))
            f.write("%-34s %10s %14s %12s %14s %12s\n" % ("kernel", "dispatches", "FETCH_SIZE KiB", "GB read", "WRITE_SIZE KiB", "GB written"))
            for k in sorted(set(cf) & set(cw)):
                fe, n = cf[k].get("FETCH_SIZE", (0.0, 0))
                wr, _ = cw[k].get("WRITE_SIZE", (0.0, 0))
                f.write("%-34s %10d %14.0f %12.3f %14.0f %12.3f\n" % (k, n, fe, fe * fs * 1024 / 1e9, wr, wr * wsc * 1024 / 1e9))
            f.write("\n")
            for k in sorted(set(cf) & set(cw)):
                fe = cf[k].get("FETCH_SIZE", (0.0, 0))[0]
                wr = cw[k].get("WRITE_SIZE", (0.0, 0))[0]
                f.write("TRAFFIC kernel=%s workload=%s density=%s fetch_KiB=%.1f write_KiB=%.1f fetch_scale=%.4f "
                        "write_scale=%.4f kernels_sha256=%s\n" % (k, a.workload, dens, fe, wr, fs, wsc, sha))
            if a.lds:
                f.write("\nLDS counters (one run, sums over all waves, mean per dispatch):\n")
                for k, cs in sorted(counters(a.lds).items()):
                    f.write("  %-34s %s\n" % (k, "  ".join("%s=%.4g" % (c, v[0]) for c, v in sorted(cs.items()))))


if __name__ == "__main__":
    main()
