#!/usr/bin/env python3
"""Short text summaries of rocprofv3 runs of bench.py (csv output), and the HBM-traffic table bench.py reads.

    python3 paper_2604_03425_amd/profile_summary.py kernels DIR        # --kernel-trace --stats run: top kernels
    python3 paper_2604_03425_amd/profile_summary.py counters DIR...    # --pmc runs: per-kernel counter averages
    python3 paper_2604_03425_amd/profile_summary.py traffic CAL_FETCH CAL_WRITE FETCH WRITE [OUT.json]
        # four --pmc runs (FETCH_SIZE / WRITE_SIZE on `bench.py --workload calibrate`, then on the default
        # bench.py): prints the calibration and the HBM bytes per launch of every kernel and writes them, with the
        # digest of the sources they were measured on, to OUT.json (default profiles/keyswitch_micro_traffic.json,
        # the file bench.py reads)

Runs anywhere (no GPU, no torch): it only reads the csv files.
"""
import collections
import csv
import glob
import json
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, HERE)
from srcdigest import source_digest  # noqa: E402

COPY_KERNEL = "ckks_prof_copy_kernel"
COPY_KIB = (1 << 30) // 1024     # KiB read (and written) per launch of `bench.py --workload calibrate`


def kind(name):
    """rocprofv3 kernel name -> the kernel-kind name bench.py uses."""
    n = name.strip()
    if n.startswith("void "):
        n = n[5:]
    n = n.split("(")[0]
    base = n.split("<")[0]
    if base in ("modup_kernel", "moddown_kernel"):
        return base
    if base == "ntt16_bconv_rows_kernel":
        return base + "<" + n.split("<")[1].split(",")[0].strip(" >") + ">"
    return n


def read_counters(d):
    """{(kind, counter): (launches, sum)} over every counter_collection csv under d."""
    agg = collections.defaultdict(lambda: [0, 0.0])
    for f in glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True):
        for r in csv.DictReader(open(f)):
            k = (kind(r["Kernel_Name"]), r["Counter_Name"])
            agg[k][0] += 1
            agg[k][1] += float(r["Counter_Value"])
    return agg


def cmd_kernels(d):
    for f in sorted(glob.glob(os.path.join(d, "**", "*kernel_stats.csv"), recursive=True)):
        print("%-46s %8s %14s %12s %7s" % ("kernel", "calls", "total_us", "avg_us", "%"))
        for r in list(csv.DictReader(open(f)))[:16]:
            print("%-46s %8s %14.1f %12.2f %7.2f" % (kind(r["Name"])[:46], r["Calls"], float(r["TotalDurationNs"]) / 1e3,
                                                     float(r["AverageNs"]) / 1e3, float(r["Percentage"])))


def cmd_counters(dirs):
    agg = collections.defaultdict(dict)
    for d in dirs:
        for (k, c), (n, s) in read_counters(d).items():
            agg[k][c] = (n, s / n)
    order = sorted(agg, key=lambda k: -agg[k].get("SQ_BUSY_CYCLES", (0, 0))[1] * agg[k].get("SQ_BUSY_CYCLES", (0, 0))[0])
    names = sorted({c for k in agg for c in agg[k]})
    for k in order:
        if k.startswith("at::") or "rocclr" in k:
            continue
        n = max(v[0] for v in agg[k].values())
        print("== %s (%d launches; averages per launch)" % (k, n))
        for c in names:
            if c in agg[k]:
                print("   %-26s %16.0f" % (c, agg[k][c][1]))


def cmd_traffic(cal_fetch, cal_write, fetch, write, out=None):
    cf, cw = read_counters(cal_fetch), read_counters(cal_write)
    nf, sf = cf[(COPY_KERNEL, "FETCH_SIZE")]
    nw, sw = cw[(COPY_KERNEL, "WRITE_SIZE")]
    f_fetch, f_write = COPY_KIB / (sf / nf), COPY_KIB / (sw / nw)
    print("calibration (%s, %d KiB read and written per launch):" % (COPY_KERNEL, COPY_KIB))
    print("    FETCH_SIZE reads %.1f per launch -> factor %.4f to KiB" % (sf / nf, f_fetch))
    print("    WRITE_SIZE reads %.1f per launch -> factor %.4f to KiB" % (sw / nw, f_write))
    rf, rw = read_counters(fetch), read_counters(write)
    kinds = sorted({k for (k, c) in list(rf) + list(rw) if not k.startswith("at::") and "rocclr" not in k and k != COPY_KERNEL})
    table = {}
    print("\n%-40s %9s %16s %16s %18s" % ("kernel", "launches", "FETCH_SIZE/launch", "WRITE_SIZE/launch", "HBM bytes/launch"))
    for k in kinds:
        n1, s1 = rf.get((k, "FETCH_SIZE"), (0, 0.0))
        n2, s2 = rw.get((k, "WRITE_SIZE"), (0, 0.0))
        if not n1 or not n2:
            continue
        b = (s1 / n1 * f_fetch + s2 / n2 * f_write) * 1024
        table[k] = int(round(b))
        print("%-40s %9d %16.1f %16.1f %18d" % (k, n1, s1 / n1, s2 / n2, table[k]))
    rec = {"source_sha256": source_digest(), "fetch_factor_to_KiB": round(f_fetch, 4), "write_factor_to_KiB": round(f_write, 4),
           "note": "HBM bytes per launch, average over the launches of a step (one on 64 ciphertexts, one on 32)",
           "hbm_bytes_per_launch": table}
    out = out or os.path.join(os.path.dirname(HERE), "profiles", "keyswitch_micro_traffic.json")
    with open(out, "w") as f:
        json.dump(rec, f, indent=1, sort_keys=True)
        f.write("\n")
    print("\nwrote %s (sources %s)" % (out, rec["source_sha256"][:16]))


if __name__ == "__main__":
    if len(sys.argv) >= 3 and sys.argv[1] == "kernels":
        cmd_kernels(sys.argv[2])
    elif len(sys.argv) >= 3 and sys.argv[1] == "counters":
        cmd_counters(sys.argv[2:])
    elif len(sys.argv) in (6, 7) and sys.argv[1] == "traffic":
        cmd_traffic(*sys.argv[2:])
    else:
        print(__doc__)
        sys.exit(2)
