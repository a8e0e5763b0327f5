"""Turns rocprofv3 CSV output of `bench.py` runs into the short text summaries kept with the
sources: per-kernel time (from a --kernel-trace --stats run) and per-kernel HBM traffic (from
two --pmc runs, FETCH_SIZE and WRITE_SIZE).

The traffic counters are scaled by what the same counter reads for the plain copy kernel that
`bench.py` launches with a known size (256 MiB read, 256 MiB written per launch), because
FETCH_SIZE does not count every byte on this part.

    python -m paper_2602_08007_amd.profile_summary stats  <dir of the --stats run>
    python -m paper_2602_08007_amd.profile_summary traffic <dir of FETCH_SIZE run> <dir of WRITE_SIZE run>
"""
from __future__ import annotations

import collections
import csv
import glob
import os
import sys

COPY_BYTES = 64 * 1024 * 1024 * 4          # one direction of bench.py's calibration copy


def _find(d, suffix):
    hits = sorted(glob.glob(os.path.join(d, "**", "*" + suffix), recursive=True))
    if not hits:
        raise SystemExit("no *%s under %s" % (suffix, d))
    return hits[0]


def _short(name):
    name = name.replace("(anonymous namespace)::", "").replace("void tsr::", "").replace("tsr::", "")
    return name.split("(")[0]


def stats(d):
    rows = list(csv.DictReader(open(_find(d, "kernel_stats.csv"))))
    print("%-58s %8s %12s %12s %7s" % ("kernel", "calls", "total_ms", "avg_us", "pct"))
    for r in rows:
        if "tsr::" not in r["Name"]:
            continue
        print("%-58s %8d %12.3f %12.2f %7.2f" % (_short(r["Name"])[:58], int(r["Calls"]), float(r["TotalDurationNs"]) / 1e6,
                                                 float(r["AverageNs"]) / 1e3, float(r["Percentage"])))


def _counter(d, counter):
    acc = collections.defaultdict(list)
    for r in csv.DictReader(open(_find(d, "counter_collection.csv"))):
        if r["Counter_Name"] == counter and "tsr::" in r["Kernel_Name"]:
            acc[_short(r["Kernel_Name"])].append(float(r["Counter_Value"]))
    return acc


def traffic(d_fetch, d_write):
    fetch, write = _counter(d_fetch, "FETCH_SIZE"), _counter(d_write, "WRITE_SIZE")

    def mean(v):
        return sum(v) / len(v)
    if "stream_kernel" not in fetch or "stream_kernel" not in write:
        raise SystemExit("the calibration copy kernel is missing from the trace")
    f_scale = COPY_BYTES / (mean(fetch["stream_kernel"]) * 1024.0)
    w_scale = COPY_BYTES / (mean(write["stream_kernel"]) * 1024.0)
    print("# counters in KiB per dispatch; scale = known bytes of the copy kernel / counter reading")
    print("fetch_scale: %.4f" % f_scale)
    print("write_scale: %.4f" % w_scale)
    print("%-58s %6s %14s %14s %14s" % ("# kernel", "n", "fetch_MB", "write_MB", "total_MB (scaled)"))
    lift_total = None
    for k in sorted(set(fetch) | set(write)):
        fb = mean(fetch[k]) * 1024.0 * f_scale if k in fetch else 0.0
        wb = mean(write[k]) * 1024.0 * w_scale if k in write else 0.0
        print("# %-56s %6d %14.2f %14.2f %14.2f" % (k[:56], len(fetch.get(k, write.get(k))), fb / 1e6, wb / 1e6, (fb + wb) / 1e6))
        if k.startswith("lift_kernel"):
            lift_total = (lift_total or 0.0) + fb + wb
    if lift_total is not None:
        print("tvt_traffic_bytes_per_launch: %.0f" % lift_total)


if __name__ == "__main__":
    if len(sys.argv) >= 3 and sys.argv[1] == "stats":
        stats(sys.argv[2])
    elif len(sys.argv) >= 4 and sys.argv[1] == "traffic":
        traffic(sys.argv[2], sys.argv[3])
    else:
        raise SystemExit(__doc__)
