"""Turn rocprofv3 output into the short text summaries kept under profiles/.

    python -m paper_1906_06440_amd.profile_summary stats   <out>/run_kernel_stats.csv [--top 18]
    python -m paper_1906_06440_amd.profile_summary pmc     <out>/run_counter_collection.csv [--match brg]
    python -m paper_1906_06440_amd.profile_summary traffic --fetch F.csv --write W.csv --copy-fetch CF.csv --copy-write CW.csv
                                                           --kernels "conv_tile_f32:1,conv_wt_transpose_f32:1" --sources a.hpp,b.hip

`stats` prints the per-kernel table of a `rocprofv3 --kernel-trace --stats --output-format csv` run (times in us).
`pmc` prints, per kernel and grid size, the mean over dispatches of every counter of a `rocprofv3 --pmc ...
--output-format csv` run.  `traffic` combines a FETCH_SIZE and a WRITE_SIZE run (KiB per dispatch) of a workload with
the same two runs of `bench.py --workload copy` (a device copy of 256 MiB, i.e. 262144 KiB read and as much written)
into HBM bytes per step: each counter is scaled by 262144 / (what it reads for the copy), summed over the listed
kernels times their launches per step, and printed as one `TRAFFIC {json}` line that bench.py reads back, with a hash
of the kernel sources the figure belongs to.
"""
from __future__ import annotations

import argparse
import collections
import csv
import hashlib
import json
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
COPY_KIB = 262144.0


def stats(path, top):
    rows = list(csv.DictReader(open(path)))
    print("%-100s %6s %12s %10s %10s %7s" % ("kernel", "calls", "avg_us", "min_us", "max_us", "pct"))
    for r in rows[:top]:
        print("%-100s %6s %12.2f %10.2f %10.2f %7.2f" % (r["Name"][:100], r["Calls"], float(r["AverageNs"]) / 1e3,
                                                         float(r["MinNs"]) / 1e3, float(r["MaxNs"]) / 1e3, float(r["Percentage"])))


def _per_dispatch(path):
    """{(kernel, grid): {counter: [value per dispatch]}}; rows of one dispatch and counter (one per hardware
    instance on some counters) are summed."""
    acc = collections.defaultdict(float)
    meta = {}
    for r in csv.DictReader(open(path)):
        key = (r["Dispatch_Id"], r["Counter_Name"])
        acc[key] += float(r["Counter_Value"])
        meta[r["Dispatch_Id"]] = (r["Kernel_Name"], r.get("Grid_Size", ""))
    out = collections.defaultdict(lambda: collections.defaultdict(list))
    for (disp, ctr), v in acc.items():
        out[meta[disp]][ctr].append(v)
    return out


def pmc(path, match):
    for (kern, grid), ctrs in _per_dispatch(path).items():
        if match and match not in kern:
            continue
        print("%s  [grid %s]" % (kern[:110], grid))
        for c in sorted(ctrs):
            v = ctrs[c]
            print("   %-30s mean %.5g over %d dispatches" % (c, sum(v) / len(v), len(v)))


def _kernel_mean(path, counter, substr):
    vals = []
    for (kern, _), ctrs in _per_dispatch(path).items():
        if substr in kern and counter in ctrs:
            vals += ctrs[counter]
    if not vals:
        raise SystemExit("no dispatch of a kernel matching %r with counter %s in %s" % (substr, counter, path))
    return sum(vals) / len(vals)


def traffic(a):
    f_scale = COPY_KIB / _kernel_mean(a.copy_fetch, "FETCH_SIZE", "copyBuffer")
    w_scale = COPY_KIB / _kernel_mean(a.copy_write, "WRITE_SIZE", "copyBuffer")
    total, detail = 0.0, []
    for item in a.kernels.split(","):
        name, launches = item.rsplit(":", 1)
        f = _kernel_mean(a.fetch, "FETCH_SIZE", name)
        w = _kernel_mean(a.write, "WRITE_SIZE", name)
        total += float(launches) * (f * f_scale + w * w_scale) * 1024.0
        detail.append({"kernel": name, "launches_per_step": float(launches), "fetch_kib": round(f, 1), "write_kib": round(w, 1)})
    srcs = a.sources.split(",")
    h = hashlib.sha1()
    for s in sorted(srcs):
        with open(os.path.join(HERE, "csrc", s), "rb") as fh:
            h.update(fh.read())
    print("TRAFFIC " + json.dumps({"bytes_per_step": int(total), "fetch_scale": round(f_scale, 4), "write_scale": round(w_scale, 4),
                                   "kernels": detail, "sources": sorted(srcs), "sources_sha": h.hexdigest()[:16]}))


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    p = sub.add_parser("stats")
    p.add_argument("csv")
    p.add_argument("--top", type=int, default=18)
    p = sub.add_parser("pmc")
    p.add_argument("csv")
    p.add_argument("--match", default="brg")
    p = sub.add_parser("traffic")
    for k in ("fetch", "write", "copy-fetch", "copy-write", "kernels", "sources"):
        p.add_argument("--" + k, required=True)
    a = ap.parse_args()
    if a.cmd == "stats":
        stats(a.csv, a.top)
    elif a.cmd == "pmc":
        pmc(a.csv, a.match)
    else:
        traffic(a)


if __name__ == "__main__":
    sys.exit(main())
