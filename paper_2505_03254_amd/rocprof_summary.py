"""Turns rocprofv3 CSV output into the short text summaries kept under profiles/.

  python -m paper_2505_03254_amd.rocprof_summary stats <name>_kernel_stats.csv
      per-kernel call count and average / min / max duration of this library's kernels

  python -m paper_2505_03254_amd.rocprof_summary traffic <fetch>_counter_collection.csv \
          <write>_counter_collection.csv --copy-bytes <bytes copied per prom::copy_kernel launch>
      HBM bytes per launch of every kernel from the FETCH_SIZE and WRITE_SIZE counters (KiB per
      dispatch), each scaled by what the same counter reads for prom::copy_kernel, which moves a
      known number of bytes in each direction.

  python -m paper_2505_03254_amd.rocprof_summary counters <a>_counter_collection.csv [<b>_... ...]
      average per launch of every counter in the given files, per kernel (optionally only
      kernels whose name contains --match)
"""
from __future__ import annotations

import argparse
import collections
import csv
import sys

OURS = ("prom::",)


def _is_ours(name: str) -> bool:
    return any(tag in name for tag in OURS)


def stats(path: str) -> None:
    rows = [r for r in csv.DictReader(open(path)) if _is_ours(r["Name"])]
    print(f"{'kernel':<78}{'calls':>7}{'avg us':>10}{'min us':>10}{'max us':>10}{'% time':>8}")
    for r in rows:
        print(f"{r['Name'][:76]:<78}{int(r['Calls']):>7}{float(r['AverageNs']) / 1e3:>10.2f}"
              f"{float(r['MinNs']) / 1e3:>10.2f}{float(r['MaxNs']) / 1e3:>10.2f}{float(r['Percentage']):>8.2f}")


def _per_kernel(path: str, counter: str):
    agg = collections.OrderedDict()
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] != counter or not _is_ours(r["Kernel_Name"]):
            continue
        agg.setdefault(r["Kernel_Name"], []).append(float(r["Counter_Value"]))
    return agg


def traffic(fetch_csv: str, write_csv: str, copy_bytes: int) -> None:
    fetch = _per_kernel(fetch_csv, "FETCH_SIZE")
    write = _per_kernel(write_csv, "WRITE_SIZE")
    copy_name = next(k for k in fetch if "copy_kernel" in k)
    f_scale = copy_bytes / 1024.0 / (sum(fetch[copy_name]) / len(fetch[copy_name]))
    w_scale = copy_bytes / 1024.0 / (sum(write[copy_name]) / len(write[copy_name]))
    print(f"# counters are KiB per dispatch; scale factors from prom::copy_kernel "
          f"({copy_bytes} bytes each way): FETCH_SIZE x {f_scale:.4f}, WRITE_SIZE x {w_scale:.4f}")
    print(f"{'kernel':<78}{'launches':>9}{'read MB':>10}{'write MB':>10}{'total MB':>10}")
    for k in fetch:
        if k not in write:
            continue
        rd = f_scale * 1024.0 * sum(fetch[k]) / len(fetch[k])
        wr = w_scale * 1024.0 * sum(write[k]) / len(write[k])
        print(f"{k[:76]:<78}{len(fetch[k]):>9}{rd / 1e6:>10.2f}{wr / 1e6:>10.2f}{(rd + wr) / 1e6:>10.2f}")
    print()
    for k in fetch:
        if k in write and "copy_kernel" not in k:
            rd = f_scale * 1024.0 * sum(fetch[k]) / len(fetch[k])
            wr = w_scale * 1024.0 * sum(write[k]) / len(write[k])
            print(f"traffic_bytes_per_launch[{k}] = {int(rd + wr)}")


def counters(paths, match: str) -> None:
    agg = collections.OrderedDict()
    for path in paths:
        for r in csv.DictReader(open(path)):
            k = r["Kernel_Name"]
            if not _is_ours(k) or (match and match not in k):
                continue
            agg.setdefault(k, collections.OrderedDict()).setdefault(r["Counter_Name"], []).append(
                float(r["Counter_Value"]))
    for k, cs in agg.items():
        print(k[:100])
        for c, v in cs.items():
            print(f"    {c:<34}{sum(v) / len(v):>16.0f}   (launches: {len(v)})")


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    s = sub.add_parser("stats")
    s.add_argument("csv")
    t = sub.add_parser("traffic")
    t.add_argument("fetch_csv")
    t.add_argument("write_csv")
    t.add_argument("--copy-bytes", type=int, required=True)
    c = sub.add_parser("counters")
    c.add_argument("csv", nargs="+")
    c.add_argument("--match", default="")
    a = ap.parse_args(argv)
    if a.cmd == "stats":
        stats(a.csv)
    elif a.cmd == "counters":
        counters(a.csv, a.match)
    else:
        traffic(a.fetch_csv, a.write_csv, a.copy_bytes)
    return 0


if __name__ == "__main__":
    sys.exit(main())
