"""Turn rocprofv3 CSV output into the short text summaries kept under profiles/.

  python -m paper_2401_14021_amd.prof_summary trace <dir> [--label TEXT]
      <dir> holds *_kernel_trace.csv from `rocprofv3 --kernel-trace --stats --output-format csv`.
      Prints per-kernel call counts and average durations; launches of the scan kernels are
      grouped into duration classes, because one retrieval call launches the same kernel
      several times (the stages of its ladder, which differ in size by the growth factors).

  python -m paper_2401_14021_amd.prof_summary pmc <dir>
      <dir> holds *_counter_collection.csv from `rocprofv3 --pmc ... --output-format csv`.
      Prints, per kernel and launch-duration class, the mean and the sum of each counter.
"""
from __future__ import annotations

import collections
import csv
import glob
import os
import re
import sys


def _short(name: str) -> str:
    name = re.sub(r"\(anonymous namespace\)::", "", name)
    name = re.sub(r"^void ", "", name)
    return name.split("(")[0][:90]


def _rows(d: str, pat: str):
    files = sorted(glob.glob(os.path.join(d, "**", pat), recursive=True))
    if not files:
        raise SystemExit(f"no {pat} under {d}")
    for f in files:
        with open(f, newline="") as fh:
            yield from csv.DictReader(fh)


def trace(d: str) -> None:
    per = collections.defaultdict(list)
    for r in _rows(d, "*kernel_trace.csv"):
        per[_short(r["Kernel_Name"])].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    total = sum(sum(v) for v in per.values())
    print(f"{'kernel':92s} {'calls':>6s} {'avg_us':>10s} {'total_ms':>9s} {'share':>6s}")
    for k, v in sorted(per.items(), key=lambda kv: -sum(kv[1])):
        if sum(v) / total < 0.002 and "ralm" not in k:
            continue
        if "scan_" in k and len(v) > 1:
            # one retrieval call launches the scan several times on very different row counts:
            # group launches whose durations are within a factor 1.5 of each other
            classes, cur = [], []
            for x in sorted(v, reverse=True):
                if cur and cur[0] > 1.5 * x:
                    classes.append(cur)
                    cur = []
                cur.append(x)
            classes.append(cur)
            for c in classes:
                print(f"{k + f' [launch class ~{c[0]/1e3:.2f} ms]':92s} {len(c):6d} {sum(c)/len(c):10.1f} "
                      f"{sum(c)/1e3:9.2f} {100*sum(c)/total:5.1f}%")
        else:
            print(f"{k:92s} {len(v):6d} {sum(v)/len(v):10.1f} {sum(v)/1e3:9.2f} {100*sum(v)/total:5.1f}%")


def _classes(vals):
    """Group (duration, value) pairs whose durations are within a factor 1.5 of each other."""
    out, cur = [], []
    for v in sorted(vals, reverse=True):
        if cur and cur[0][0] > 1.5 * v[0]:
            out.append(cur)
            cur = []
        cur.append(v)
    out.append(cur)
    return out


def pmc(d: str) -> None:
    per = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in _rows(d, "*counter_collection.csv"):
        k = _short(r["Kernel_Name"])
        if "ralm" not in k:
            continue
        dur = int(r["End_Timestamp"]) - int(r["Start_Timestamp"])
        per[k][r["Counter_Name"]].append((dur, float(r["Counter_Value"])))
    for k, cs in sorted(per.items()):
        print(k)
        for c, vals in sorted(cs.items()):
            for cl in _classes(vals):
                print(f"    {c:24s} launches={len(cl):3d} mean={sum(v[1] for v in cl)/len(cl):.6g} "
                      f"sum={sum(v[1] for v in cl):.6g} mean_duration_us={sum(v[0] for v in cl)/len(cl)/1e3:.1f}")


if __name__ == "__main__":
    if len(sys.argv) < 3 or sys.argv[1] not in ("trace", "pmc"):
        raise SystemExit(__doc__)
    (trace if sys.argv[1] == "trace" else pmc)(sys.argv[2])
