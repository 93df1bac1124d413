"""Turn the CSV files of a rocprofv3 run into the short markdown tables kept under profiles/.

    python -m paper_1609_01882_amd.benchmarks.profile_summary stats  DIR            # per-kernel calls / avg / min / max
    python -m paper_1609_01882_amd.benchmarks.profile_summary trace  DIR [--tail N] # the last N launches, in order
    python -m paper_1609_01882_amd.benchmarks.profile_summary pmc    DIR            # counter means per kernel and launch

DIR is what was given to rocprofv3 as `-d`; only the library's own kernels (namespace psc) and the
runtime's copy kernel (the calibration copy) are listed."""
from __future__ import annotations

import collections
import csv
import glob
import sys


def short(name: str) -> str:
    return name.replace("void ", "").replace("psc::(anonymous namespace)::", "").replace("psc::", "").split("(")[0]


def _find(d: str, pattern: str) -> str:
    hits = glob.glob(f"{d}/**/*{pattern}", recursive=True)
    if not hits:
        raise SystemExit(f"no *{pattern} under {d}")
    return hits[0]


def _ours(name: str) -> bool:
    return "psc::" in name or "copyBuffer" in name


def stats(d: str) -> str:
    rows = [r for r in csv.DictReader(open(_find(d, "kernel_stats.csv"))) if _ours(r["Name"])]
    out = ["| kernel | calls | avg (us) | min (us) | max (us) |", "|---|---|---|---|---|"]
    for r in rows:
        out.append(f"| `{short(r['Name'])}` | {r['Calls']} | {float(r['AverageNs']) / 1e3:.1f} | "
                   f"{int(r['MinNs']) / 1e3:.1f} | {int(r['MaxNs']) / 1e3:.1f} |")
    return "\n".join(out)


def trace(d: str, tail: int) -> str:
    rows = [r for r in csv.DictReader(open(_find(d, "kernel_trace.csv"))) if _ours(r["Kernel_Name"])]
    rows.sort(key=lambda r: int(r["Start_Timestamp"]))
    out = ["| kernel | us |", "|---|---|"]
    total = 0.0
    for r in rows[-tail:]:
        us = (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3
        total += us
        out.append(f"| `{short(r['Kernel_Name'])}` | {us:.1f} |")
    out.append(f"\nSum of these kernel durations: {total / 1e3:.3f} ms.")
    return "\n".join(out)


def pmc(d: str) -> str:
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(_find(d, "counter_collection.csv"))):
        if _ours(r["Kernel_Name"]):
            acc[short(r["Kernel_Name"])][r["Counter_Name"]].append(float(r["Counter_Value"]))
    out = ["| kernel | counter | launches | mean | max |", "|---|---|---|---|---|"]
    for k in sorted(acc):
        for c in sorted(acc[k]):
            v = acc[k][c]
            out.append(f"| `{k}` | {c} | {len(v)} | {sum(v) / len(v):.6g} | {max(v):.6g} |")
    return "\n".join(out)


def main(argv):
    if len(argv) < 3 or argv[1] not in ("stats", "trace", "pmc"):
        raise SystemExit(__doc__)
    if argv[1] == "stats":
        print(stats(argv[2]))
    elif argv[1] == "trace":
        tail = int(argv[argv.index("--tail") + 1]) if "--tail" in argv else 40
        print(trace(argv[2], tail))
    else:
        print(pmc(argv[2]))


if __name__ == "__main__":
    main(sys.argv)
