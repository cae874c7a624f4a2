"""Condense rocprofv3 CSV output into the few figures a roofline needs.

    python -m paper_2504_15364_amd.rocprof_summary stats   <dir> [--first K]  # --kernel-trace --stats run
    python -m paper_2504_15364_amd.rocprof_summary counter <dir> <COUNTER> [--copy-bytes N]

`stats` prints, per kernel, launches / average / median / min / max duration from the
kernel trace; with --first K also the average over the first K launches of each kernel in
time order (bench.py runs its timed steady-state steps first, the secondary measurements
after them).  `counter` prints the per-dispatch mean of one hardware counter for each
kernel of this library and, when --copy-bytes is given, the same counter for the plain
copy kernel of that size the benchmark ran for calibration (bench.py --pmc-calibration),
with the resulting bytes-per-count factor and the calibrated per-launch byte count.
Reads files only; touches no GPU.
"""
from __future__ import annotations

import collections
import csv
import glob
import os
import sys


def _find(root, suffix):
    hits = sorted(glob.glob(os.path.join(root, "**", "*" + suffix), recursive=True))
    if not hits:
        sys.exit(f"no *{suffix} under {root}")
    return hits


def short(name):
    name = name.split("(")[0]
    return name.replace("void ", "").replace("kd::", "")[-64:]


def stats(root, first=0):
    rows = []
    for f in _find(root, "kernel_trace.csv"):
        rows += list(csv.DictReader(open(f)))
    rows.sort(key=lambda r: int(r["Start_Timestamp"]))
    agg = collections.defaultdict(list)
    for r in rows:
        agg[short(r["Kernel_Name"])].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    total = sum(sum(v) for v in agg.values())
    head = f"{'avg_first_' + str(first):>16s}" if first else ""
    print(f"{'kernel':64s} {'calls':>7s} {'avg_us':>9s} {'med_us':>9s} {'min_us':>9s} {'max_us':>9s} {'%time':>6s}{head}")
    for k, v in sorted(agg.items(), key=lambda kv: -sum(kv[1])):
        s = sorted(v)
        extra = f"{sum(v[:first]) / len(v[:first]):16.2f}" if first else ""
        print(f"{k:64s} {len(v):7d} {sum(v) / len(v):9.2f} {s[len(v) // 2]:9.2f} {s[0]:9.2f} {s[-1]:9.2f} "
              f"{100 * sum(v) / total:6.1f}{extra}")


def counter(root, name, copy_bytes):
    rows = []
    for f in _find(root, "counter_collection.csv"):
        rows += list(csv.DictReader(open(f)))
    agg = collections.defaultdict(list)
    for r in rows:
        if r["Counter_Name"] == name:
            agg[short(r["Kernel_Name"])].append(float(r["Counter_Value"]))
    factor = None
    if copy_bytes:
        # the calibration copy is the only launch that moves exactly copy_bytes: pick the kernel whose
        # name says copy/elementwise and whose count is the largest
        cands = {k: v for k, v in agg.items() if "copy" in k.lower() or "elementwise" in k.lower()}
        if cands:
            k = max(cands, key=lambda k: max(cands[k]))
            top = max(cands[k])
            vals = [x for x in cands[k] if x > 0.5 * top]
            mean = sum(vals) / len(vals)
            factor = copy_bytes / mean
            print(f"calibration: {k}  n={len(vals)}  mean {name} = {mean:.1f}  for {copy_bytes} bytes "
                  f"-> {factor:.2f} bytes per count")
    print(f"{'kernel':64s} {'n':>6s} {'mean ' + name:>20s} {'calibrated bytes':>18s}")
    for k, v in sorted(agg.items()):
        if "step_" not in k and "compact" not in k and "merge" not in k and "ksum" not in k:
            continue
        m = sum(v) / len(v)
        cal = f"{m * factor:18.0f}" if factor else f"{'-':>18s}"
        print(f"{k:64s} {len(v):6d} {m:20.1f} {cal}")


def main(argv):
    if len(argv) >= 2 and argv[0] == "stats":
        stats(argv[1], int(argv[argv.index("--first") + 1]) if "--first" in argv else 0)
    elif len(argv) >= 3 and argv[0] == "counter":
        cb = int(argv[argv.index("--copy-bytes") + 1]) if "--copy-bytes" in argv else 0
        counter(argv[1], argv[2], cb)
    else:
        sys.exit(__doc__)


if __name__ == "__main__":
    main(sys.argv[1:])
