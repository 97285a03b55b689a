"""Summarises rocprofv3 CSV output: per-kernel launch counts, average duration and
average counter values.  Usage: python -m paper_2604_24273_amd.profile_summary <output-dir>"""
from __future__ import annotations

import collections
import csv
import glob
import os
import sys


def summarise(root: str) -> str:
    lines = []
    for path in sorted(glob.glob(os.path.join(root, "**", "*kernel_trace.csv"), recursive=True)):
        dur = collections.defaultdict(list)
        for r in csv.DictReader(open(path)):
            dur[r["Kernel_Name"]].append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
        total = sum(sum(v) for v in dur.values()) or 1
        lines.append("# kernel trace: %s" % os.path.relpath(path, root))
        lines.append("%-88s %8s %12s %12s %7s" % ("kernel", "calls", "avg_us", "total_ms", "share"))
        for k, v in sorted(dur.items(), key=lambda kv: -sum(kv[1])):
            lines.append("%-88s %8d %12.2f %12.3f %6.1f%%" % (k[:88], len(v), sum(v) / len(v) / 1e3, sum(v) / 1e6,
                                                              100.0 * sum(v) / total))
    for path in sorted(glob.glob(os.path.join(root, "**", "*counter_collection.csv"), recursive=True)):
        agg = collections.defaultdict(lambda: collections.defaultdict(list))
        for r in csv.DictReader(open(path)):
            agg[r["Kernel_Name"]][r["Counter_Name"]].append(float(r["Counter_Value"]))
        lines.append("# counters: %s (average per dispatch)" % os.path.relpath(path, root))
        for k, d in sorted(agg.items()):
            for c, v in sorted(d.items()):
                lines.append("%-88s %-28s %8d dispatches  avg %.6g" % (k[:88], c, len(v), sum(v) / len(v)))
    return "\n".join(lines)


if __name__ == "__main__":
    print(summarise(sys.argv[1] if len(sys.argv) > 1 else "."))
