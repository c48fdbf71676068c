#!/usr/bin/env python3
"""Turn a rocprofv3 result database (rocpd sqlite, the default output) into a short text table.

    python -m paper_2008_01425_amd.rocprof_summary RESULTS.db [--pmc]

Without --pmc: per kernel name and grid size, the number of dispatches and the average / min /
max duration (what `rocprofv3 --kernel-trace --stats` collected).  With --pmc: per kernel, the
average per-dispatch value of every collected counter.
"""
from __future__ import annotations

import collections
import re
import sqlite3
import sys


def _short(name: str) -> str:
    return re.sub(r"\(.*", "", name).replace("void ", "")


def kernel_stats(path: str) -> str:
    cur = sqlite3.connect(path).cursor()
    cols = [r[1] for r in cur.execute("pragma table_info(kernels)")]
    ix = {c: i for i, c in enumerate(cols)}
    agg = collections.defaultdict(list)
    for r in cur.execute("select * from kernels"):
        agg[(_short(r[ix["name"]]), r[ix["grid_x"]])].append(r[ix["end"]] - r[ix["start"]])
    tot = sum(sum(v) for v in agg.values()) or 1
    out = [f"{'kernel':58s} {'grid_x':>9s} {'calls':>6s} {'avg_us':>9s} {'min_us':>9s} {'max_us':>9s} {'total_ms':>9s} {'%':>6s}"]
    for (k, g), v in sorted(agg.items(), key=lambda kv: -sum(kv[1])):
        out.append(f"{k[:58]:58s} {g:9d} {len(v):6d} {sum(v)/len(v)/1e3:9.2f} {min(v)/1e3:9.2f} "
                   f"{max(v)/1e3:9.2f} {sum(v)/1e6:9.3f} {100*sum(v)/tot:6.2f}")
    return "\n".join(out)


def pmc_stats(path: str) -> str:
    cur = sqlite3.connect(path).cursor()
    cols = [r[1] for r in cur.execute("pragma table_info(counters_collection)")]
    ix = {c: i for i, c in enumerate(cols)}
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in cur.execute("select * from counters_collection"):
        agg[(_short(r[ix["kernel_name"]]), r[ix["grid_size"]])][r[ix["counter_name"]]].append(r[ix["value"]])
    out = [f"{'kernel':58s} {'grid':>9s} {'counter':>14s} {'dispatches':>10s} {'avg/dispatch':>16s}"]
    for (k, g), d in sorted(agg.items(), key=lambda kv: -sum(sum(v) for v in kv[1].values())):
        for cname, v in sorted(d.items()):
            out.append(f"{k[:58]:58s} {g:9d} {cname:>14s} {len(v):10d} {sum(v)/len(v):16.1f}")
    return "\n".join(out)


if __name__ == "__main__":
    if len(sys.argv) < 2:
        sys.exit(__doc__)
    print(pmc_stats(sys.argv[1]) if "--pmc" in sys.argv[2:] else kernel_stats(sys.argv[1]))
