#!/usr/bin/env python3
"""Turn a rocprofv3 result database (rocpd sqlite, the default output) into a short text table.

    python -m paper_2008_01425_amd.rocprof_summary RESULTS.db [--pmc]
    python -m paper_2008_01425_amd.rocprof_summary --traffic FETCH.db WRITE.db CALIBRATION_MiB

Without --pmc: per kernel name and grid size, the number of dispatches and the average / min /
max duration (what `rocprofv3 --kernel-trace --stats` collected).  With --pmc: per kernel, the
average per-dispatch value of every collected counter.  --traffic: from one FETCH_SIZE and one
WRITE_SIZE run of `bench.py --counters MiB`, the bytes per launch of every kernel kind that
crossed the L2 -> fabric boundary, each counter scaled by what it reads for the plain device
copies of known size at the end of that run; the `traffic <kind> <read> <written> <total>`
lines are what bench.py reads back from profiles/.
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


def kernel_kind(name: str):
    """Kernel name -> the kind pg_profile_collect reports it under (None: not a pass over X)."""
    m = re.match(r"pg::(row_kernel|row_wide_kernel|mrow_kernel|vec_row_kernel)<(.*)>", name)
    if m:
        upd, swp, grad = [t.strip() == "true" for t in m.group(2).split(",")[-3:]]
        if grad:
            return "update_sgd"
        return "update_sweep_p" if upd and swp else ("update" if upd else "sweep_p")
    if re.match(r"pg::(col_kernel|mcol_kernel|vec_col_kernel)<", name):
        return "sweep_q"
    return None


def _counter_avgs(path: str, counter: str):
    """{(kernel, grid): (dispatches, average value per dispatch)} of one counter."""
    cur = sqlite3.connect(path).cursor()
    cols = [r[1] for r in cur.execute("pragma table_info(counters_collection)")]
    ix = {c: i for i, c in enumerate(cols)}
    agg = collections.defaultdict(list)
    for r in cur.execute("select * from counters_collection"):
        if r[ix["counter_name"]] == counter:
            agg[(_short(r[ix["kernel_name"]]), r[ix["grid_size"]])].append(r[ix["value"]])
    return {k: (len(v), sum(v) / len(v)) for k, v in agg.items()}


def traffic(fetch_db: str, write_db: str, calib_mib: int) -> str:
    fetch, write = _counter_avgs(fetch_db, "FETCH_SIZE"), _counter_avgs(write_db, "WRITE_SIZE")
    known_kib = calib_mib * 1024.0

    def factor(tab):
        # the calibration copies: the copy kernel's dispatches with the largest grid
        copies = {k: v for k, v in tab.items() if "copyBuffer" in k[0]}
        key = max(copies, key=lambda k: k[1])
        return known_kib / copies[key][1], copies[key]
    ff, fc = factor(fetch)
    wf, wc = factor(write)
    out = [f"calibration: {fc[0]} plain device copies of {calib_mib} MiB each read and write {known_kib:.0f} KiB;",
           f"  FETCH_SIZE reads {fc[1]:.1f} KiB per copy -> scale factor {ff:.3f}; WRITE_SIZE reads {wc[1]:.1f} KiB -> scale factor {wf:.3f}",
           "",
           f"{'kernel':58s} {'grid':>9s} {'kind':>15s} {'launches':>8s} {'read MB':>10s} {'written MB':>11s}"]
    kinds = collections.defaultdict(lambda: [0.0, 0.0])
    for key in sorted(fetch, key=lambda k: -fetch[k][1]):
        kind = kernel_kind(key[0])
        if kind is None:
            continue
        rd = fetch[key][1] * ff * 1024.0
        wr = write.get(key, (0, 0.0))[1] * wf * 1024.0
        kinds[kind][0] += rd
        kinds[kind][1] += wr
        out.append(f"{key[0][:58]:58s} {key[1]:9d} {kind:>15s} {fetch[key][0]:8d} {rd / 1e6:10.1f} {wr / 1e6:11.1f}")
    out += ["", "bytes per launch of a kernel kind (summed over that kind's kernel instantiations, each of which",
            "runs once per pass); 1 KiB = 1024 B:"]
    for kind, (rd, wr) in sorted(kinds.items()):
        out.append(f"traffic {kind} {rd:.0f} {wr:.0f} {rd + wr:.0f}")
    return "\n".join(out)


if __name__ == "__main__":
    if len(sys.argv) < 2:
        sys.exit(__doc__)
    if sys.argv[1] == "--traffic":
        print(traffic(sys.argv[2], sys.argv[3], int(sys.argv[4])))
        sys.exit(0)
    print(pmc_stats(sys.argv[1]) if "--pmc" in sys.argv[2:] else kernel_stats(sys.argv[1]))
