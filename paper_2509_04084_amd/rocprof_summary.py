#!/usr/bin/env python3
"""Per-kernel text summary of a rocprofv3 result database (``*_results.db``).

    python3 -m paper_2509_04084_amd.rocprof_summary trace  <db>            # --kernel-trace run
    python3 -m paper_2509_04084_amd.rocprof_summary pmc    <db> [<db> ..]  # --pmc runs (one counter each)

``trace`` prints calls / total / average / min / max duration per kernel of this
library (kernels of other libraries, e.g. the input generators, are left out
unless ``--all`` is given).  ``pmc`` prints the average counter value per launch
for every kernel and counter found, in MiB when the counter is FETCH_SIZE or
WRITE_SIZE (rocprofv3 reports those in KiB).  The output is what the files under
``profiles/`` hold.
"""
from __future__ import annotations

import sqlite3
import sys

OURS = ("k_main", "k_prep", "k_upload", "k_hist", "k_bin", "k_gather", "k_select", "k_emit", "k_full_",
        "k_chunks", "k_merge_", "k_sparse_adam", "k_combine_", "k_snapshot", "k_adam")


def _short(name: str) -> str:
    name = name.replace("(anonymous namespace)::", "").replace("void ", "")
    return name.split("(")[0]


def _ours(name: str) -> bool:
    return any(tag in name for tag in OURS)


def trace(db_path: str, everything: bool = False) -> str:
    cur = sqlite3.connect(db_path).cursor()
    rows = cur.execute("select name, count(*), sum(end-start)/1e6, avg(end-start)/1e3, min(end-start)/1e3, "
                       "max(end-start)/1e3 from kernels group by name order by 3 desc").fetchall()
    out = [f"{'kernel':28s} {'calls':>6s} {'total_ms':>10s} {'avg_us':>10s} {'min_us':>10s} {'max_us':>10s}"]
    for name, calls, tot, avg, mn, mx in rows:
        if everything or _ours(name):
            out.append(f"{_short(name)[:28]:28s} {calls:6d} {tot:10.3f} {avg:10.1f} {mn:10.1f} {mx:10.1f}")
    return "\n".join(out)


def pmc(db_paths) -> str:
    out = [f"{'kernel':28s} {'counter':12s} {'launches':>8s} {'avg/launch':>14s} {'avg_us':>10s}"]
    for db_path in db_paths:
        cur = sqlite3.connect(db_path).cursor()
        rows = cur.execute("select kernel_name, counter_name, count(*), avg(value), avg(duration)/1e3 "
                           "from counters_collection group by kernel_name, counter_name "
                           "order by sum(duration) desc").fetchall()
        for name, counter, cnt, val, dur in rows:
            if not _ours(name):
                continue
            if counter in ("FETCH_SIZE", "WRITE_SIZE"):
                shown = f"{val / 1024.0:10.2f} MiB"
            else:
                shown = f"{val:14.1f}"
            out.append(f"{_short(name)[:28]:28s} {counter:12s} {cnt:8d} {shown:>14s} {dur:10.1f}")
    return "\n".join(out)


def main(argv) -> int:
    if len(argv) < 3 or argv[1] not in ("trace", "pmc"):
        print(__doc__)
        return 2
    if argv[1] == "trace":
        print(trace(argv[2], everything="--all" in argv[3:]))
    else:
        print(pmc(argv[2:]))
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
