#!/usr/bin/env python3
"""Per-kernel text summary of a rocprofv3 result database (``*_results.db``).

    python3 rocprof_summary.py trace  <db>            # --kernel-trace run
    python3 rocprof_summary.py pmc    <db> [<db> ..]  # --pmc runs (one counter each)
    python3 rocprof_summary.py traffic <sparse pmc summary> <dense pmc summary>

``trace`` prints calls / total / average / min / max duration per kernel of this
library (kernels of other libraries, e.g. the input generators, are left out
unless ``--all`` is given).  ``pmc`` prints the average counter value per launch
for every kernel and counter found, in MiB when the counter is FETCH_SIZE or
WRITE_SIZE (rocprofv3 reports those in KiB).  ``traffic`` turns two such ``pmc``
summaries of ``bench.py`` (legs ``sparse,copycal`` and ``dense,copycal``) into HBM
bytes per entry-point call: every counter is scaled by what it reads for the 1 GiB
plain copy of the copycal leg, and the kernels of an entry point are added up.  The
output is what the files under ``profiles/`` hold.
"""
from __future__ import annotations

import sqlite3
import sys

OURS = ("k_main", "k_prep", "k_upload", "k_hist", "k_bin", "k_gather", "k_select", "k_emit", "k_full", "k_paths",
        "k_chunks", "k_subtab", "k_merge_", "k_sparse_adam", "k_combine_", "k_snapshot", "k_adam")


def _short(name: str) -> str:
    name = name.replace("(anonymous namespace)::", "").replace("void ", "")
    return name.split("(")[0].replace(", ", ",")  # no blanks: the summaries are parsed by column


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


# kernel-name prefixes (template arguments follow some of them)
COMPRESS_KERNELS = ("k_upload", "k_prep", "k_main", "k_hist", "k_bin", "k_gather", "k_select", "k_emit", "k_full")


def _table(path):
    rows = {}
    with open(path) as f:
        for line in f.read().splitlines()[1:]:
            p = line.split()
            if len(p) >= 5 and p[1] in ("FETCH_SIZE", "WRITE_SIZE"):
                rows[(p[0], p[1])] = (int(p[2]), float(p[3]))  # launches, MiB per launch
    return rows


def traffic(sparse_txt: str, dense_txt: str, compress_calls: int = 20, snapshot_iters: int = 4) -> str:
    mib = 1 << 20
    S, D = _table(sparse_txt), _table(dense_txt)
    # calibration copy: the only k_snapshot launch of the sparse run moves 1 GiB in and 1 GiB out
    ff = 1024.0 / S[("k_snapshot", "FETCH_SIZE")][1]
    fw = 1024.0 / S[("k_snapshot", "WRITE_SIZE")][1]

    def total(rows, prefixes, calls):
        f = sum(n * v for (k, c), (n, v) in rows.items() if c == "FETCH_SIZE" and k.startswith(tuple(prefixes)))
        w = sum(n * v for (k, c), (n, v) in rows.items() if c == "WRITE_SIZE" and k.startswith(tuple(prefixes)))
        return (f * ff + w * fw) / calls * mib

    snap = [k for k in ("k_snapshot", "k_snapshot_batch")]
    sf = sum(D[(k, "FETCH_SIZE")][0] * D[(k, "FETCH_SIZE")][1] for k in snap if (k, "FETCH_SIZE") in D) * ff
    sw = sum(D[(k, "WRITE_SIZE")][0] * D[(k, "WRITE_SIZE")][1] for k in snap if (k, "WRITE_SIZE") in D) * fw
    out = {
        "ld_compress_topk": total(S, COMPRESS_KERNELS, compress_calls),
        "ld_merge_sparse": total(S, ("k_chunks", "k_merge_sweep"), 1),
        "ld_snapshot_layers": (sf + sw - 2048.0) / snapshot_iters * mib,  # minus the calibration copy
        "ld_merge_dense_adam": total(D, ("k_adam",), 1),
    }
    lines = [f"# calibration (1 GiB plain copy): FETCH_SIZE x {ff:.3f}, WRITE_SIZE x {fw:.3f}"]
    for k, v in out.items():
        lines.append(f"traffic {k} {round(v)}")
    return "\n".join(lines)


def main(argv) -> int:
    if len(argv) >= 4 and argv[1] == "traffic":
        print(traffic(argv[2], argv[3]))
        return 0
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
