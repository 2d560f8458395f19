"""Turns a rocprofv3 result database (rocpd SQLite, the default output of `rocprofv3 ... -d DIR -o NAME`)
into the short text summaries kept under profiles/: per-kernel call counts and durations, and, for a
`--pmc` run, the mean counter values per kernel.

    python -m paper_2505_19342_amd.rocprof_summary DIR/NAME_results.db [--skip-first N]
"""
from __future__ import annotations

import argparse
import collections
import sqlite3


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("db")
    ap.add_argument("--skip-first", type=int, default=0, help="ignore the first N dispatches of every kernel (warm-up)")
    args = ap.parse_args()
    con = sqlite3.connect(args.db)
    cur = con.cursor()
    rows = cur.execute("select name, duration from kernels order by start").fetchall()
    per = collections.OrderedDict()
    for name, dur in rows:
        per.setdefault(name, []).append(dur)
    total = sum(sum(v[args.skip_first:]) for v in per.values()) or 1
    print(f"{'calls':>6} {'avg_us':>10} {'min_us':>10} {'max_us':>10} {'share':>7}  kernel")
    for name, durs in sorted(per.items(), key=lambda kv: -sum(kv[1][args.skip_first:])):
        d = durs[args.skip_first:] or durs
        print(f"{len(d):6d} {sum(d) / len(d) / 1e3:10.2f} {min(d) / 1e3:10.2f} {max(d) / 1e3:10.2f} {sum(d) / total:7.1%}  {name[:110]}")
    try:
        crow = cur.execute("select kernel_name, counter_name, value, dispatch_id from counters_collection order by dispatch_id").fetchall()
    except sqlite3.Error:
        crow = []
    if crow:
        agg = collections.OrderedDict()
        seen = collections.Counter()
        last = {}
        for k, c, v, did in crow:
            if last.get((k, c)) != did:
                seen[(k, c)] += 1
                last[(k, c)] = did
            if seen[(k, c)] <= args.skip_first:
                continue
            a = agg.setdefault((k, c), [0.0, set()])
            a[0] += v
            a[1].add(did)
        print("\nmean counter value per dispatch (summed over the counter's instances)")
        for (k, c), (s, dids) in agg.items():
            print(f"  {c:28s} {s / max(len(dids), 1):18.1f}  {k[:90]}")


if __name__ == "__main__":
    main()
