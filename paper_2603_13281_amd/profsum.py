"""Turn a rocprofv3 results database (rocpd sqlite) into a short text summary.

    python -m paper_2603_13281_amd.profsum <results.db> [--copy-bytes N]

Prints the per-kernel call count / total / average duration table (kernel-trace runs) and, for
--pmc runs, the average counter value per kernel.  With --copy-bytes N the value of FETCH_SIZE /
WRITE_SIZE (KiB) of the plain copy kernel that moved N bytes gives the scale factor
(bytes really moved per counted KiB) that is applied to the other kernels.
"""
from __future__ import annotations

import argparse
import sqlite3


def short(name: str) -> str:
    name = name.replace("void ", "").replace("icarus::(anonymous namespace)::", "icarus::")
    cut = name.find("(")
    return (name if cut < 0 else name[:cut])[:72]


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("db")
    ap.add_argument("--copy-bytes", type=float, default=0.0)
    ap.add_argument("--copy-kernel", default="bench_copy", help="substring naming the calibration copy kernel")
    args = ap.parse_args()
    c = sqlite3.connect(args.db).cursor()
    tables = {r[0] for r in c.execute("select name from sqlite_master where type in ('table','view')")}
    if "top_kernels" in tables:
        rows = list(c.execute("select name, total_calls, total_duration, average, percentage from top_kernels"))
        if rows:
            print(f"{'kernel':72s} {'calls':>7s} {'total_us':>12s} {'avg_us':>10s} {'%':>6s}")
            for name, calls, tot, avg, pct in rows[:25]:
                print(f"{short(name):72s} {calls:7d} {tot:12.1f} {avg:10.2f} {pct:6.2f}")
    if "counters_collection" in tables:
        q = ("select kernel_name, counter_name, avg(value), count(*), avg(duration) from counters_collection "
             "group by kernel_name, counter_name")
        rows = list(c.execute(q))
        if rows:
            factor = {}
            if args.copy_bytes:
                for k, cn, v, n, dur in rows:
                    if args.copy_kernel in k and v:
                        factor[cn] = args.copy_bytes / (v * 1024.0)
                        print(f"calibration: copy kernel moved {args.copy_bytes:.0f} bytes, {cn} read {v:.0f} KiB "
                              f"-> {factor[cn]:.3f} bytes per counted byte")
            print(f"{'kernel':72s} {'counter':>12s} {'avg_value':>14s} {'n':>5s} {'avg_us':>9s} {'scaled_MB':>10s}")
            for k, cn, v, n, dur in sorted(rows, key=lambda r: -(r[4] or 0)):
                scaled = f"{v * 1024 * factor[cn] / 1e6:10.1f}" if cn in factor else ""
                print(f"{short(k):72s} {cn:>12s} {v:14.1f} {n:5d} {(dur or 0) / 1e3:9.1f} {scaled}")


if __name__ == "__main__":
    main()
