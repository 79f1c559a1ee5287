"""Turns a rocprofv3 result database (rocprofv3 --kernel-trace --stats ... writes *_results.db) into a
short text table: per kernel name the number of dispatches, total and average duration.

usage: python -m paper_2011_13635_amd.profile_summary <results.db> [--command "<command that made it>"]
"""
from __future__ import annotations

import argparse
import sqlite3
import sys


def summarize(db_path: str, command: str = "") -> str:
    con = sqlite3.connect(db_path)
    rows = con.execute("select name, count(*), sum(duration), avg(duration), min(duration), max(duration) "
                       "from kernels group by name order by sum(duration) desc").fetchall()
    total = sum(r[2] for r in rows) or 1
    lines = []
    if command:
        lines.append(f"command: {command}")
    lines.append(f"kernel dispatches: {sum(r[1] for r in rows)}, total kernel time {total / 1e6:.3f} ms")
    lines.append(f"{'calls':>7} {'total_us':>11} {'avg_us':>9} {'min_us':>9} {'max_us':>9} {'%':>6}  kernel")
    for name, n, tot, avg, mn, mx in rows:
        lines.append(f"{n:7d} {tot / 1e3:11.1f} {avg / 1e3:9.2f} {mn / 1e3:9.2f} {mx / 1e3:9.2f} {100 * tot / total:6.2f}  {name}")
    # the MFMA GEMM is one templated kernel: its variants together, for comparison with bench.py's avg_launch_us
    g = [r for r in rows if "k_gemm_mfma" in r[0]]
    if g:
        n, tot = sum(r[1] for r in g), sum(r[2] for r in g)
        lines.append(f"k_gemm_mfma, all variants: {n} dispatches, avg {tot / n / 1e3:.2f} us, {100 * tot / total:.2f} % of kernel time")
    return "\n".join(lines) + "\n"


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("db")
    ap.add_argument("--command", default="")
    args = ap.parse_args()
    sys.stdout.write(summarize(args.db, args.command))


if __name__ == "__main__":
    main()
