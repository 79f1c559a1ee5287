"""Turns a rocprofv3 result database (rocprofv3 --kernel-trace --stats ... writes *_results.db) into a
short text table: per kernel name the number of dispatches, total and average duration.

usage: python -m paper_2011_13635_amd.profile_summary <results.db> [--command "<command that made it>"] [--last-steps N]

--last-steps N adds a second table over the last N steps only (a step starts at its k_batch_scan dispatch).
bench.py runs its per-class event timing last, with the side stream off, so those are the steps in which every
kernel ran alone: their durations are the ones bench.py's roofline figure is to be compared with.
"""
from __future__ import annotations

import argparse
import sqlite3
import sys


def summarize(db_path: str, command: str = "", last_steps: int = 0) -> str:
    con = sqlite3.connect(db_path)
    rows = con.execute("select name, count(*), sum(duration), avg(duration), min(duration), max(duration) "
                       "from kernels group by name order by sum(duration) desc").fetchall()
    out = table(rows, command)
    if last_steps > 0:
        starts = [r[0] for r in con.execute("select start from kernels where name like '%k_batch_scan%' order by start")]
        if len(starts) >= last_steps:
            t0 = starts[-last_steps]
            rows = con.execute("select name, count(*), sum(duration), avg(duration), min(duration), max(duration) "
                               "from kernels where start >= ? group by name order by sum(duration) desc", (t0,)).fetchall()
            out += f"\nlast {last_steps} steps only (event-timing pass of bench.py: one stream, every kernel alone)\n"
            out += table(rows, "", per_step=last_steps)
    return out


def table(rows, command: str = "", per_step: int = 0) -> str:
    total = sum(r[2] for r in rows) or 1
    lines = []
    if command:
        lines.append(f"command: {command}")
    lines.append(f"kernel dispatches: {sum(r[1] for r in rows)}, total kernel time {total / 1e6:.3f} ms")
    lines.append(f"{'calls':>7} {'total_us':>11} {'avg_us':>9} {'min_us':>9} {'max_us':>9} {'%':>6}  kernel")
    for name, n, tot, avg, mn, mx in rows:
        lines.append(f"{n:7d} {tot / 1e3:11.1f} {avg / 1e3:9.2f} {mn / 1e3:9.2f} {mx / 1e3:9.2f} {100 * tot / total:6.2f}  {name}")
    # the MFMA GEMMs are two templated kernels: their variants together, for comparison with bench.py's avg_launch_us
    g = [r for r in rows if "k_gemm_mfma" in r[0] or "k_gemm_ring" in r[0]]
    if g:
        n, tot = sum(r[1] for r in g), sum(r[2] for r in g)
        lines.append(f"GEMM kernels (k_gemm_ring + k_gemm_mfma), all variants: {n} dispatches, avg {tot / n / 1e3:.2f} us, {100 * tot / total:.2f} % of kernel time")
        if per_step:
            lines.append(f"GEMM kernels per step: {n / per_step:.1f} dispatches, {tot / per_step / 1e6:.4f} ms"
                         f" (+ k_splitk_reduce {sum(r[2] for r in rows if 'k_splitk_reduce' in r[0]) / per_step / 1e6:.4f} ms)")
    return "\n".join(lines) + "\n"


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("db")
    ap.add_argument("--command", default="")
    ap.add_argument("--last-steps", type=int, default=0)
    args = ap.parse_args()
    sys.stdout.write(summarize(args.db, args.command, args.last_steps))


if __name__ == "__main__":
    main()
