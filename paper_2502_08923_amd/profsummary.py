"""Turn a rocprofv3 `--kernel-trace` result database into a short per-kernel text table.

    python -m paper_2502_08923_amd.profsummary <output dir>/bench_results.db [--skip N]

Only reads the database rocprofv3 wrote; runs nothing on the GPU.
"""
from __future__ import annotations

import argparse
import sqlite3


def summarize(db_path: str, top: int = 30) -> str:
    cur = sqlite3.connect(db_path).cursor()
    rows = list(cur.execute(
        "select name, count(*), sum(end-start), avg(end-start), min(end-start), max(end-start) "
        "from kernels group by name order by 3 desc"))
    total = sum(r[2] for r in rows) or 1
    out = [f"{'kernel':72s} {'calls':>6s} {'total_ms':>10s} {'avg_us':>9s} {'min_us':>9s} {'max_us':>9s} {'%':>6s}"]
    for name, n, tot, avg, mn, mx in rows[:top]:
        out.append(f"{name[:72]:72s} {n:6d} {tot / 1e6:10.3f} {avg / 1e3:9.2f} {mn / 1e3:9.2f} "
                   f"{mx / 1e3:9.2f} {100 * tot / total:6.1f}")
    return "\n".join(out)


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("db")
    ap.add_argument("--top", type=int, default=30)
    a = ap.parse_args()
    print(summarize(a.db, a.top))
