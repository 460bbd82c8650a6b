"""Turns a rocprofv3 result database (rocpd sqlite, the default output) into a short text summary:
per-kernel call counts and durations, and - if the run collected counters - per-dispatch counter values.

    python -m paper_1910_11141_amd.rocprof_summary <results.db> [more.db ...]
"""
import sqlite3
import sys


def short(name: str, width: int = 72) -> str:
    name = name.replace("(anonymous namespace)::", "")
    return name if len(name) <= width else name[: width - 3] + "..."


def summarize(path: str) -> str:
    db = sqlite3.connect(path)
    out = [f"== {path}"]
    rows = list(db.execute("select name, total_calls, total_duration, average, percentage from top_kernels"))
    if rows:
        out.append(f"{'kernel':72s} {'calls':>6s} {'total_ms':>11s} {'avg_ms':>11s} {'%':>7s}")
        for name, calls, total, avg, pct in rows:
            out.append(f"{short(name):72s} {calls:6d} {total / 1e3:11.3f} {avg / 1e3:11.3f} {pct:7.3f}")
    pmc = list(db.execute("select name, counter_name, counter_value, duration from pmc_events order by id"))
    if pmc:
        out.append("")
        out.append(f"{'dispatch (in order)':72s} {'counter':>12s} {'value':>16s} {'dur_us':>10s}")
        for name, cname, val, dur in pmc:
            out.append(f"{short(name):72s} {cname:>12s} {val:16.3f} {dur / 1e3:10.1f}")
    return "\n".join(out)


if __name__ == "__main__":
    for p in sys.argv[1:]:
        print(summarize(p))
        print()
