"""Text summary of a rocprofv3 result database (per-kernel calls / total / average), the
form kept under profiles/.

    python -m paper_2503_05840_amd.prof_summary OUTDIR/NAME_results.db ["command line"]
"""
import sqlite3
import sys


def summarize(db_path: str, command: str = "") -> str:
    con = sqlite3.connect(db_path)
    rows = con.execute("select name, total_calls, total_duration, average, percentage from top_kernels").fetchall()
    lines = []
    if command:
        lines.append(f"command: {command}")
    lines.append("source : rocprofv3 --kernel-trace --stats (durations in microseconds)")
    lines.append(f"{'calls':>7} {'total_us':>12} {'avg_us':>10} {'pct':>6}  kernel")
    for name, calls, total, avg, pct in rows:
        short = name.replace("slim::(anonymous namespace)::", "")
        short = short.split("(")[0] if len(short) > 110 else short
        lines.append(f"{calls:>7} {total:>12.1f} {avg:>10.3f} {pct:>6.2f}  {short}")
    try:
        pmc = con.execute("select * from counters_collection limit 1").fetchall()
    except sqlite3.Error:
        pmc = []
    if pmc:
        cur = con.execute("select kernel_name, counter_name, avg(value), count(*) from counters_collection "
                          "group by kernel_name, counter_name")
        lines.append("")
        lines.append("counters (average per dispatch):")
        for k, c, v, n in cur:
            k = k.replace("slim::(anonymous namespace)::", "").split("(")[0]
            lines.append(f"  {c:<22} {v:>16.1f}  n={n:<5} {k}")
    return "\n".join(lines) + "\n"


if __name__ == "__main__":
    sys.stdout.write(summarize(sys.argv[1], sys.argv[2] if len(sys.argv) > 2 else ""))
