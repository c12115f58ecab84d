"""Turn rocprofv3 results into the short text summaries kept under profiles/:
  python3 prof_summary.py <results.db>                 kernel-trace database (rocpd SQLite)
  python3 prof_summary.py <x_counter_collection.csv>   --pmc run with --output-format csv
For counters the summary is the mean value per dispatch of every (kernel, counter) pair."""
import csv
import re
import sqlite3
import sys


def _short(name: str) -> str:
    short = name.replace("(anonymous namespace)::", "").replace("void ", "")
    return re.sub(r"\(.*", "", short)


def summarize_pmc(csv_path: str, only: str = "fg::"):
    """Mean per dispatch of each counter for kernels whose name contains `only` (all if empty)."""
    acc = {}
    with open(csv_path, newline="") as f:
        for row in csv.DictReader(f):
            name = row["Kernel_Name"]
            if only and only not in name and "elementwise" not in name and "copy" not in name.lower():
                continue
            key = (_short(name)[:72], row["Counter_Name"])
            d = acc.setdefault(key, {})
            d[row["Dispatch_Id"]] = d.get(row["Dispatch_Id"], 0.0) + float(row["Counter_Value"])
    out = ["%-72s %-28s %9s %16s" % ("kernel", "counter", "dispatches", "mean/dispatch")]
    for (k, cn), d in sorted(acc.items()):
        out.append("%-72s %-28s %9d %16.1f" % (k, cn, len(d), sum(d.values()) / len(d)))
    return "\n".join(out)


def summarize(db_path: str):
    c = sqlite3.connect(db_path)
    cols = [r[1] for r in c.execute("pragma table_info(kernels)")]
    name_col = "name" if "name" in cols else [x for x in cols if "name" in x][0]
    rows = c.execute("select %s, count(*), sum(end-start), min(end-start), max(end-start) from kernels "
                     "group by %s order by 3 desc" % (name_col, name_col)).fetchall()
    total = sum(r[2] for r in rows) or 1
    out = ["%-72s %9s %12s %11s %11s %11s %6s" % ("kernel", "calls", "total_ms", "avg_us", "min_us", "max_us", "%")]
    for name, n, tot, mn, mx in rows:
        short = _short(name)
        out.append("%-72s %9d %12.3f %11.2f %11.2f %11.2f %6.2f" % (short[:72], n, tot / 1e6, tot / n / 1e3, mn / 1e3,
                                                                    mx / 1e3, 100.0 * tot / total))
    return "\n".join(out)


if __name__ == "__main__":
    print(summarize_pmc(sys.argv[1]) if sys.argv[1].endswith(".csv") else summarize(sys.argv[1]))
