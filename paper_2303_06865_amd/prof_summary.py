"""Turn a rocprofv3 result (rocpd SQLite database, or *_kernel_stats.csv) into the short text
summary kept under profiles/:  python -m paper_2303_06865_amd.prof_summary <results.db> [title]"""
import re
import sqlite3
import sys


def summarize(db_path: str):
    c = sqlite3.connect(db_path)
    cols = [r[1] for r in c.execute("pragma table_info(kernels)")]
    name_col = "name" if "name" in cols else [x for x in cols if "name" in x][0]
    rows = c.execute("select %s, count(*), sum(end-start), min(end-start), max(end-start) from kernels "
                     "group by %s order by 3 desc" % (name_col, name_col)).fetchall()
    total = sum(r[2] for r in rows) or 1
    out = ["%-72s %9s %12s %11s %11s %11s %6s" % ("kernel", "calls", "total_ms", "avg_us", "min_us", "max_us", "%")]
    for name, n, tot, mn, mx in rows:
        short = name.replace("(anonymous namespace)::", "").replace("void ", "")
        short = re.sub(r"\(.*", "", short)
        out.append("%-72s %9d %12.3f %11.2f %11.2f %11.2f %6.2f" % (short[:72], n, tot / 1e6, tot / n / 1e3, mn / 1e3,
                                                                    mx / 1e3, 100.0 * tot / total))
    return "\n".join(out)


if __name__ == "__main__":
    print(summarize(sys.argv[1]))
