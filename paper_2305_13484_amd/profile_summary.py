"""Text summary of a rocprofv3 results database (rocpd SQLite): per-kernel time statistics of a --kernel-trace run, or
per-kernel counter averages of a --pmc run.  Usage:
    python -m paper_2305_13484_amd.profile_summary kernels <results.db>
    python -m paper_2305_13484_amd.profile_summary counters <results.db> [kernel-name substring]
    python -m paper_2305_13484_amd.profile_summary iterations <results.db>
`iterations` splits a kernel trace into fused iterations (from one embedding launch to the next; only those that end
with the argmax launch, i.e. no pre-processing passes) and reports how long an iteration's kernels are busy, how long
the iteration spans on the GPU clock, and the gaps between consecutive launches.
"""
import collections
import re
import sqlite3
import sys


def short(name: str) -> str:
    return re.sub(r"\(.*", "", name)[:72]


def kernels(db_path: str) -> str:
    cur = sqlite3.connect(db_path).cursor()
    rows = cur.execute("select name, count(*), sum(end-start), avg(end-start), min(end-start), max(end-start) "
                       "from kernels group by name order by 3 desc").fetchall()
    tot = sum(r[2] for r in rows)
    span = cur.execute("select min(start), max(end) from kernels").fetchone()
    out = ["kernel time total %.2f ms over a span of %.2f ms (GPU busy %.1f%%)"
           % (tot / 1e6, (span[1] - span[0]) / 1e6, 100.0 * tot / (span[1] - span[0])),
           "%-72s %8s %10s %6s %9s %9s %9s" % ("kernel", "calls", "total ms", "%", "avg us", "min us", "max us")]
    for n, c, s, a, mn, mx in rows[:40]:
        out.append("%-72s %8d %10.2f %6.1f %9.2f %9.2f %9.2f" % (short(n), c, s / 1e6, 100.0 * s / tot, a / 1e3,
                                                              mn / 1e3, mx / 1e3))
    return "\n".join(out)


def counters(db_path: str, needle: str = "") -> str:
    cur = sqlite3.connect(db_path).cursor()
    rows = cur.execute("select kernel_name, counter_name, avg(value), count(*) from counters_collection "
                       "group by kernel_name, counter_name").fetchall()
    tab = collections.defaultdict(dict)
    for k, c, v, n in rows:
        tab[short(k)][c] = (v, n)
    out = []
    for k in sorted(tab):
        if needle in k:
            n = list(tab[k].values())[0][1]
            out.append("%-72s dispatches %7d  " % (k, n) + "  ".join("%s avg %.1f" % (c, v) for c, (v, _) in sorted(tab[k].items())))
    return "\n".join(out)


def iterations(db_path: str) -> str:
    import statistics
    rows = sqlite3.connect(db_path).execute(
        "select name, start, end from kernels where name like '%flk%' order by start").fetchall()
    its, cur = [], []
    for n, s, e in rows:
        if "embed_kernel" in n and cur:
            its.append(cur)
            cur = []
        cur.append((n, s, e))
    its.append(cur)
    its = [it for it in its if any("argmax_kernel" in n for n, _, _ in it)]
    busy = [sum(e - s for _, s, e in it) / 1e3 for it in its]
    span = [(it[-1][2] - it[0][1]) / 1e3 for it in its]
    period = [(its[i + 1][0][1] - its[i][0][1]) / 1e3 for i in range(len(its) - 1)]
    gaps = sorted(b[1] - a[2] for it in its for a, b in zip(it, it[1:]))
    return "\n".join([
        "fused iterations %d, launches per iteration (median) %d" % (len(its), statistics.median(len(it) for it in its)),
        "kernels busy per iteration: median %.1f us; iteration span: median %.1f us; start to start: median %.1f us; "
        "sum busy / sum span %.4f" % (statistics.median(busy), statistics.median(span), statistics.median(period),
                                      sum(busy) / sum(span)),
        "gaps between consecutive launches of an iteration: median %.2f us, mean %.2f us, p90 %.2f us"
        % (gaps[len(gaps) // 2] / 1e3, sum(gaps) / len(gaps) / 1e3, gaps[int(len(gaps) * 0.9)] / 1e3)])


if __name__ == "__main__":
    mode, path = sys.argv[1], sys.argv[2]
    if mode == "kernels":
        print(kernels(path))
    elif mode == "iterations":
        print(iterations(path))
    else:
        print(counters(path, sys.argv[3] if len(sys.argv) > 3 else ""))
