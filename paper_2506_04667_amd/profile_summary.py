"""Reduce a rocprofv3 result database (``*_results.db``, the rocpd SQLite output) to the short text tables kept
under ``profiles/``.

    python -m paper_2506_04667_amd.profile_summary trace RESULTS.db [--steps N] [--limit K]
        per-kernel call count, mean / min / max duration and share of the GPU time; with --steps N also one line
        per layer step for the first N steps (a step starts at each gate kernel): the duration of every kernel
        of the step, their sum, the step's span from first start to last end, and the idle time in between.
    python -m paper_2506_04667_amd.profile_summary pmc RESULTS.db [--copy-bytes B]
        per kernel and counter: dispatches, mean value, mean duration.  With --copy-bytes B the dispatch of the
        library's plain copy kernel (moe_probe_stream with a destination, B bytes) calibrates FETCH_SIZE /
        WRITE_SIZE (KiB per dispatch): factor = (B / 1024) / counter value of that copy, and every kernel's mean
        is also printed scaled to bytes.

Reads the ``kernels`` and ``counters_collection`` views that rocprofv3 writes; nothing here runs on the GPU.
"""
import argparse
import re
import sqlite3
import sys


def _short(name, n=96):
    name = re.sub(r"\(anonymous namespace\)::", "", name)
    name = re.sub(r"^void ", "", name)
    name = re.sub(r"\(.*\)$", "", name)
    return name if len(name) <= n else name[: n - 3] + "..."


def _columns(con, table):
    return [r[1] for r in con.execute("pragma table_info(%s)" % table)]


def trace(db, steps, limit, out=sys.stdout):
    con = sqlite3.connect(db)
    cols = _columns(con, "kernels")
    if "duration" not in cols:
        raise SystemExit("no `kernels` view with a duration column in %s (columns: %s)" % (db, cols))
    rows = list(con.execute("select name, start, duration from kernels order by start"))
    by = {}
    for name, start, dur in rows:
        by.setdefault(name, []).append(dur)
    total = float(sum(sum(v) for v in by.values())) or 1.0
    out.write("%-96s %6s %9s %9s %9s %6s\n" % ("kernel", "calls", "avg_us", "min_us", "max_us", "pct"))
    for name, v in sorted(by.items(), key=lambda kv: -sum(kv[1]))[:limit]:
        out.write("%-96s %6d %9.1f %9.1f %9.1f %6.1f\n" % (_short(name), len(v), sum(v) / len(v) / 1e3, min(v) / 1e3,
                                                          max(v) / 1e3, 100.0 * sum(v) / total))
    if steps <= 0:
        return
    # a layer step starts at each gate kernel (the fused gate, or the transpose of the unfused path)
    starts = [i for i, r in enumerate(rows) if "gate_fused_kernel" in r[0] or "transpose_pad_kernel" in r[0]]
    out.write("\n# per layer step (us): kernels in launch order | sum of kernel times | span first start .. last end | idle inside the span | gap to the previous step's end\n")
    prev_end = None
    for s in range(min(steps, len(starts))):
        lo = starts[s]
        hi = starts[s + 1] if s + 1 < len(starts) else len(rows)
        # the step's own kernels: up to and including the first combine kernel after the gate
        step_rows = []
        for r in rows[lo:hi]:
            step_rows.append(r)
            if "combine_kernel" in r[0]:
                break
        durs = [r[2] / 1e3 for r in step_rows]
        span = (step_rows[-1][1] + step_rows[-1][2] - step_rows[0][1]) / 1e3
        gap = "" if prev_end is None else "%8.1f" % ((step_rows[0][1] - prev_end) / 1e3)
        out.write("step %3d: %s | %7.1f | %7.1f | %6.1f | %s\n" % (s + 1, " ".join("%6.1f" % d for d in durs), sum(durs), span,
                                                                span - sum(durs), gap))
        prev_end = step_rows[-1][1] + step_rows[-1][2]
    if starts:
        out.write("# kernel order inside a step: %s\n" % ", ".join(_short(r[0], 40) for r in step_rows))


def pmc(db, copy_bytes, out=sys.stdout):
    con = sqlite3.connect(db)
    cols = _columns(con, "counters_collection")
    name_col = "kernel_name" if "kernel_name" in cols else "name"
    rows = list(con.execute("select %s, counter_name, count(*), avg(value), avg(duration), max(value) from counters_collection "
                            "group by %s, counter_name order by avg(duration) * count(*) desc" % (name_col, name_col)))
    factor = {}
    if copy_bytes:
        for name, counter, n, mean, dur, vmax in rows:
            if "stream_probe_kernel<true>" in name and counter in ("FETCH_SIZE", "WRITE_SIZE"):
                factor[counter] = (copy_bytes / 1024.0) / vmax
                out.write("# calibration: %s of the %d-byte copy kernel reads %.1f (KiB units) -> factor %.4f\n" % (counter, copy_bytes, vmax, factor[counter]))
    out.write("%-80s %-28s %5s %14s %10s %16s\n" % ("kernel", "counter", "n", "mean", "avg_us", "scaled_bytes"))
    for name, counter, n, mean, dur, vmax in rows:
        scaled = "%16.0f" % (mean * factor[counter] * 1024.0) if counter in factor else ""
        out.write("%-80s %-28s %5d %14.6g %10.1f %s\n" % (_short(name, 80), counter, n, mean, dur / 1e3, scaled))


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    t = sub.add_parser("trace")
    t.add_argument("db")
    t.add_argument("--steps", type=int, default=0)
    t.add_argument("--limit", type=int, default=20)
    p = sub.add_parser("pmc")
    p.add_argument("db")
    p.add_argument("--copy-bytes", type=int, default=0)
    a = ap.parse_args(argv)
    if a.cmd == "trace":
        trace(a.db, a.steps, a.limit)
    else:
        pmc(a.db, a.copy_bytes)


if __name__ == "__main__":
    main()
