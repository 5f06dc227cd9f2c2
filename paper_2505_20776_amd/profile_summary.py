"""Text summaries of rocprofv3 runs of this library (the .db files rocprofv3 writes).

    python -m paper_2505_20776_amd.profile_summary kernels  RUN.db
    python -m paper_2505_20776_amd.profile_summary counters RUN.db
    python -m paper_2505_20776_amd.profile_summary traffic  FETCH.db WRITE.db --out profiles/NAME.txt

`kernels` prints calls / total / average / min / max duration per kernel of this library; `counters` the
per-dispatch average of every collected counter per kernel; `traffic` turns one FETCH_SIZE pass and one
WRITE_SIZE pass of the default benchmark into HBM bytes per launch of the dominant kernel.  Both counters
report KiB per dispatch; each is scaled by what the same counter reads for gather_copy_kernel, a plain copy
that reads and writes exactly 2 x Hkv x 1024 x 128 bf16 values = 4 MiB per dispatch in the default
benchmark.  The result file is what bench.py quotes as roofline.traffic.
"""
import argparse
import datetime
import sqlite3
import subprocess
import sys

OURS = "specext"


def _rows(db, query):
    con = sqlite3.connect(db)
    try:
        return con.execute(query).fetchall()
    finally:
        con.close()


def kernels(db, out=sys.stdout):
    rows = _rows(db, "select name, count(*), sum(duration), avg(duration), min(duration), max(duration) from kernels "
                     "group by name order by sum(duration) desc")
    rows = [r for r in rows if OURS in r[0]]
    total = sum(r[2] for r in rows) or 1
    print(f"{'kernel':72s} {'calls':>7s} {'total_us':>11s} {'avg_us':>9s} {'min_us':>9s} {'max_us':>9s} {'pct':>6s}", file=out)
    for name, calls, tot, avg, mn, mx in rows:
        print(f"{name[:72]:72s} {calls:7d} {tot / 1e3:11.1f} {avg / 1e3:9.2f} {mn / 1e3:9.2f} {mx / 1e3:9.2f} {100 * tot / total:6.2f}", file=out)


def counters(db, out=sys.stdout):
    rows = _rows(db, "select kernel_name, counter_name, count(*), avg(value) from counters_collection "
                     "group by kernel_name, counter_name order by kernel_name, counter_name")
    for name, counter, n, avg in rows:
        if OURS in name:
            print(f"{name[:72]:72s} {counter:28s} dispatches={n:5d} avg={avg:16.1f}", file=out)


def _avg(db, counter, kernel_like):
    rows = _rows(db, f"select kernel_name, count(*), avg(value) from counters_collection where counter_name = '{counter}' "
                     "group by kernel_name")
    hits = [(n, c, a) for n, c, a in rows if kernel_like in n]
    if not hits:
        raise SystemExit(f"no dispatch of a kernel matching {kernel_like!r} with counter {counter} in {db}")
    n, c, a = max(hits, key=lambda r: r[1])
    return n, c, a


def traffic(fetch_db, write_db, kernel, copy_kernel, copy_kib, out_path):
    kname, kcalls, fetch_kib = _avg(fetch_db, "FETCH_SIZE", kernel)
    _, _, write_kib = _avg(write_db, "WRITE_SIZE", kernel)
    _, _, copy_fetch = _avg(fetch_db, "FETCH_SIZE", copy_kernel)
    _, _, copy_write = _avg(write_db, "WRITE_SIZE", copy_kernel)
    f_fetch, f_write = copy_kib / copy_fetch, copy_kib / copy_write
    fetch_bytes = fetch_kib * f_fetch * 1024
    write_bytes = write_kib * f_write * 1024
    try:
        commit = subprocess.run(["git", "rev-parse", "--short=12", "HEAD"], capture_output=True, text=True).stdout.strip() or "?"
        dirty = subprocess.run(["git", "status", "--porcelain", "--", "paper_2505_20776_amd/csrc"], capture_output=True,
                               text=True).stdout.strip()
        if dirty:
            commit += "+uncommitted-kernel-changes"
    except OSError:
        commit = "?"
    lines = [
        "# HBM traffic of the dominant kernel of the default benchmark (config 4), per launch.",
        "# Written by `python -m paper_2505_20776_amd.profile_summary traffic`; read by bench.py (roofline.traffic).",
        f"kernel={kname[:100]}",
        f"dispatches={kcalls}",
        f"commit={commit}",
        f"date={datetime.date.today().isoformat()}",
        f"FETCH_SIZE_KiB_per_dispatch={fetch_kib:.1f}",
        f"WRITE_SIZE_KiB_per_dispatch={write_kib:.1f}",
        f"copy_kernel={copy_kernel}",
        f"copy_KiB_read_and_written_per_dispatch={copy_kib:.1f}",
        f"copy_FETCH_SIZE_KiB={copy_fetch:.1f}",
        f"copy_WRITE_SIZE_KiB={copy_write:.1f}",
        f"fetch_scale={f_fetch:.4f}",
        f"write_scale={f_write:.4f}",
        f"fetch_bytes_per_launch={fetch_bytes:.0f}",
        f"write_bytes_per_launch={write_bytes:.0f}",
        f"traffic_bytes_per_launch={fetch_bytes + write_bytes:.0f}",
    ]
    text = "\n".join(lines) + "\n"
    if out_path:
        with open(out_path, "w") as f:
            f.write(text)
    sys.stdout.write(text)


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    for name in ("kernels", "counters"):
        sp = sub.add_parser(name)
        sp.add_argument("db")
    sp = sub.add_parser("traffic")
    sp.add_argument("fetch_db")
    sp.add_argument("write_db")
    sp.add_argument("--kernel", default="prefix_rows_kernel<8, false, 1, ")
    sp.add_argument("--copy-kernel", default="gather_copy_kernel")
    sp.add_argument("--copy-kib", type=float, default=4096.0)
    sp.add_argument("--out", default="")
    a = ap.parse_args()
    if a.cmd == "kernels":
        kernels(a.db)
    elif a.cmd == "counters":
        counters(a.db)
    else:
        traffic(a.fetch_db, a.write_db, a.kernel, a.copy_kernel, a.copy_kib, a.out)


if __name__ == "__main__":
    main()
