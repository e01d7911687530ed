"""Turn rocprofv3 output into the short text summaries kept under profiles/.

Usage (after a rocprofv3 run that wrote into <dir>):
  python -m paper_2604_09562_amd.profiling kernels <dir>/<name>_results.db
      per-kernel table of a `--kernel-trace --stats` run (rocpd database)
  python -m paper_2604_09562_amd.profiling traffic <fetch_dir> <write_dir> --copy-bytes N
      HBM bytes per launch of every kernel from two `--pmc` runs (FETCH_SIZE, then WRITE_SIZE,
      csv output), each counter scaled by what it reads for the plain device copy of N bytes
      that `bench.py --calibrate-copy` launches in the same run
"""
from __future__ import annotations

import argparse
import collections
import csv
import glob
import os
import sqlite3
import sys

COPY_KERNEL_HINTS = ("copyBuffer", "CopyFunctor", "direct_copy")


def kernel_table(db_path: str) -> str:
    c = sqlite3.connect(db_path)
    rows = c.execute("select name, count(*), avg(end-start), min(end-start), max(end-start), sum(end-start) "
                     "from kernels group by name order by 6 desc").fetchall()
    tot = sum(r[5] for r in rows) or 1
    out = [f"{'kernel':96s} {'calls':>6s} {'avg_us':>9s} {'min_us':>9s} {'max_us':>9s} {'pct':>6s}"]
    for n, k, a, mi, ma, s in rows:
        out.append(f"{n[:96]:96s} {k:6d} {a / 1e3:9.2f} {mi / 1e3:9.2f} {ma / 1e3:9.2f} {100 * s / tot:6.2f}")
    return "\n".join(out)


def _counter_means(run_dir: str, counter: str):
    files = glob.glob(os.path.join(run_dir, "**", "*counter_collection.csv"), recursive=True)
    if not files:
        raise FileNotFoundError(f"no counter_collection.csv under {run_dir}")
    acc = collections.defaultdict(list)
    with open(files[0]) as f:
        for r in csv.DictReader(f):
            if r["Counter_Name"] == counter:
                acc[r["Kernel_Name"]].append((float(r["Counter_Value"]), int(r["Grid_Size"])))
    return acc


def traffic_table(fetch_dir: str, write_dir: str, copy_bytes: int) -> str:
    fetch = _counter_means(fetch_dir, "FETCH_SIZE")
    write = _counter_means(write_dir, "WRITE_SIZE")

    def calib(acc, label):
        # the calibration copy is the largest launch of a plain copy kernel in the run
        cands = [(max(v for v, _ in rows), k) for k, rows in acc.items() if any(h in k for h in COPY_KERNEL_HINTS)]
        if not cands:
            raise RuntimeError(f"no copy kernel found in the {label} run")
        top, name = max(cands)
        vals = [v for v, _ in acc[name] if v > 0.99 * top]
        return name, sum(vals) / len(vals)

    fname, fval = calib(fetch, "FETCH_SIZE")
    wname, wval = calib(write, "WRITE_SIZE")
    f_scale, w_scale = copy_bytes / fval, copy_bytes / wval   # bytes per counter unit
    out = [f"calibration copy: {copy_bytes} bytes read and written per launch",
           f"  FETCH_SIZE of {fname[:60]}: {fval:.6g} -> {f_scale:.4g} bytes per unit",
           f"  WRITE_SIZE of {wname[:60]}: {wval:.6g} -> {w_scale:.4g} bytes per unit", "",
           f"{'kernel':70s} {'launches':>8s} {'read_MB':>10s} {'write_MB':>10s}"]
    for k in sorted(fetch, key=lambda k: -sum(v for v, _ in fetch[k])):
        fv = [v for v, _ in fetch[k]]
        wv = [v for v, _ in write.get(k, [(0.0, 0)])]
        out.append(f"{k[:70]:70s} {len(fv):8d} {sum(fv) / len(fv) * f_scale / 1e6:10.2f} "
                   f"{sum(wv) / len(wv) * w_scale / 1e6:10.2f}")
    return "\n".join(out)


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    k = sub.add_parser("kernels")
    k.add_argument("db")
    t = sub.add_parser("traffic")
    t.add_argument("fetch_dir")
    t.add_argument("write_dir")
    t.add_argument("--copy-bytes", type=int, required=True)
    a = ap.parse_args(argv)
    if a.cmd == "kernels":
        print(kernel_table(a.db))
    else:
        print(traffic_table(a.fetch_dir, a.write_dir, a.copy_bytes))
    return 0


if __name__ == "__main__":
    sys.exit(main())
