"""Turn the output of three rocprofv3 runs of bench.py into a short text summary and a machine-readable traffic record.

    cd /tmp && export TMPDIR=/tmp            # R = repository root, OUT = any scratch folder
    rocprofv3 --kernel-trace --stats -d OUT/trace -o trace -- python3 R/bench.py --steps 16 --warmup 8 --no-cpu-baseline --no-placement-search
    rocprofv3 --pmc FETCH_SIZE -d OUT/fetch -o fetch -- python3 R/bench.py --steps 8 --warmup 0 --no-cpu-baseline --no-placement-search --calibrate-copy
    rocprofv3 --pmc WRITE_SIZE -d OUT/write -o write -- python3 R/bench.py --steps 8 --warmup 0 --no-cpu-baseline --no-placement-search --calibrate-copy
    python3 -m paper_2502_11058_amd.profile_summary OUT --workload llama2_7b --traffic-json R/profiles/traffic.json > R/profiles/<name>.txt

ROCm 7.2's rocprofv3 writes one SQLite file per run (rocpd); this module reads its `top_kernels`, `kernels` and
`counters_collection` views.  FETCH_SIZE / WRITE_SIZE are per-dispatch readings whose unit differs between
counters and ROCm versions, so each is scaled by what the same counter reads for a plain elementwise copy of known
size in the same run (bench.py --calibrate-copy: the library's ddp_stream_probe with one read and one write stream of
1 GiB each, the same 128-bit streaming accesses as the measured kernels).  The traffic record keeps, per workload and bench.py kernel name, the HBM bytes per launch so
obtained, with the commit and the commands: bench.py reports it as roofline.traffic and says where it came from.
"""
from __future__ import annotations

import argparse
import collections
import json
import os
import sqlite3
import subprocess
import sys

CAL_BYTES = float(1 << 30)          # bytes read, and bytes written, by one calibration copy

# bench.py's kernel names -> how to recognise their dispatches
def _bench_name(kernel: str) -> str | None:
    if "update_dense_kernel" in kernel or "ddp::update_kernel" in kernel or "::update_kernel<" in kernel:
        return "local_update"
    if "mean_kernel" in kernel or "mean_dense_kernel" in kernel:
        return "partial_average"
    if "copy_kernel<false" in kernel or "copy_dense_kernel<false" in kernel:
        return "pack"
    if "copy_kernel<true" in kernel or "copy_dense_kernel<true" in kernel:
        return "unpack"
    if "fused_dense_kernel" in kernel or "fused_kernel" in kernel:
        return "fused_scheduled_layer"
    return None


def short(n: str) -> str:
    n = n.replace("void ", "").replace("ddp::(anonymous namespace)::", "ddp::")
    n = n.replace("at::native::(anonymous namespace)::", "at::").replace("at::native::", "at::")
    return n[:100]


def _db(path: str) -> sqlite3.Connection:
    files = [f for f in os.listdir(path) if f.endswith("_results.db")]
    if not files:
        raise SystemExit(f"no *_results.db under {path}")
    return sqlite3.connect(os.path.join(path, files[0]))


def counter_means(path: str, counter: str):
    """-> ({(kernel, workgroups): [values]}, calibration scale in bytes per counter unit)."""
    db = _db(path)
    per = collections.defaultdict(list)
    cal = []
    for name, cname, val, grid, wg in db.execute("select kernel_name, counter_name, value, grid_size, workgroup_size from counters_collection"):
        if cname != counter:
            continue
        per[(name, grid // max(wg, 1))].append(val)
        if "probe_kernel<1, 1>" in name:
            cal.append(val)
    if not cal:
        raise SystemExit(f"{path}: no calibration copy found (run bench.py with --calibrate-copy)")
    cal.sort()
    return per, CAL_BYTES / cal[len(cal) // 2]


def counters_table(path: str, min_dispatches: int = 1) -> None:
    """Any --pmc run: mean of every counter per (kernel, grid size), for the library's kernels."""
    db = _db(path)
    per = collections.defaultdict(lambda: collections.defaultdict(list))
    names = []
    for name, cname, val, grid, wg in db.execute("select kernel_name, counter_name, value, grid_size, workgroup_size from counters_collection"):
        if "ddp::" not in name:
            continue
        per[(name, grid // max(wg, 1))][cname].append(val)
        if cname not in names:
            names.append(cname)
    print(f"{'kernel':72s} {'workgroups':>10s} {'n':>4s} " + " ".join(f"{c[:26]:>26s}" for c in names))
    for key, cs in sorted(per.items(), key=lambda kv: -kv[0][1]):
        n = len(next(iter(cs.values())))
        if n < min_dispatches:
            continue
        print(f"{short(key[0])[:72]:72s} {key[1]:10d} {n:4d} " + " ".join(f"{sum(cs[c]) / max(len(cs[c]), 1):26.1f}" for c in names))


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("out", help="folder holding trace/, fetch/ and write/ of the three rocprofv3 runs (or, with --counters, of one --pmc run)")
    ap.add_argument("--workload", default="llama2_7b")
    ap.add_argument("--traffic-json", default=None, help="update this file with the measured bytes per launch")
    ap.add_argument("--trace-only", action="store_true", help="`out` holds only trace/: print the kernel-trace tables, no traffic")
    ap.add_argument("--counters", action="store_true", help="`out` is the folder of a single rocprofv3 --pmc run: print the mean of every counter per kernel")
    a = ap.parse_args()
    if a.counters:
        counters_table(a.out)
        return 0

    print("== rocprofv3 --kernel-trace --stats: per-kernel durations (us)")
    print(f"{'kernel':100s} {'calls':>6s} {'total_us':>12s} {'avg_us':>11s} {'pct':>6s}")
    tdb = _db(os.path.join(a.out, "trace"))
    for name, calls, tot, avg, pct in tdb.execute("select name,total_calls,total_duration,average,percentage from top_kernels"):
        if pct < 0.005:
            continue
        print(f"{short(name):100s} {calls:6d} {tot:12.1f} {avg:11.2f} {pct:6.2f}")
    print("\n== the same trace, the library's kernels by grid size (a launch over the whole model vs over a range of layers)")
    print(f"{'kernel':64s} {'workgroups':>11s} {'calls':>6s} {'avg_us':>11s} {'min_us':>11s} {'max_us':>11s}")
    for name, grid, calls, avg, mn, mx in tdb.execute(
            "select name, grid_x / workgroup_x, count(*), avg(duration) / 1e3, min(duration) / 1e3, max(duration) / 1e3 from kernels "
            "where name like '%ddp::%' group by name, grid_x order by sum(duration) desc limit 24"):
        print(f"{short(name)[:64]:64s} {grid:11d} {calls:6d} {avg:11.2f} {mn:11.2f} {mx:11.2f}")

    if a.trace_only:
        return 0
    fetch, fscale = counter_means(os.path.join(a.out, "fetch"), "FETCH_SIZE")
    write, wscale = counter_means(os.path.join(a.out, "write"), "WRITE_SIZE")
    print(f"\n== rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE per dispatch, scaled by the 1 GiB calibration copy "
          f"(FETCH_SIZE unit = {fscale:.1f} B, WRITE_SIZE unit = {wscale:.1f} B)")
    print(f"{'kernel':64s} {'workgroups':>11s} {'n':>4s} {'read GB':>10s} {'written GB':>11s} {'total GB':>10s}")
    rows = []
    for key in fetch:
        if "ddp::" not in key[0] or key not in write:
            continue
        f = sum(fetch[key]) / len(fetch[key]) * fscale
        w = sum(write[key]) / len(write[key]) * wscale
        rows.append((f + w, key, len(fetch[key]), f, w))
    rows.sort(reverse=True)
    best = {}
    for tot, key, n, f, w in rows[:24]:
        print(f"{short(key[0])[:64]:64s} {key[1]:11d} {n:4d} {f / 1e9:10.4f} {w / 1e9:11.4f} {tot / 1e9:10.4f}")
        bn = _bench_name(key[0])
        if bn and bn not in best:          # rows are sorted: the largest launch of each kind (the whole-model / whole-slot one)
            best[bn] = {"bytes_per_launch": tot, "read_bytes": f, "written_bytes": w, "workgroups": key[1], "dispatches": n,
                        "kernel": short(key[0])}
    if a.traffic_json:
        try:
            commit = subprocess.run(["git", "-C", os.path.dirname(os.path.abspath(a.traffic_json)), "rev-parse", "--short", "HEAD"],
                                    capture_output=True, text=True).stdout.strip() or None
        except OSError:
            commit = None
        try:
            with open(a.traffic_json) as fh:
                rec = json.load(fh)
        except (OSError, ValueError):
            rec = {}
        for bn, v in best.items():
            v.update({"commit": commit, "fetch_unit_bytes": fscale, "write_unit_bytes": wscale,
                      "how": "rocprofv3 --pmc FETCH_SIZE and --pmc WRITE_SIZE (two runs of bench.py --calibrate-copy), mean per dispatch of the "
                             "largest launch of this kernel, each counter scaled by its reading for a 1 GiB elementwise copy"})
        rec[a.workload] = best
        with open(a.traffic_json, "w") as fh:
            json.dump(rec, fh, indent=1, sort_keys=True)
            fh.write("\n")
        print(f"\nwrote {os.path.basename(a.traffic_json)}: " + ", ".join(f"{k} {v['bytes_per_launch'] / 1e9:.3f} GB" for k, v in best.items()))
    return 0


if __name__ == "__main__":
    sys.exit(main())
