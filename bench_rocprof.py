"""Text summaries of rocprofv3 output (its rocpd SQLite databases).

    python bench_rocprof.py trace   RUN_DIR
    python bench_rocprof.py traffic FETCH_DIR WRITE_DIR \
        --copy-bytes 1073741824 --workload cfg2 --kernel gate_up_swiglu=gemm_skinny_kernel<4, 4, 1> \
        [--json profiles/hbm_traffic_measured.json]
    python bench_rocprof.py counters RUN_DIR [--match SUBSTRING ...]

`trace` prints calls / average / min / max / total per kernel of a
`rocprofv3 --kernel-trace --stats` run.  `traffic` reads one `--pmc FETCH_SIZE`
run and one `--pmc WRITE_SIZE` run of the same command, scales each counter by
what it shows for the library's streaming copy of known size (which reads and
writes exactly --copy-bytes), and prints HBM bytes per launch for every kernel;
with --json it records the kernels named by --kernel (label=substring of the
kernel name; several substrings joined by | are summed, for an operation made
of several kernels) for bench.py's `roofline.traffic`.  `counters` prints the
per-kernel average of every counter of a `--pmc` run (kernels whose name holds
one of the --match substrings; all without).
"""
from __future__ import annotations

import argparse
import glob
import json
import os
import re
import sqlite3


def _db(path):
    if os.path.isdir(path):
        found = sorted(glob.glob(os.path.join(path, "**", "*.db"), recursive=True))
        if not found:
            raise SystemExit(f"no .db under {path}")
        path = found[-1]
    return sqlite3.connect(path)


def _short(name):
    name = re.sub(r"\(anonymous namespace\)::", "", name)
    name = re.sub(r"^void ", "", name)
    return re.sub(r"\(.*\)$", "", name)


def trace(run_dir):
    cur = _db(run_dir).cursor()
    rows = cur.execute("select name, count(*), avg(end-start), min(end-start), max(end-start), "
                       "sum(end-start) from kernels group by name order by sum(end-start) desc").fetchall()
    total = sum(r[5] for r in rows) or 1
    print(f"{'kernel':72s} {'calls':>7s} {'avg_us':>9s} {'min_us':>9s} {'max_us':>9s} {'total_ms':>9s} {'%':>6s}")
    for n, c, a, mi, ma, s in rows:
        print(f"{_short(n)[:72]:72s} {c:7d} {a / 1e3:9.2f} {mi / 1e3:9.2f} {ma / 1e3:9.2f} "
              f"{s / 1e6:9.3f} {100 * s / total:6.2f}")
    print(f"total kernel time {total / 1e6:.3f} ms")


def _counter(run_dir, counter):
    cur = _db(run_dir).cursor()
    rows = cur.execute("select kernel_name, count(*), avg(value) from counters_collection "
                       "where counter_name = ? group by kernel_name", (counter,)).fetchall()
    return {_short(k): (n, v) for k, n, v in rows}


def _largest_copy(run_dir, counter):
    """Counter value of the biggest streaming copies of the run (the benchmark's
    reference copy; its shorter calibration copies are left out)."""
    cur = _db(run_dir).cursor()
    vals = [v for (v,) in cur.execute("select value from counters_collection where counter_name = ? "
                                      "and kernel_name like '%stream_copy_kernel%'", (counter,))]
    if not vals:
        raise SystemExit("the streaming copy is not in the run")
    top = [v for v in vals if v >= 0.9 * max(vals)]
    return sum(top) / len(top), len(top)


def traffic(fetch_dir, write_dir, copy_bytes, workload, kernels, json_path):
    fetch = _counter(fetch_dir, "FETCH_SIZE")
    write = _counter(write_dir, "WRITE_SIZE")
    f_copy, n_f = _largest_copy(fetch_dir, "FETCH_SIZE")
    w_copy, n_w = _largest_copy(write_dir, "WRITE_SIZE")
    # counters are in KiB; the copy moved copy_bytes each way
    f_scale = copy_bytes / (f_copy * 1024.0)
    w_scale = copy_bytes / (w_copy * 1024.0)
    print(f"copy of {copy_bytes} bytes ({n_f} / {n_w} launches): FETCH_SIZE {f_copy:.1f} KiB, WRITE_SIZE "
          f"{w_copy:.1f} KiB per launch -> scale factors {f_scale:.4f} (read), {w_scale:.4f} (write)")
    print(f"{'kernel':72s} {'launches':>8s} {'read_MB':>10s} {'write_MB':>10s} {'total_MB':>10s}")
    out = {}
    for k in sorted(fetch, key=lambda k: -fetch[k][1]):
        r = fetch[k][1] * 1024.0 * f_scale
        w = write.get(k, (0, 0.0))[1] * 1024.0 * w_scale
        print(f"{k[:72]:72s} {fetch[k][0]:8d} {r / 1e6:10.3f} {w / 1e6:10.3f} {(r + w) / 1e6:10.3f}")
        out[k] = (r, w)
    if json_path:
        try:
            with open(json_path) as f:
                rec = json.load(f)
        except (OSError, ValueError):
            rec = {}
        for spec in kernels:
            label, _, pat = spec.partition("=")
            pats = [q.replace(" ", "") for q in pat.split("|")]
            hits = [k for k in out if any(q in k.replace(" ", "") for q in pats)]
            if not hits:
                raise SystemExit(f"no kernel matches {pat!r}")
            r = sum(out[k][0] for k in hits)
            w = sum(out[k][1] for k in hits)
            rec[f"{workload}/{label}"] = {"bytes_per_launch": int(round(r + w)), "read": int(round(r)),
                                          "written": int(round(w)), "kernels": hits,
                                          "read_scale": round(f_scale, 4), "write_scale": round(w_scale, 4)}
        with open(json_path, "w") as f:
            json.dump(rec, f, indent=1, sort_keys=True)
            f.write("\n")


def counters(run_dir, match):
    cur = _db(run_dir).cursor()
    rows = cur.execute("select kernel_name, counter_name, count(*), avg(value) from counters_collection "
                       "group by kernel_name, counter_name").fetchall()
    per = {}
    for k, c, n, v in rows:
        name = _short(k)
        if match and not any(m.replace(" ", "") in name.replace(" ", "") for m in match):
            continue
        per.setdefault(name, {})[c] = (n, v)
    for name in sorted(per):
        print(name)
        for c, (n, v) in sorted(per[name].items()):
            print(f"   {c:32s} launches={n:5d} avg={v:16.1f}")


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="cmd", required=True)
    t = sub.add_parser("trace")
    t.add_argument("run_dir")
    p = sub.add_parser("traffic")
    p.add_argument("fetch_dir")
    p.add_argument("write_dir")
    p.add_argument("--copy-bytes", type=int, default=1 << 30)
    p.add_argument("--workload", default="cfg2")
    p.add_argument("--kernel", action="append", default=[])
    p.add_argument("--json", default=None)
    c = sub.add_parser("counters")
    c.add_argument("run_dir")
    c.add_argument("--match", action="append", default=[])
    a = ap.parse_args()
    if a.cmd == "trace":
        trace(a.run_dir)
    elif a.cmd == "counters":
        counters(a.run_dir, a.match)
    else:
        traffic(a.fetch_dir, a.write_dir, a.copy_bytes, a.workload, a.kernel, a.json)


if __name__ == "__main__":
    main()
