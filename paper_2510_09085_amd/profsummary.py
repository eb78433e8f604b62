"""Turn rocprofv3 output databases (rocpd / SQLite) into the short text summaries kept
under profiles/.

  python -m paper_2510_09085_amd.profsummary kernels  RESULTS.db [N]
      per (kernel, grid) launch count and total / average / min / max duration
  python -m paper_2510_09085_amd.profsummary counters RESULTS.db [SUBSTR]
      mean value per launch of every collected counter, per kernel whose name contains SUBSTR
  python -m paper_2510_09085_amd.profsummary traffic  FETCH.db WRITE.db PROBE.json KERNEL_SUBSTR OUT.json
      HBM bytes per launch of one kernel: FETCH_SIZE and WRITE_SIZE (KiB per dispatch), each
      scaled by what the same counter reads for the plain device copy of known size that
      `bench.py --counter-probe prune` runs beside it; writes the record bench.py looks up
"""
from __future__ import annotations

import json
import re
import sqlite3
import sys
from collections import defaultdict


def _short(name: str) -> str:
    name = name.replace("fltop::(anonymous namespace)::", "fltop::")
    name = re.sub(r"^void ", "", name)
    return re.sub(r"\((?!anonymous).*$", "", name)[:64]


def kernels(db: str, top: int = 20) -> str:
    con = sqlite3.connect(db)
    rows = con.execute(
        "select name, grid_x / max(workgroup_x, 1) * max(grid_y / max(workgroup_y, 1), 1), "
        "count(*), sum(end - start), avg(end - start), min(end - start), max(end - start) "
        "from kernels group by 1, 2 order by 4 desc").fetchall()
    total = sum(r[3] for r in rows) or 1
    out = [f"{'kernel':64s} {'workgroups':>10s} {'calls':>6s} {'total_us':>11s} {'avg_us':>9s} "
           f"{'min_us':>9s} {'max_us':>9s} {'%':>6s}"]
    for name, wgs, calls, tot, avg, mn, mx in rows[:top]:
        out.append(f"{_short(name):64s} {int(wgs):10d} {calls:6d} {tot / 1e3:11.1f} "
                   f"{avg / 1e3:9.2f} {mn / 1e3:9.2f} {mx / 1e3:9.2f} {100 * tot / total:6.2f}")
    return "\n".join(out)


def _counter_rows(db: str, substr: str):
    con = sqlite3.connect(db)
    rows = con.execute("select kernel_name, counter_name, value, duration from counters_collection "
                       "order by dispatch_id").fetchall()
    return [r for r in rows if substr in r[0]]


def counters(db: str, substr: str = "") -> str:
    acc = defaultdict(list)
    dur = defaultdict(list)
    for name, counter, value, duration in _counter_rows(db, substr):
        acc[(_short(name), counter)].append(value)
        dur[_short(name)].append(duration)
    out = [f"{'kernel':56s} {'counter':24s} {'launches':>8s} {'mean per launch':>18s}"]
    for (name, counter), vals in sorted(acc.items()):
        out.append(f"{name:56s} {counter:24s} {len(vals):8d} {sum(vals) / len(vals):18.1f}")
    for name, d in sorted(dur.items()):
        out.append(f"{name:56s} {'duration_us':24s} {len(d):8d} {sum(d) / len(d) / 1e3:18.2f}")
    return "\n".join(out)


def traffic(fetch_db: str, write_db: str, probe_json: str, substr: str, out_json: str) -> str:
    probe = json.load(open(probe_json))
    copy_bytes = probe["copy_bytes_each_way"]

    def mean_kib(db, sub, counter, only_full_copies=False):
        vals = [v for _, c, v, _ in _counter_rows(db, sub) if c == counter]
        if only_full_copies:  # the calibration copies are the largest ones in the run
            vals = [v for v in vals if v >= 0.9 * max(vals)]
        return sum(vals) / len(vals)

    f_copy = mean_kib(fetch_db, "copyBuffer", "FETCH_SIZE", True) * 1024
    w_copy = mean_kib(write_db, "copyBuffer", "WRITE_SIZE", True) * 1024
    f_scale, w_scale = copy_bytes / f_copy, copy_bytes / w_copy
    f_k = mean_kib(fetch_db, substr, "FETCH_SIZE") * 1024 * f_scale
    w_k = mean_kib(write_db, substr, "WRITE_SIZE") * 1024 * w_scale
    rec = {
        "kernel": substr, "workload": probe["workload"], "rel_threshold": probe["rel_threshold"],
        "fetch_scale_from_copy": round(f_scale, 4), "write_scale_from_copy": round(w_scale, 4),
        "hbm_read_bytes_per_launch": round(f_k), "hbm_write_bytes_per_launch": round(w_k),
        "hbm_bytes_per_launch": round(f_k + w_k),
        "sources": probe["sources"], "source_sha256": probe["source_sha256"],
    }
    for key in ("emission_bytes_per_launch", "written_bytes_approx", "frames"):
        if key in probe:
            rec[key] = probe[key]
    with open(out_json, "w") as fh:
        json.dump(rec, fh, indent=1)
        fh.write("\n")
    return json.dumps(rec, indent=1)


def main(argv):
    if len(argv) < 3:
        print(__doc__)
        return 2
    cmd = argv[1]
    if cmd == "kernels":
        print(kernels(argv[2], int(argv[3]) if len(argv) > 3 else 20))
    elif cmd == "counters":
        print(counters(argv[2], argv[3] if len(argv) > 3 else ""))
    elif cmd == "traffic":
        print(traffic(*argv[2:7]))
    else:
        print(__doc__)
        return 2
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
