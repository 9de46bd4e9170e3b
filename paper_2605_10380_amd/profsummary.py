"""Turns rocprofv3 output into the short text summaries kept under profiles/.

    python -m paper_2605_10380_amd.profsummary trace  <results.db> [rows]
    python -m paper_2605_10380_amd.profsummary pmc    <fetch_counter_collection.csv> <write_counter_collection.csv> [rows]
    python -m paper_2605_10380_amd.profsummary counters <kernel regex> <counter_collection.csv> [more .csv ...]

`trace`: per kernel (name, grid) calls, average / minimum / total duration from a
`rocprofv3 --kernel-trace --stats` run.  `pmc`: HBM bytes per launch from two `rocprofv3 --pmc`
runs (FETCH_SIZE, then WRITE_SIZE) of `bench.py --calibrate-copy`; each counter is scaled by what
it reads for the plain 256 MiB copy kernel that run contains.  `counters`: for every (kernel, grid)
whose name matches the regex, the average per launch of every counter found in the given
`rocprofv3 --pmc ... --output-format csv` files (one file per counter pass).
"""
import collections
import csv
import re
import sqlite3
import sys

COPY_KIB = 256 * 1024          # the calibration kernel copies 256 MiB


def short(name: str) -> str:
    return re.sub(r"\(.*", "", name).replace("void ", "").replace("ax::", "")


def trace(db_path: str, rows: int = 24) -> str:
    cur = sqlite3.connect(db_path).cursor()
    q = ("select name, grid_x / workgroup_x, grid_y, grid_z, workgroup_x, count(*), avg(duration), min(duration), "
         "sum(duration), max(vgpr_count), max(lds_size), max(scratch_size) from kernels "
         "group by name, grid_x, grid_y, grid_z order by sum(duration) desc")
    data = cur.execute(q).fetchall()
    total = sum(r[8] for r in data)
    out = [f"{'kernel':58s} {'grid (blocks)':>16s} {'wg':>5s} {'calls':>6s} {'avg_us':>8s} {'min_us':>8s} {'total_ms':>9s} {'%':>6s} vgpr lds scratch"]
    for r in data[:rows]:
        out.append(f"{short(r[0])[:58]:58s} {str((r[1], r[2], r[3])):>16s} {r[4]:5d} {r[5]:6d} {r[6] / 1e3:8.2f} "
                   f"{r[7] / 1e3:8.2f} {r[8] / 1e6:9.3f} {100 * r[8] / total:6.2f} {r[9]} {r[10]} {r[11]}")
    out.append(f"all kernels: {total / 1e6:.3f} ms")
    return "\n".join(out)


def _load(path):
    agg = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        agg[(short(r["Kernel_Name"]), r["Grid_Size"], r["Workgroup_Size"])].append(float(r["Counter_Value"]))
    return agg


def pmc(fetch_csv: str, write_csv: str, rows: int = 16) -> str:
    f, w = _load(fetch_csv), _load(write_csv)
    avg = lambda a, k: sum(a[k]) / len(a[k]) if k in a else float("nan")
    ck = [k for k in f if "plain_copy" in k[0]][0]
    sf, sw = COPY_KIB / avg(f, ck), COPY_KIB / avg(w, ck)
    out = [f"calibration: plain_copy_kernel of 256 MiB reads FETCH_SIZE = {avg(f, ck):.0f}, WRITE_SIZE = {avg(w, ck):.0f} "
           f"-> {sf:.4f} KiB per FETCH_SIZE unit, {sw:.4f} KiB per WRITE_SIZE unit",
           f"{'kernel':58s} {'grid (threads)':>14s} {'wg':>5s} {'calls':>6s} {'fetch MiB/launch':>17s} {'write MiB/launch':>17s}"]
    order = sorted(f, key=lambda k: -sum(f[k]))
    for k in order[:rows]:
        out.append(f"{k[0][:58]:58s} {k[1]:>14s} {k[2]:>5s} {len(f[k]):6d} {avg(f, k) * sf / 1024:17.3f} {avg(w, k) * sw / 1024:17.3f}")
    return "\n".join(out)


def counters(pattern: str, paths) -> str:
    rx = re.compile(pattern)
    vals = collections.defaultdict(lambda: collections.defaultdict(list))     # kernel key -> counter -> values
    for path in paths:
        for r in csv.DictReader(open(path)):
            name = short(r["Kernel_Name"])
            if rx.search(name):
                vals[(name, r["Grid_Size"], r["Workgroup_Size"])][r["Counter_Name"]].append(float(r["Counter_Value"]))
    out = []
    for key in sorted(vals, key=lambda k: (k[0], int(k[1]))):
        per = vals[key]
        calls = max(len(v) for v in per.values())
        out.append(f"{key[0]}  grid (threads) {key[1]}  wg {key[2]}  launches {calls}")
        for cname in sorted(per):
            v = per[cname]
            out.append(f"    {cname:36s} {sum(v) / len(v):16.1f}")
    return "\n".join(out)


if __name__ == "__main__":
    if len(sys.argv) >= 3 and sys.argv[1] == "trace":
        print(trace(sys.argv[2], int(sys.argv[3]) if len(sys.argv) > 3 else 24))
    elif len(sys.argv) >= 4 and sys.argv[1] == "pmc":
        print(pmc(sys.argv[2], sys.argv[3], int(sys.argv[4]) if len(sys.argv) > 4 else 16))
    elif len(sys.argv) >= 4 and sys.argv[1] == "counters":
        print(counters(sys.argv[2], sys.argv[3:]))
    else:
        sys.exit(__doc__)
