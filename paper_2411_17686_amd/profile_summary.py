"""Turns a rocprofv3 result database into the short text tables kept under profiles/.

    python -m paper_2411_17686_amd.profile_summary kernels  <bench_results.db>
    python -m paper_2411_17686_amd.profile_summary counters <bench_results.db> [name-filter]

`kernels`: per kernel and launch shape (total threads of the grid) of a `rocprofv3 --kernel-trace
--stats` run the number of dispatches and the average / minimum / maximum duration in
microseconds.  `counters`: per kernel, launch shape and counter of a `rocprofv3 --pmc ...
--kernel-trace` run the average value per dispatch.  Launch shapes are kept apart because one
run issues the same kernel at several problem sizes; with a single counter the six largest single
dispatches follow (the calibration copy of known size among them).  CPU only (sqlite3): it reads what the
profiler wrote and computes nothing else.
"""
import collections
import sqlite3
import sys


def short(name):
    return name.replace("void ", "").replace("ficoco::", "").split("(")[0][:64]


def kernels(db):
    c = sqlite3.connect(db)
    rows = c.execute("select name, count(*), avg(end-start), min(end-start), max(end-start), sum(end-start), "
                     "grid_x*grid_y*grid_z as threads from kernels group by name, threads "
                     "order by sum(end-start) desc").fetchall()
    tot = sum(r[5] for r in rows) or 1
    print("%-56s %9s %6s %9s %9s %9s %6s" % ("kernel", "threads", "calls", "avg_us", "min_us", "max_us", "pct"))
    for r in rows[:30]:
        print("%-56s %9d %6d %9.2f %9.2f %9.2f %5.1f%%" % (short(r[0])[:56], r[6], r[1], r[2] / 1e3, r[3] / 1e3, r[4] / 1e3,
                                                        100 * r[5] / tot))


def counters(db, flt=""):
    c = sqlite3.connect(db)
    rows = c.execute("select kernel_name, counter_name, avg(value), count(*), avg(end-start), grid_size "
                     "from counters_collection group by kernel_name, grid_size, counter_name").fetchall()
    vals, meta = collections.defaultdict(dict), {}
    for k, cn, v, n, du, g in rows:
        if flt and flt not in k:
            continue
        vals[(short(k)[:56], g)][cn] = v
        meta[(short(k)[:56], g)] = (du / 1e3, n)
    names = sorted({cn for k in vals for cn in vals[k]})
    print("%-56s %10s %6s %9s" % ("kernel (average per dispatch)", "threads", "calls", "us") + "".join(" %18s" % n[:18] for n in names))
    for k in sorted(vals, key=lambda k: -meta[k][0] * meta[k][1])[:30]:
        print("%-56s %10d %6d %9.1f" % (k[0], k[1], meta[k][1], meta[k][0])
              + "".join(" %18.1f" % vals[k].get(n, float("nan")) for n in names))
    if len(names) == 1 and not flt:
        # single dispatches with the largest readings: a calibration kernel of known traffic (a big
        # plain copy) shares its name and launch shape with small copies, so it shows here
        print("\nlargest single dispatches by %s" % names[0])
        for k, g, v, du in c.execute("select kernel_name, grid_size, value, end-start from counters_collection "
                                     "order by value desc limit 6"):
            print("%-56s %10d %6s %9.1f %18.1f" % (short(k)[:56], g, "", du / 1e3, v))


if __name__ == "__main__":
    if len(sys.argv) < 3 or sys.argv[1] not in ("kernels", "counters"):
        sys.exit(__doc__)
    if sys.argv[1] == "kernels":
        kernels(sys.argv[2])
    else:
        counters(sys.argv[2], sys.argv[3] if len(sys.argv) > 3 else "")
