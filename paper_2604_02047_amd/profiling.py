"""Text summaries of a rocprofv3 run (its rocpd SQLite output): per-kernel durations, and HBM
traffic per launch from the FETCH_SIZE / WRITE_SIZE counters, scaled by what the same counter read
for the library's copy probe (a kernel that moves a known number of bytes) in the same run.

    python -m paper_2604_02047_amd.profiling kernels <run_results.db>
    python -m paper_2604_02047_amd.profiling traffic <fetch_run.db> <write_run.db> <copy_probe_bytes>
    python -m paper_2604_02047_amd.profiling counters <pmc_run.db> [<pmc_run.db> ...]

Reads only; prints to stdout.  Nothing here runs on the GPU.
"""
import collections
import re
import sqlite3
import sys


def short_name(name):
    name = re.sub(r"\s+", " ", name)
    m = re.search(r"(k_[a-z0-9_]+?)(?=[A-Z<(]|$)", name)   # also inside a mangled name; drops its suffix
    if m:
        t = re.search(re.escape(m.group(1)) + r"(<[^(]*>)", name)
        return m.group(1) + (t.group(1) if t else "")
    return re.sub(r"\(.*", "", name)[-60:]


def kernel_stats(db):
    """[(name, calls, avg_us, min_us, max_us, total_ms)] sorted by total time."""
    c = sqlite3.connect(db)
    rows = c.execute("select name, count(*), avg(end-start), min(end-start), max(end-start), sum(end-start) "
                     "from kernels group by name order by sum(end-start) desc").fetchall()
    return [(short_name(n), k, a / 1e3, lo / 1e3, hi / 1e3, t / 1e6) for n, k, a, lo, hi, t in rows]


def print_kernels(db):
    """Library kernels one per row; everything else (input generation and staging done with torch
    before the timed region) summed in one row."""
    rows = kernel_stats(db)
    tot = sum(r[5] for r in rows)
    print(f"{'kernel':64s} {'calls':>7s} {'avg_us':>9s} {'min_us':>9s} {'max_us':>9s} {'total_ms':>9s} {'%':>6s}")
    other_calls, other_ms = 0, 0.0
    for n, k, a, lo, hi, t in rows:
        if not n.startswith("k_"):
            other_calls, other_ms = other_calls + k, other_ms + t
            continue
        print(f"{n[:64]:64s} {k:7d} {a:9.2f} {lo:9.2f} {hi:9.2f} {t:9.2f} {100 * t / tot:6.2f}")
    print(f"{'(kernels of other libraries: setup and staging)':64s} {other_calls:7d} {'':9s} {'':9s} {'':9s} "
          f"{other_ms:9.2f} {100 * other_ms / tot:6.2f}")


def counter_per_kernel(db, counter):
    """{(kernel, workgroups_x, grid_y): (launches, mean counter value per launch, mean duration us)}."""
    c = sqlite3.connect(db)
    q = ("select k.name, k.grid_x, k.grid_y, k.workgroup_x, p.dispatch_id, sum(p.counter_value), k.end - k.start "
         "from pmc_events p join kernels k on p.dispatch_id = k.dispatch_id where p.counter_name = ? "
         "group by p.dispatch_id")
    acc = collections.defaultdict(list)
    for name, gx, gy, wx, _, val, dur in c.execute(q, (counter,)):
        acc[(short_name(name), gx // wx if wx else gx, gy)].append((val, dur))
    return {k: (len(v), sum(x for x, _ in v) / len(v), sum(d for _, d in v) / len(v) / 1e3) for k, v in acc.items()}


def last_step_total(db, counter):
    """(sum of the counter, dispatches) over the last verification step of the run: from the last
    k_build_mask dispatch up to (not including) the copy probe that follows the steps."""
    c = sqlite3.connect(db)
    q = ("select p.dispatch_id, k.name, sum(p.counter_value) from pmc_events p join kernels k "
         "on p.dispatch_id = k.dispatch_id where p.counter_name = ? group by p.dispatch_id order by k.start")
    rows = [(d, short_name(n), v) for d, n, v in c.execute(q, (counter,))]
    first = max((i for i, r in enumerate(rows) if r[1].startswith("k_build_mask")), default=None)
    if first is None:
        return None
    step = []
    for r in rows[first:]:
        if r[1].startswith("k_copy_probe"):
            break
        if r[1].startswith("k_"):
            step.append(r)
    return sum(r[2] for r in step), len(step)


def source_hash():
    """First 12 hex digits of the SHA-256 over the library's sources (csrc/ and include/goose.h, sorted by
    name): says which build a counter summary belongs to."""
    import hashlib
    import os
    pkg = os.path.dirname(os.path.abspath(__file__))
    files = sorted(os.path.join(pkg, "csrc", f) for f in os.listdir(os.path.join(pkg, "csrc")))
    files.append(os.path.join(os.path.dirname(pkg), "include", "goose.h"))
    h = hashlib.sha256()
    for f in files:
        with open(f, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:12]


def print_traffic(fetch_db, write_db, probe_bytes):
    fetch = counter_per_kernel(fetch_db, "FETCH_SIZE")
    write = counter_per_kernel(write_db, "WRITE_SIZE")
    pf = [v for k, v in fetch.items() if k[0].startswith("k_copy_probe")]
    pw = [v for k, v in write.items() if k[0].startswith("k_copy_probe")]
    if not pf or not pw:
        raise SystemExit("no k_copy_probe dispatch in the run: cannot calibrate")
    # the counters are documented in KiB; the probe says what one byte of HBM traffic reads as
    f_unit = probe_bytes / pf[0][1]
    w_unit = probe_bytes / pw[0][1]
    print(f"copy probe of {probe_bytes} bytes: FETCH_SIZE reads {pf[0][1]:.1f} -> {f_unit:.2f} bytes per count "
          f"(1024 if it counted KiB exactly); WRITE_SIZE reads {pw[0][1]:.1f} -> {w_unit:.2f} bytes per count")
    import datetime
    print(f"recorded {datetime.date.today().isoformat()} for the library sources with hash {source_hash()}")
    lf, lw = last_step_total(fetch_db, "FETCH_SIZE"), last_step_total(write_db, "WRITE_SIZE")
    if lf and lw:
        print(f"last step of the run: {lf[1]} launches, fetch {lf[0] * f_unit / 1e6:.2f} MB, write {lw[0] * w_unit / 1e6:.2f} MB")
    print(f"{'kernel':52s} {'wgs_x':>6s} {'gy':>3s} {'n':>5s} {'avg_us':>8s} {'fetch_MB':>10s} {'write_MB':>10s}")
    for key in sorted(fetch, key=lambda k: -fetch[k][0] * fetch[k][2]):
        if not key[0].startswith("k_"):
            continue
        n, fv, dur = fetch[key]
        wv = write.get(key, (0, float('nan'), 0))[1]
        print(f"{key[0][:52]:52s} {key[1]:6d} {key[2]:3d} {n:5d} {dur:8.1f} {fv * f_unit / 1e6:10.2f} "
              f"{wv * w_unit / 1e6:10.2f}")


def print_counters(dbs):
    """Per kernel and launch shape: the mean over its launches of every counter the runs collected (a raw
    counter summed over its hardware instances, a derived metric as rocprofv3 evaluated it)."""
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    durs = collections.defaultdict(list)
    names = []
    for db in dbs:
        c = sqlite3.connect(db)
        q = ("select k.name, k.grid_x, k.grid_y, k.workgroup_x, p.counter_name, p.dispatch_id, sum(p.counter_value), "
             "k.end - k.start from pmc_events p join kernels k on p.dispatch_id = k.dispatch_id "
             "group by p.dispatch_id, p.counter_name")
        for name, gx, gy, wx, cn, _, val, dur in c.execute(q):
            key = (short_name(name), gx // wx if wx else gx, gy)
            acc[key][cn].append(val)
            durs[key].append(dur)
            if cn not in names:
                names.append(cn)
    print(f"{'kernel':44s} {'wgs_x':>6s} {'gy':>3s} {'n':>5s} {'avg_us':>8s} " + " ".join(f"{n[-22:]:>22s}" for n in names))
    for key in sorted(acc, key=lambda k: -sum(durs[k])):
        if not key[0].startswith("k_"):
            continue
        v = acc[key]
        n = max(len(x) for x in v.values())
        print(f"{key[0][:44]:44s} {key[1]:6d} {key[2]:3d} {n:5d} {sum(durs[key]) / len(durs[key]) / 1e3:8.1f} " +
              " ".join(f"{sum(v[cn]) / len(v[cn]):22.5g}" if cn in v else f"{'-':>22s}" for cn in names))


def main(argv):
    if len(argv) >= 3 and argv[1] == "kernels":
        print_kernels(argv[2])
    elif len(argv) >= 5 and argv[1] == "traffic":
        print_traffic(argv[2], argv[3], int(argv[4]))
    elif len(argv) >= 3 and argv[1] == "counters":
        print_counters(argv[2:])
    else:
        raise SystemExit(__doc__)


if __name__ == "__main__":
    main(sys.argv)
