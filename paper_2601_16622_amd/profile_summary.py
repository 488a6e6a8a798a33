"""Turns rocprofv3 result databases into the short text summaries kept under profiles/.

    python -m paper_2601_16622_amd.profile_summary trace  <trace_results.db> [rows]
    python -m paper_2601_16622_amd.profile_summary pmc    <fetch_results.db> <write_results.db> <copy_bytes>

`trace` prints per-kernel call counts and mean durations (what `rocprofv3 --kernel-trace --stats` collects).
`counters` prints the mean of every collected counter for the kernels whose name contains a pattern.
`pmc` prints FETCH_SIZE / WRITE_SIZE per kernel (KiB per dispatch), scaled by what the same counters read for the
plain device copy of <copy_bytes> bytes that `bench.py --copy-calibration` runs in the same process.
"""
import sqlite3
import sys


def trace(db, rows=14):
    con = sqlite3.connect(db)
    print(f"{'calls':>6} {'mean_us':>12} {'total_ms':>10} {'%':>6}  kernel")
    for name, calls, total, avg, pct in con.execute(
            "select name, total_calls, total_duration, average, percentage from top_kernels limit %d" % int(rows)):
        print(f"{calls:6d} {avg:12.2f} {total / 1e3:10.3f} {pct:6.2f}  {name[:110]}")


def _per_kernel(db, counter):
    con = sqlite3.connect(db)
    rows = con.execute("select kernel_name, count(*), avg(value), max(value) from counters_collection "
                       "where counter_name=? group by kernel_name", (counter,)).fetchall()
    return {r[0]: r[1:] for r in rows}


def pmc(fetch_db, write_db, copy_bytes):
    fetch, write = _per_kernel(fetch_db, "FETCH_SIZE"), _per_kernel(write_db, "WRITE_SIZE")
    copy_kib = copy_bytes / 1024.0
    copy_name = "__amd_rocclr_copyBuffer"
    f_scale = copy_kib / fetch[copy_name][2]
    w_scale = copy_kib / write[copy_name][2]
    print(f"copy of {copy_bytes} bytes: FETCH_SIZE reads {fetch[copy_name][2]:.1f} KiB (scale {f_scale:.3f}), "
          f"WRITE_SIZE reads {write[copy_name][2]:.1f} KiB (scale {w_scale:.3f})")
    print(f"{'dispatches':>10} {'fetch_MB':>12} {'write_MB':>12}  kernel (scaled, per dispatch)")
    marked = False
    for name in sorted(fetch, key=lambda k: -fetch[k][1]):
        if name.startswith("void at::") or name == copy_name:
            continue
        f = fetch[name][1] * f_scale * 1024 / 1e6
        w = write.get(name, (0, 0, 0))[1] * w_scale * 1024 / 1e6
        print(f"{fetch[name][0]:10d} {f:12.2f} {w:12.2f}  {name[:100]}")
        if not marked and ("k_tile_heads" in name or "k_fused" in name):   # the attention kernel of the timed path
            print(f"traffic_bytes_per_launch: {(f + w) * 1e6:.0f}")
            marked = True


def counters(db, pattern):
    """Mean value per dispatch of every counter collected in this run, for kernels whose name contains `pattern`."""
    con = sqlite3.connect(db)
    rows = con.execute("select kernel_name, counter_name, avg(value), count(*) from counters_collection "
                       "group by kernel_name, counter_name").fetchall()
    seen = {}
    for name, counter, value, n in rows:
        if pattern in name:
            seen.setdefault(name, []).append((counter, value, n))
    for name, items in seen.items():
        print(name[:110])
        for counter, value, n in sorted(items):
            print(f"    {counter:<32} {value:16.6g}   (mean over {n} dispatches)")


if __name__ == "__main__":
    if sys.argv[1] == "trace":
        trace(sys.argv[2], sys.argv[3] if len(sys.argv) > 3 else 14)
    elif sys.argv[1] == "counters":
        counters(sys.argv[2], sys.argv[3])
    else:
        pmc(sys.argv[2], sys.argv[3], int(sys.argv[4]))
