"""Turns the CSV output of four rocprofv3 runs of bench.py into the short text summary kept under profiles/ and into
the per-kernel traffic table bench.py reads (profiles/measured_traffic.json).

    cd /tmp && export TMPDIR=/tmp          # R = the repository
    rocprofv3 --kernel-trace --stats --output-format csv -d OUT/trace -o t -- python3 R/bench.py --workload W --steps 5 --warmup 2 --no-cpu-baseline --no-extras
    rocprofv3 --pmc FETCH_SIZE --output-format csv -d OUT/fetch -o f -- python3 R/bench.py --workload W --steps 3 --warmup 1 --no-cpu-baseline --no-extras
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d OUT/write -o w -- python3 R/bench.py --workload W --steps 3 --warmup 1 --no-cpu-baseline --no-extras
    rocprofv3 --pmc TCC_HIT_sum TCC_MISS_sum TCC_REQ_sum --output-format csv -d OUT/l2 -o l -- python3 R/bench.py --workload W --steps 3 --warmup 1 --no-cpu-baseline --no-extras
    python3 -m paper_2604_06956_amd.profile_summary OUT W [table dtype] [--update-traffic] > profiles/W_step_kernels.txt

FETCH_SIZE and WRITE_SIZE are in KiB per dispatch.  On this GPU FETCH_SIZE reads half of the bytes a plain copy kernel
reads (np_util_stream_copy, 2 GiB, counts 1 GiB), WRITE_SIZE reads them exactly: the factors 2.0 and 1.0 below, checked
again whenever the trace holds a stream_copy dispatch.  FETCH_SIZE counts what L2 asks of the fabric, so Infinity Cache
hits are part of it.
"""
from __future__ import annotations

import collections
import csv
import glob
import json
import os
import sys

FETCH_SCALE, WRITE_SCALE = 2.0, 1.0
SHORT = (("bwd_main_kernel", "bwd_main"), ("bwd_fixup_kernel", "bwd_fixup"), ("bwd_prepare_kernel", "bwd_prepare"),
         ("fwd_pool", "fwd_pool"), ("fwd_seq", "fwd_seq"), ("fwd_rows", "fwd_rows"), ("adagrad_kernel", "sparse_adagrad"),
         ("dedup_emit", "dedup_emit"), ("dedup_count_heads", "dedup_count_heads"), ("dedup_counts", "dedup_counts"),
         ("dedup_tile_heads", "dedup_tile_heads"), ("dedup_tile_scan", "dedup_tile_scan"),
         ("part_scatter_kernel<np::EmitOrder", "dedup_order_scatter"), ("part_hist_kernel<np::EmitOrder", "dedup_order_hist"),
         ("bwd_rows", "bwd_rows"), ("bwd_single", "bwd_single"), ("gather_rate", "gather_rate"),
         ("part_scatter_kernel<np::Sort", "dedup_sort_scatter"), ("part_hist_kernel<np::Sort", "dedup_sort_hist"),
         ("part_scatter_kernel<np::Route", "route_scatter"), ("part_hist_kernel<np::Route", "route_hist"),
         ("part_scatter_kernel<np::TileOrder", "bwd_order_scatter"), ("part_hist_kernel<np::TileOrder", "bwd_order_hist"),
         ("part_colscan", "colscan"), ("stream_copy", "stream_copy"), ("table_init", "table_init"))


def short(name: str) -> str:
    for pat, s in SHORT:
        if pat in name:
            return s
    return name[:40]


def find(out: str, pat: str):
    g = glob.glob(os.path.join(out, pat), recursive=True)
    return g[0] if g else None


def counter_means(path: str, wanted):
    """-> {kernel short name: {counter: (mean, min, max, dispatches)}}"""
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    if path:
        with open(path) as f:
            for r in csv.DictReader(f):
                if r.get("Counter_Name") in wanted:
                    acc[short(r["Kernel_Name"])][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return {k: {c: (sum(v) / len(v), min(v), max(v), len(v)) for c, v in d.items()} for k, d in acc.items()}


def main(argv) -> int:
    if len(argv) < 3:
        print(__doc__)
        return 2
    out, workload = argv[1], argv[2]
    dtype = argv[3] if len(argv) > 3 and not argv[3].startswith("--") else "f32"
    update = "--update-traffic" in argv
    st = find(out, "trace/**/*kernel_stats.csv")
    print(f"# kernel stats (rocprofv3 --kernel-trace --stats), workload {workload}, table {dtype}")
    if st:
        with open(st) as f:
            for r in list(csv.DictReader(f))[:24]:
                print(f"{short(r.get('Name', '')):22s} calls={r.get('Calls'):>5s} avg_us={float(r.get('AverageNs', 0)) / 1e3:10.1f} "
                      f"total_ms={float(r.get('TotalDurationNs', 0)) / 1e6:9.2f} pct={r.get('Percentage')}")
    fetch = counter_means(find(out, "fetch/**/*counter_collection.csv"), ("FETCH_SIZE",))
    write = counter_means(find(out, "write/**/*counter_collection.csv"), ("WRITE_SIZE",))
    l2 = counter_means(find(out, "l2/**/*counter_collection.csv"), ("TCC_HIT_sum", "TCC_MISS_sum", "TCC_REQ_sum"))
    if "stream_copy" in fetch and "stream_copy" in write:
        print(f"# calibration: stream_copy (2 GiB = 2097152 KiB each way) reads FETCH_SIZE {fetch['stream_copy']['FETCH_SIZE'][0]:.0f} KiB, "
              f"WRITE_SIZE {write['stream_copy']['WRITE_SIZE'][0]:.0f} KiB")
    print(f"# traffic per launch: FETCH_SIZE x {FETCH_SCALE} and WRITE_SIZE x {WRITE_SCALE} KiB -> GB (mean over dispatches; min..max of the raw counter), "
          "L2 requests per launch and hit rate")
    table = {}
    for k in sorted(set(fetch) | set(write), key=lambda k: -(fetch.get(k, {}).get("FETCH_SIZE", (0,))[0])):
        f = fetch.get(k, {}).get("FETCH_SIZE", (0.0, 0.0, 0.0, 0))
        w = write.get(k, {}).get("WRITE_SIZE", (0.0, 0.0, 0.0, 0))
        fb, wb = f[0] * 1024 * FETCH_SCALE, w[0] * 1024 * WRITE_SCALE
        if fb + wb < 20e6:
            continue
        m = {c: v[0] for c, v in l2.get(k, {}).items()}
        h, ms = m.get("TCC_HIT_sum", 0.0), m.get("TCC_MISS_sum", 0.0)
        hr = h / (h + ms) if h + ms > 0 else float("nan")
        print(f"{k:22s} fetch {fb / 1e9:7.3f} GB ({f[1]:.0f}..{f[2]:.0f} KiB, n={f[3]})  write {wb / 1e9:7.3f} GB ({w[1]:.0f}..{w[2]:.0f} KiB, n={w[3]})  "
              f"L2 req {m.get('TCC_REQ_sum', 0):.4g} hit rate {hr:.3f}")
        table[k] = {"fetch_bytes": fb, "write_bytes": wb, "l2_requests": m.get("TCC_REQ_sum"), "l2_hit_rate": None if hr != hr else hr}
    if update:
        root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
        path = os.path.join(root, "profiles", "measured_traffic.json")
        try:
            with open(path) as f:
                allt = json.load(f)
        except (OSError, ValueError):
            allt = {}
        allt[f"{workload}/{dtype}"] = table
        with open(path, "w") as f:
            json.dump(allt, f, indent=1, sort_keys=True)
            f.write("\n")
        print(f"# wrote {workload}/{dtype} into profiles/measured_traffic.json", file=sys.stderr)
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
