#!/usr/bin/env python3
"""Benchmark of the sparse-embedding hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload large|skew|seq|dlrm|tiny]

One step = one pass of the whole path (np_dedup, np_route, np_lookup_fwd, np_lookup_bwd,
np_sparse_adagrad) over one synthetic batch, inputs already resident in HBM.  Consecutive steps alternate
between two batches (the second built with 30 % distinct-key overlap where the configuration asks for it),
and the Adagrad update stays live between steps.  Prints ONE JSON line:

  value       lookups per second over the whole five-call step (np_dedup and np_route included)
  fwd_bwd_update  the subset the metric's name speaks of: np_lookup_fwd + np_lookup_bwd + np_sparse_adagrad
  roofline    the longest-running kernel: algorithmic bytes per launch / its mean duration (HIP events
              recorded by the library around the launches, on the launch stream) against 8 TB/s
  cpu_baseline  the CPU oracle on batch 0 on the host's cores (one thread, and one process per core)
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "measured_traffic.json")
GPU_BOX_CPU_SHARE = 16    # worker processes the CPU leg may use on a one-GPU machine, whatever os.cpu_count() shows


def algorithmic_bytes(n: int, U: int, B: int, D: int, S: int, mode: int, max_len: int, table_elem: int = 4) -> dict:
    """Compulsory HBM bytes of each call (every distinct row / element crosses HBM once)."""
    row = 4 * D
    trow = table_elem * D   # a table row as stored
    seq = mode == 2
    out_bytes = B * max_len * D * 2 if seq else B * row
    dy_bytes = n * D * 2 if seq else B * row
    return {
        "np_dedup": 8 * n + 4 * n + 4 * n + 16 * U,
        "np_route": 8 * U + 8 * U + 4 * U + 4 * U + 4 * S,
        "np_lookup_fwd": U * trow + 4 * n + 4 * B + out_bytes,
        "np_lookup_bwd": dy_bytes + 8 * n + 4 * U + U * row,
        "np_sparse_adagrad": U * row + 2 * U * trow + 16 * U,
    }


def measured_traffic(workload: str, kernel: str, table_dtype: str):
    """HBM-side bytes per launch of `kernel` from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs kept under profiles/
    (scaled by the copy-kernel calibration; the file is rewritten by `python -m paper_2604_06956_amd.profile_summary`
    together with the text summaries).  None when no profile of this workload / table type is on file."""
    try:
        with open(TRAFFIC_FILE) as f:
            table = json.load(f)
    except (OSError, ValueError):
        return None
    rec = table.get(f"{workload}/{table_dtype}", {}).get(kernel)
    return None if rec is None else float(rec["fetch_bytes"]) + float(rec["write_bytes"])


# the kernel that carries (nearly all of) each call's algorithmic bytes
KERNEL_OF_CALL = {"sparse_adagrad": "np_sparse_adagrad", "bwd_main": "np_lookup_bwd", "fwd_pool": "np_lookup_fwd",
                  "fwd_seq": "np_lookup_fwd"}


def call_of_kernel(k: str) -> str:
    return ("np_dedup" if k.startswith("dedup") else "np_route" if k.startswith("route") else
            "np_lookup_fwd" if k.startswith("fwd") else "np_lookup_bwd" if k.startswith("bwd") else "np_sparse_adagrad")


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="large")
    ap.add_argument("--table-dtype", choices=("f32", "bf16", "f16"), default="f32",
                    help="storage type of the table; bf16 / f16 run np_lookup_fwd_t / np_sparse_adagrad_t (not the headline)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-div", type=int, default=1, help="the CPU legs run on the first 1/div of batch 0's bags")
    ap.add_argument("--no-extras", action="store_true",
                    help="only the headline step and its per-kernel table (what a profiler run wants)")
    ap.add_argument("--cluster-only-8", action="store_true",
                    help="key-centric sample clustering for N = 8 only instead of every N of the micro-batch table (it runs on the host)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus above 1 is not supported (no collectives are built; "
              "the All2All exchanges are represented by np_route's send buffer).", file=sys.stderr)
        return 2

    from paper_2604_06956_amd import workloads as wl

    cfg = wl.config(args.workload)
    t_gen = time.time()
    b0 = wl.make_batch(cfg, 0, with_dy=False)
    b1 = wl.make_batch(cfg, 1, prev=b0, with_dy=False)
    batches = [b0, b1]
    stats = [wl.batch_stats(b.keys) for b in batches]
    K0, K1 = np.unique(b0.keys), np.unique(b1.keys)
    overlap = float(np.intersect1d(K0, K1, assume_unique=True).size / K1.size)
    del K0, K1
    gen_s = time.time() - t_gen

    # ---- the oracle on the host's cores, before this process touches the GPU (its worker processes are forked)
    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(cfg, b0, wl, args.cpu_sample_div, args.table_dtype)

    import torch
    from paper_2604_06956_amd import binding as B

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")

    R, D, S = cfg.num_rows, cfg.dim, cfg.num_shards
    seq = cfg.mode == wl.SEQ
    lowp_table = args.table_dtype != "f32"     # a 16-bit table, bf16 or fp16
    table = torch.empty((R, D), dtype={"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[args.table_dtype],
                        device=dev)
    state = torch.zeros(R, dtype=torch.float32, device=dev)
    if lowp_table:
        B.np_util_table_init_t(table, cfg.table_seed)
        fwd_call, adagrad_call = B.np_lookup_fwd_t, B.np_sparse_adagrad_t
    else:
        B.np_util_table_init(table, cfg.table_seed)
        fwd_call, adagrad_call = B.np_lookup_fwd, B.np_sparse_adagrad

    n_max = max(b.n for b in batches)
    cap = max(s["U"] for s in stats) + 1024
    max_len = max(b.max_len for b in batches)
    gen = torch.Generator(device=dev)
    gen.manual_seed(wl.BASE_SEED + cfg.index)
    dbatch = []
    for b in batches:
        shape = (cfg.num_bags, max_len, D) if seq else (cfg.num_bags, D)
        dY = torch.randn(shape, dtype=torch.float32, device=dev, generator=gen)
        if seq:
            dY = dY.bfloat16()
        dbatch.append(dict(keys=torch.from_numpy(b.keys).to(dev), off=torch.from_numpy(b.bag_offsets).to(dev), dY=dY, n=b.n))

    i32, i64 = torch.int32, torch.int64

    def dedup_buffers():
        return dict(unique=torch.empty(n_max, dtype=i64, device=dev), inverse=torch.empty(n_max, dtype=i32, device=dev),
                    counts=torch.empty(n_max, dtype=i32, device=dev), occ_offsets=torch.empty(n_max + 1, dtype=i32, device=dev),
                    occ=torch.empty(n_max, dtype=i32, device=dev), num_unique=torch.zeros(1, dtype=i32, device=dev))

    dd = dedup_buffers()
    # the unique-key count is known on the host for these synthetic batches, so U-sized buffers use cap, not n
    rr = dict(send_keys=torch.empty(cap, dtype=i64, device=dev), splits=torch.empty(S, dtype=i32, device=dev),
              send_offsets=torch.empty(S + 1, dtype=i32, device=dev), send_from_unique=torch.empty(cap, dtype=i32, device=dev),
              unique_to_send=torch.empty(cap, dtype=i32, device=dev))
    out_dtype = B.BF16 if seq else B.F32
    out = torch.empty((cfg.num_bags, max_len, D) if seq else (cfg.num_bags, D),
                      dtype=torch.bfloat16 if seq else torch.float32, device=dev)
    grads = torch.empty((cap, D), dtype=torch.float32, device=dev)
    ws_d = torch.empty(max(B.np_dedup_workspace_bytes(n_max, cfg.key_bits), 256), dtype=torch.uint8, device=dev)
    ws_r = torch.empty(max(B.np_route_workspace_bytes(cap, S), 256), dtype=torch.uint8, device=dev)
    ws_b = torch.empty(max(B.np_lookup_bwd_workspace_bytes(cfg.num_bags, n_max, D, cfg.mode), 256), dtype=torch.uint8, device=dev)

    # np_route needs only np_dedup's output and nothing before np_lookup_bwd needs np_route's, so it runs on a second
    # stream (default priority) beside np_lookup_fwd; events order the two streams around it
    side_stream = torch.cuda.Stream()
    ev_dedup = torch.cuda.Event()
    ev_route = torch.cuda.Event()

    def step(i: int, fwd_by: str = "keys", want_inverse: bool = True) -> None:
        """The five calls on one batch.  The table is local to this worker, so the forward reads it by key (list_keys = the
        batch's keys, idx = NULL); np_dedup still produces all of its outputs.  Gradients are reduced into send order and
        applied with the send-ordered keys (the layout of the gradient All2All).  fwd_by = "inverse" is the requester-side
        form of the forward, through (unique, inverse)."""
        bt = dbatch[i % 2]
        n = bt["n"]
        main_stream = torch.cuda.current_stream()   # the recording stream while a graph is being captured
        B.np_dedup(bt["keys"], cfg.key_bits, out=dd, ws=ws_d, want_inverse=want_inverse)
        ev_dedup.record(main_stream)
        side_stream.wait_event(ev_dedup)
        with torch.cuda.stream(side_stream):
            B.np_route(dd["unique"], dd["num_unique"], cap, S, cfg.shard_fn, out=rr, ws=ws_r)
            ev_route.record(side_stream)
        if fwd_by == "keys":
            fwd_call(table, bt["keys"], None, bt["off"], n, cfg.mode, max_len, out_dtype, out=out)
        else:
            fwd_call(table, dd["unique"], dd["inverse"], bt["off"], n, cfg.mode, max_len, out_dtype,
                     num_list=dd["num_unique"], cap=cap, out=out)
        main_stream.wait_event(ev_route)
        B.np_lookup_bwd(bt["dY"], D, cfg.mode, max_len, bt["off"], n, dd["occ_offsets"], dd["occ"], dd["num_unique"], cap,
                        unique_to_send=rr["unique_to_send"], grads=grads, ws=ws_b)
        adagrad_call(table, state, rr["send_keys"], grads, dd["num_unique"], cap, cfg.lr, cfg.eps)

    def timed_loop(fn, reps: int, warm: int = 2) -> float:
        """Mean wall milliseconds of fn(step index) over `reps` calls, bracketed by device synchronisations."""
        for i in range(warm):
            fn(args.warmup + i)
        torch.cuda.synchronize()
        t = time.perf_counter()
        for i in range(reps):
            fn(args.warmup + i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t) * 1e3 / reps

    def rate(ms: float) -> float:
        return n_steps_lookups(dbatch, args) / (ms * 1e-3 * args.steps)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    assert int(dd["num_unique"].item()) == stats[(args.warmup - 1) % 2]["U"] if args.warmup > 0 else True

    # ---- timed region: exactly K steps; the library records HIP events on the launch stream around the row kernels
    # that can be the dominant one (events around all ~27 launches of a step cost about 3 % of it)
    B.np_prof_only(list(KERNEL_OF_CALL))
    B.np_prof_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    timed_records = B.np_prof_collect(65536)
    B.np_prof_enable(False)
    B.np_prof_only(None)
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    lookups = n_steps_lookups(dbatch, args)
    value = lookups / (t1 - t0)

    # ---- the same K steps again, untimed for the headline, with events around every launch: the per-kernel table
    B.np_prof_enable(True)
    torch.cuda.synchronize()
    ta = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    ms_per_step_all_events = (time.perf_counter() - ta) * 1e3 / args.steps
    records = B.np_prof_collect(65536)
    B.np_prof_enable(False)

    kern = {}
    for name, ms in records:
        k = kern.setdefault(name, [0, 0.0])
        k[0] += 1
        k[1] += ms
    kernels = {k: {"launches_per_step": v[0] / args.steps, "ms_per_step": v[1] / args.steps, "avg_ms": v[1] / v[0]}
               for k, v in kern.items()}
    call_ms = {}
    for k, v in kernels.items():
        call_ms[call_of_kernel(k)] = call_ms.get(call_of_kernel(k), 0.0) + v["ms_per_step"]

    n_avg = float(np.mean([s["n"] for s in stats]))
    U_avg = float(np.mean([s["U"] for s in stats]))
    alg = algorithmic_bytes(int(n_avg), int(U_avg), cfg.num_bags, D, S, cfg.mode, max_len, 2 if lowp_table else 4)
    # the dominant kernel and its mean duration come from the events of the timed region
    timed = {}
    for name, ms in timed_records:
        tk = timed.setdefault(name, [0, 0.0])
        tk[0] += 1
        tk[1] += ms
    dominant = max(timed, key=lambda k: timed[k][1])
    dom_call = KERNEL_OF_CALL[dominant]
    dom_avg_ms = timed[dominant][1] / timed[dominant][0]
    achieved = alg[dom_call] / (dom_avg_ms * 1e-3) / 1e9
    fbu_ms = sum(call_ms.get(c, 0.0) for c in ("np_lookup_fwd", "np_lookup_bwd", "np_sparse_adagrad"))
    fbu_bytes = alg["np_lookup_fwd"] + alg["np_lookup_bwd"] + alg["np_sparse_adagrad"]

    # ---- np_route on its own (in the step it shares the GPU with the forward, so its event times there are not its cost)
    B.np_route(dd["unique"], dd["num_unique"], cap, S, cfg.shard_fn, out=rr, ws=ws_r)
    torch.cuda.synchronize()
    r0, r1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    r0.record()
    for _ in range(10):
        B.np_route(dd["unique"], dd["num_unique"], cap, S, cfg.shard_fn, out=rr, ws=ws_r)
    r1.record()
    torch.cuda.synchronize()
    route_alone_ms = r0.elapsed_time(r1) / 10

    # ---- bandwidth yardstick: a plain 16-byte copy kernel, 2 GiB each way
    words = 2 ** 31
    src = torch.empty(words, dtype=torch.uint8, device=dev)
    dst = torch.empty(words, dtype=torch.uint8, device=dev)
    B.np_util_stream_copy(dst, src)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        B.np_util_stream_copy(dst, src)
    e1.record()
    torch.cuda.synchronize()
    copy_gbs = 2 * words * 5 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del src, dst


    line = {
        "metric": "embedding lookups/sec (fwd+bwd+update) and achieved HBM GB/s on 1 MI355X",
        "value": value,
        "unit": "lookups/s",
        "value_is": "lookups per second over the WHOLE five-call step (np_dedup + np_route + np_lookup_fwd + np_lookup_bwd + "
                    "np_sparse_adagrad), the conservative reading of the metric; fwd_bwd_update.lookups_per_s is the three-call "
                    "subset the metric's name speaks of",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {len(cfg.table_rows)} table(s), {R} rows x dim {D} {args.table_dtype}, batch {cfg.batch} x "
                               f"{cfg.features} features, Zipf({cfg.alpha}), {S} shards, mode "
                               f"{['sum', 'mean', 'seq-bf16'][cfg.mode]}; step = dedup+route+fwd+bwd+adagrad",
                   "n_lookups": [s["n"] for s in stats], "unique_keys": [s["U"] for s in stats],
                   "hottest_key_count": [s["hottest"] for s in stats], "distinct_key_overlap": overlap,
                   "num_bags": cfg.num_bags, "max_len": max_len},
        "roofline": {"bound": "hbm", "kernel": dominant, "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": measured_traffic(cfg.name, dominant, args.table_dtype),
                     "algorithmic_bytes_per_launch": alg[dom_call], "avg_launch_ms": dom_avg_ms,
                     "launches_timed": timed[dominant][0]},
        "cpu_baseline": cpu,
        "fwd_bwd_update": {"ms_per_step": fbu_ms, "lookups_per_s": n_avg / (fbu_ms * 1e-3) if fbu_ms > 0 else None,
                           "algorithmic_GBps": fbu_bytes / (fbu_ms * 1e-3) / 1e9 if fbu_ms > 0 else None,
                           "frac_of_peak": fbu_bytes / (fbu_ms * 1e-3) / 1e9 / HBM_PEAK_GBS if fbu_ms > 0 else None,
                           "what": "sum of the HIP-event durations of the kernels of the three calls, per step"},
        "calls": {c: {"ms_per_step": call_ms.get(c, 0.0), "algorithmic_bytes": alg[c],
                      "algorithmic_GBps": alg[c] / (call_ms[c] * 1e-3) / 1e9 if call_ms.get(c, 0.0) > 0 else None}
                  for c in alg},
        "kernels": kernels,
        "streams": "np_route runs on a second stream beside np_lookup_fwd; its event times in `kernels` / `calls` include "
                   "that sharing, calls.np_route.alone_ms is its time with the GPU to itself",
        "ms_per_step_with_events_on_every_launch": ms_per_step_all_events,
        "stream_copy_GBps": copy_gbs,
        "input_generation_s": gen_s,
    }
    line["calls"]["np_route"]["alone_ms"] = route_alone_ms
    line["calls"]["np_route"]["alone_algorithmic_GBps"] = alg["np_route"] / (route_alone_ms * 1e-3) / 1e9
    for k in timed:   # every row kernel that was timed in the headline region, against its own call's algorithmic bytes
        line.setdefault("row_kernels", {})[k] = {
            "avg_launch_ms": timed[k][1] / timed[k][0], "algorithmic_bytes_per_launch": alg[KERNEL_OF_CALL[k]],
            "frac": alg[KERNEL_OF_CALL[k]] / (timed[k][1] / timed[k][0] * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "traffic": measured_traffic(cfg.name, k, args.table_dtype)}

    if not args.no_extras:
        extras(line, args, cfg, wl, B, torch, dev, batches, stats, dbatch, dd, rr, dedup_buffers, table, state, out, grads,
               ws_d, ws_r, ws_b, cap, n_max, max_len, out_dtype, fwd_call, adagrad_call, lowp_table, step, timed_loop, rate, alg,
               side_stream, ev_dedup, ev_route)
    print(json.dumps(line))
    return 0


def extras(line, args, cfg, wl, B, torch, dev, batches, stats, dbatch, dd, rr, dedup_buffers, table, state, out, grads, ws_d,
           ws_r, ws_b, cap, n_max, max_len, out_dtype, fwd_call, adagrad_call, lowp_table, step, timed_loop, rate, alg, side_stream,
           ev_dedup, ev_route) -> None:
    """Everything reported beside the headline: other forms of the step, the next-row features, yardsticks."""
    R, D, S = cfg.num_rows, cfg.dim, cfg.num_shards
    seq = cfg.mode == wl.SEQ
    i32, i64 = torch.int32, torch.int64
    K = args.steps

    # ---- the requester-side form of the forward: through (unique, inverse) instead of the raw keys
    inv_ms = timed_loop(lambda i: step(i, fwd_by="inverse"), K)
    line["forward_through_inverse_step"] = {
        "ms_per_step": inv_ms, "lookups_per_s": rate(inv_ms),
        "what": "np_lookup_fwd(list_keys = unique, idx = inverse): what a requester does with the owners' answers; no events"}

    # ---- the forward by key does not need np_dedup's result: it can run beside np_dedup and np_route on the second stream
    ev_begin, ev_fwd = torch.cuda.Event(), torch.cuda.Event()

    def step_fwd_beside_dedup(i: int) -> None:
        bt = dbatch[i % 2]
        n = bt["n"]
        main_stream = torch.cuda.current_stream()
        ev_begin.record(main_stream)            # after the previous step's update
        side_stream.wait_event(ev_begin)
        with torch.cuda.stream(side_stream):
            fwd_call(table, bt["keys"], None, bt["off"], n, cfg.mode, max_len, out_dtype, out=out)
            ev_fwd.record(side_stream)
        B.np_dedup(bt["keys"], cfg.key_bits, out=dd, ws=ws_d)
        B.np_route(dd["unique"], dd["num_unique"], cap, S, cfg.shard_fn, out=rr, ws=ws_r)
        main_stream.wait_event(ev_fwd)          # the dense model would sit here
        B.np_lookup_bwd(bt["dY"], D, cfg.mode, max_len, bt["off"], n, dd["occ_offsets"], dd["occ"], dd["num_unique"], cap,
                        unique_to_send=rr["unique_to_send"], grads=grads, ws=ws_b)
        adagrad_call(table, state, rr["send_keys"], grads, dd["num_unique"], cap, cfg.lr, cfg.eps)

    ovl_ms = timed_loop(step_fwd_beside_dedup, K)
    line["forward_beside_dedup_step"] = {
        "ms_per_step": ovl_ms, "lookups_per_s": rate(ovl_ms),
        "what": "np_lookup_fwd (by key) on the second stream beside np_dedup + np_route on the first; backward and update after both; no events"}

    # ---- a worker that reads its own table by key needs no inverse map at all: np_dedup without it
    local_ms = timed_loop(lambda i: step(i, want_inverse=False), K)
    line["local_table_step"] = {"ms_per_step": local_ms, "lookups_per_s": rate(local_ms),
                                "what": "as the headline, np_dedup called with inverse = NULL; no events"}

    # ---- backward and update fused (np_lookup_bwd_adagrad): its own byte model, U*row less written and read again
    def step_fused(i: int) -> None:
        bt = dbatch[i % 2]
        n = bt["n"]
        B.np_dedup(bt["keys"], cfg.key_bits, out=dd, ws=ws_d)
        B.np_route(dd["unique"], dd["num_unique"], cap, S, cfg.shard_fn, out=rr, ws=ws_r)
        fwd_call(table, bt["keys"], None, bt["off"], n, cfg.mode, max_len, out_dtype, out=out)
        (B.np_lookup_bwd_adagrad_t if lowp_table else B.np_lookup_bwd_adagrad)(
            bt["dY"], cfg.mode, max_len, bt["off"], n, dd["occ_offsets"], dd["occ"], dd["unique"], dd["num_unique"], cap, table,
            state, cfg.lr, cfg.eps, ws=ws_b)

    step_fused(0)
    B.np_prof_enable(True)
    fused_ms = timed_loop(step_fused, K, warm=0)
    frec = B.np_prof_collect(65536)
    B.np_prof_enable(False)
    fk = {}
    for name, ms in frec:
        fk[name] = fk.get(name, 0.0) + ms / K
    fused_bytes = alg["np_lookup_bwd"] + alg["np_sparse_adagrad"] - 2 * int(np.mean([s["U"] for s in stats])) * 4 * D
    bu_ms = sum(v for k, v in fk.items() if k.startswith("bwd"))
    fwd_ms = sum(v for k, v in fk.items() if k.startswith("fwd"))
    line["fused_bwd_update_step"] = {
        "ms_per_step": fused_ms, "lookups_per_s": rate(fused_ms), "bwd_update_ms": bu_ms,
        "kernels_ms": {k: v for k, v in fk.items() if k.startswith("bwd")},
        "algorithmic_bytes_bwd_update": fused_bytes,
        "bwd_update_algorithmic_GBps": fused_bytes / (bu_ms * 1e-3) / 1e9 if bu_ms > 0 else None,
        "fwd_bwd_update_frac_of_peak": ((alg["np_lookup_fwd"] + fused_bytes) / ((fwd_ms + bu_ms) * 1e-3) / 1e9 / HBM_PEAK_GBS
                                        if fwd_ms + bu_ms > 0 else None),
        "what": "np_lookup_bwd_adagrad instead of np_lookup_bwd + np_sparse_adagrad (a worker that owns the rows it reduces): "
                "the gradient rows are never written, so its byte model is the two calls' minus 2*U*row; events on every launch"}

    # ---- both sides of the sharded flow on the one GPU (what every GPU does around the three All2Alls): the owner
    # gathers the rows of the routed keys into the send buffer, the requester pools straight from that buffer through
    # lookup_to_send; backward and update as in the headline.  fp32 tables only.
    if not lowp_table:
        l2s = torch.empty(n_max, dtype=i32, device=dev)
        rows_buf = torch.empty((cap, D), dtype=torch.float32, device=dev)
        no_bags = torch.zeros(1, dtype=i32, device=dev)
        rr_full = dict(rr, lookup_to_send=l2s)

        def step_sharded(i: int) -> None:
            bt = dbatch[i % 2]
            n = bt["n"]
            B.np_dedup(bt["keys"], cfg.key_bits, out=dd, ws=ws_d)
            B.np_route(dd["unique"], dd["num_unique"], cap, S, cfg.shard_fn, inverse=dd["inverse"], n=n, out=rr_full, ws=ws_r)
            B.np_lookup_fwd(table, rr["send_keys"], None, no_bags, 0, cfg.mode, max_len, out_dtype, num_list=dd["num_unique"],
                            cap=cap, out=out, rows_out=rows_buf)
            B.np_lookup_fwd(rows_buf, None, l2s, bt["off"], n, cfg.mode, max_len, out_dtype, out=out)
            B.np_lookup_bwd(bt["dY"], D, cfg.mode, max_len, bt["off"], n, dd["occ_offsets"], dd["occ"], dd["num_unique"], cap,
                            unique_to_send=rr["unique_to_send"], grads=grads, ws=ws_b)
            B.np_sparse_adagrad(table, state, rr["send_keys"], grads, dd["num_unique"], cap, cfg.lr, cfg.eps)

        sharded_ms = timed_loop(step_sharded, K)
        line["sharded_flow_step"] = {
            "ms_per_step": sharded_ms, "lookups_per_s": rate(sharded_ms),
            "what": "owner-side row gather into the send buffer + requester-side pooling from it through lookup_to_send "
                    "(np_route with the composed map); backward and update as in the headline; no events"}
        del l2s, rows_buf

    # ---- the backward in two parts: its index work (np_lookup_bwd_prepare) behind np_route on the second stream, beside
    # the forward; the reduction (np_lookup_bwd_prepared) where np_lookup_bwd was.  Same bits.
    dy_dtype_code = B.BF16 if seq else B.F32

    def step_split(i: int) -> None:
        bt = dbatch[i % 2]
        n = bt["n"]
        main_stream = torch.cuda.current_stream()
        B.np_dedup(bt["keys"], cfg.key_bits, out=dd, ws=ws_d)
        ev_dedup.record(main_stream)
        side_stream.wait_event(ev_dedup)
        with torch.cuda.stream(side_stream):
            B.np_route(dd["unique"], dd["num_unique"], cap, S, cfg.shard_fn, out=rr, ws=ws_r)
            B.np_lookup_bwd_prepare(dy_dtype_code, D, cfg.mode, max_len, bt["off"], n, dd["occ_offsets"], dd["occ"], dd["num_unique"], ws_b)
            ev_route.record(side_stream)
        fwd_call(table, bt["keys"], None, bt["off"], n, cfg.mode, max_len, out_dtype, out=out)
        main_stream.wait_event(ev_route)
        B.np_lookup_bwd_prepared(bt["dY"], D, cfg.mode, max_len, bt["off"], n, dd["occ_offsets"], dd["occ"], dd["num_unique"], cap,
                                 ws_b, unique_to_send=rr["unique_to_send"], grads=grads)
        adagrad_call(table, state, rr["send_keys"], grads, dd["num_unique"], cap, cfg.lr, cfg.eps)

    split_ms = timed_loop(step_split, K)
    line["prepared_bwd_step"] = {"ms_per_step": split_ms, "lookups_per_s": rate(split_ms),
                                 "what": "np_lookup_bwd_prepare behind np_route on the second stream, np_lookup_bwd_prepared after the forward"}
    # the two alternatives of the backward that np_tune_set switches on (same bits, see include/nestpipe.h)
    tuned = {}
    for knob, fn in (("bwd_row_index", step_split), ("bwd_row_index", step), ("bwd_singles_by_bag", step)):
        old_v = B.np_tune_get(knob)
        B.np_tune_set(knob, 1)
        B.np_prof_enable(True)
        ms = timed_loop(fn, K)
        rec = B.np_prof_collect(65536)
        B.np_prof_enable(False)
        B.np_tune_set(knob, old_v)
        per = {}
        for name, t_ms in rec:
            if name.startswith("bwd"):
                per[name] = per.get(name, 0.0) + t_ms / (K + 2)
        tuned[knob + ("/prepared_on_second_stream" if fn is step_split else "")] = {
            "ms_per_step_with_events": ms, "bwd_kernels_ms": per, "bwd_ms": sum(per.values())}
    line["backward_variants"] = tuned

    # ---- the headline step without event recording (what the events cost), and its spread over single steps
    line["ms_per_step_without_events"] = timed_loop(step, K, warm=0)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(K + 1)]
    marks[0].record()
    for i in range(K):
        step(args.warmup + i)
        marks[i + 1].record()
    torch.cuda.synchronize()
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(K))
    line["step_time_spread"] = {"min_ms": per_step[0], "median_ms": per_step[len(per_step) // 2], "max_ms": per_step[-1]}

    # ---- the same step recorded into one HIP graph per batch and replayed (the library only enqueues kernels, so a
    # caller can do this; the launch-bound small workloads gain, configuration 5 does not)
    graphs = []
    for b in range(2):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            step(b)
        graphs.append(g)
    graph_ms = timed_loop(lambda i: graphs[i % 2].replay(), K)
    line["hip_graph_replay"] = {"ms_per_step": graph_ms, "lookups_per_s": rate(graph_ms)}
    del graphs

    # ---- gather yardstick: random 256-byte row reads with the row kernels' access pattern, by working-set size (what L2,
    # the last-level cache and HBM deliver to a gather on this GPU; the table itself is the source)
    if not lowp_table and table.numel() >= 64 * 4096:
        flat = table.view(-1)
        rows_total = flat.numel() // 64
        n_g = 32 << 20
        sink = torch.empty((n_g // 64, 64), dtype=torch.float32, device=dev)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        gy = {}
        for label, rows in (("2MB_L2", 8192), ("128MB_last_level_cache", 1 << 19), ("1GB", 1 << 22), ("whole_table_HBM", rows_total)):
            rows = min(rows, rows_total, (1 << 32) - 1)
            B.np_util_gather_rate(flat, rows, n_g, 1, sink)
            torch.cuda.synchronize()
            e0.record()
            for rep in range(3):
                B.np_util_gather_rate(flat, rows, n_g, 2 + rep, sink)
            e1.record()
            torch.cuda.synchronize()
            gy[label] = {"working_set_bytes": rows * 256, "GBps": 3 * n_g * 256 / (e0.elapsed_time(e1) * 1e-3) / 1e9}
        line["row_gather_GBps"] = gy
        del sink

    if not lowp_table and not seq:
        line["dual_buffer"] = dual_buffer(args, cfg, B, torch, dev, dbatch, dd, dedup_buffers, table, state, out, grads, ws_d, ws_b,
                                          cap, n_max, max_len, out_dtype)
    line["frozen_window_dedup"] = frozen_window(args, cfg, B, torch, batches, stats, dbatch, dd, ws_d)


def dual_buffer(args, cfg, B, torch, dev, dbatch, dd1, dedup_buffers, table, state, out, grads, ws_d, ws_b, cap, n_max, max_len,
                out_dtype) -> dict:
    """Section IV-B on the two batches: the synchronisation on its own, and the inter-batch pipeline (B_t's prefetch on a
    second stream before B_{t-1}'s update, then intersect + row copy, then B_t's forward from the prefetch buffer) against
    the plain sequential order (B_{t-1}'s backward and update on the table, then B_t's forward from the table).  Timed from
    the point where both batches are deduplicated."""
    D = cfg.dim
    i32, i64 = torch.int32, torch.int64
    dd2 = dedup_buffers()
    B.np_dedup(dbatch[0]["keys"], cfg.key_bits, out=dd1, ws=ws_d)
    B.np_dedup(dbatch[1]["keys"], cfg.key_bits, out=dd2, ws=ws_d)
    active = torch.empty((cap, D), dtype=torch.float32, device=dev)
    prefetch = torch.empty((cap, D), dtype=torch.float32, device=dev)
    astate = torch.zeros(cap, dtype=torch.float32, device=dev)
    iota = torch.arange(cap, dtype=i64, device=dev)
    no_bags = torch.zeros(1, dtype=i32, device=dev)
    isec = dict(idx_a=torch.empty(cap, dtype=i32, device=dev), idx_b=torch.empty(cap, dtype=i32, device=dev),
                num_common=torch.zeros(1, dtype=i32, device=dev))
    ws_i = torch.empty(max(int(B.lib.np_intersect_workspace_bytes(cap)), 256), dtype=torch.uint8, device=dev)
    b1, b2 = dbatch[0], dbatch[1]
    # the synchronisation alone, per kernel
    B.np_intersect(dd1["unique"], dd1["num_unique"], cap, dd2["unique"], dd2["num_unique"], cap, out=isec, ws=ws_i)
    B.np_sync_rows(active, isec["idx_a"], prefetch, isec["idx_b"], isec["num_common"], cap)
    torch.cuda.synchronize()
    B.np_prof_enable(True)
    reps = 5
    for _ in range(reps):
        B.np_intersect(dd1["unique"], dd1["num_unique"], cap, dd2["unique"], dd2["num_unique"], cap, out=isec, ws=ws_i)
        B.np_sync_rows(active, isec["idx_a"], prefetch, isec["idx_b"], isec["num_common"], cap)
    torch.cuda.synchronize()
    sync_rec = B.np_prof_collect(1024)
    B.np_prof_enable(False)
    common = int(isec["num_common"].item())
    sync_k = {}
    for name, ms in sync_rec:
        sync_k[name] = sync_k.get(name, 0.0) + ms / reps

    main = torch.cuda.current_stream()
    side = torch.cuda.Stream()
    ev_go, ev_prefetched = torch.cuda.Event(), torch.cuda.Event()

    def sequential() -> None:
        B.np_lookup_bwd(b1["dY"], D, cfg.mode, max_len, b1["off"], b1["n"], dd1["occ_offsets"], dd1["occ"], dd1["num_unique"], cap,
                        grads=grads, ws=ws_b)
        B.np_sparse_adagrad(table, state, dd1["unique"], grads, dd1["num_unique"], cap, cfg.lr, cfg.eps)
        B.np_lookup_fwd(table, dd2["unique"], dd2["inverse"], b2["off"], b2["n"], cfg.mode, max_len, out_dtype,
                        num_list=dd2["num_unique"], cap=cap, out=out)

    def pipelined() -> None:
        ev_go.record(main)
        side.wait_event(ev_go)
        with torch.cuda.stream(side):   # B_t's prefetch: its rows as the table holds them now (W_t)
            B.np_lookup_fwd(table, dd2["unique"], None, no_bags, 0, cfg.mode, max_len, out_dtype, num_list=dd2["num_unique"], cap=cap,
                            out=out, rows_out=prefetch)
            ev_prefetched.record(side)
        B.np_lookup_bwd(b1["dY"], D, cfg.mode, max_len, b1["off"], b1["n"], dd1["occ_offsets"], dd1["occ"], dd1["num_unique"], cap,
                        grads=grads, ws=ws_b)
        B.np_sparse_adagrad(active, astate, iota, grads, dd1["num_unique"], cap, cfg.lr, cfg.eps)   # the update, on the active buffer
        B.np_intersect(dd1["unique"], dd1["num_unique"], cap, dd2["unique"], dd2["num_unique"], cap, out=isec, ws=ws_i)
        main.wait_event(ev_prefetched)
        B.np_sync_rows(active, isec["idx_a"], prefetch, isec["idx_b"], isec["num_common"], cap)
        B.np_lookup_fwd(prefetch, iota, dd2["inverse"], b2["off"], b2["n"], cfg.mode, max_len, out_dtype,
                        num_list=dd2["num_unique"], cap=cap, out=out)

    def wall(fn) -> float:
        fn()
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t) * 1e3 / reps

    # B_{t-1}'s rows are in the active buffer (its own prefetch)
    B.np_lookup_fwd(table, dd1["unique"], None, no_bags, 0, cfg.mode, max_len, out_dtype, num_list=dd1["num_unique"], cap=cap, out=out,
                    rows_out=active)
    seq_ms = wall(sequential)
    pipe_ms = wall(pipelined)
    return {"common_keys": common, "sync_ms": sum(sync_k.values()), "sync_kernels_ms": sync_k,
            "row_copy_GBps": 2 * common * 4 * D / (sync_k.get("sync_rows", 1e9) * 1e-3) / 1e9,
            "two_batch_sequential_ms": seq_ms, "two_batch_pipelined_ms": pipe_ms,
            "what": "sequential = bwd(B1), adagrad on the table, fwd(B2) from the table, one stream; pipelined = prefetch of B2's rows "
                    "on a second stream beside bwd(B1) + adagrad on the active row buffer, then np_intersect + np_sync_rows, then "
                    "fwd(B2) from the prefetch buffer.  With the table in HBM the prefetch has no slower tier to hide: it is extra "
                    "traffic on the one memory system, so the pipelined order is not expected to win here"}


def frozen_window(args, cfg, B, torch, batches, stats, dbatch, dd, ws_d) -> dict:
    """Frozen-window micro-batching (Section V): keys are deduplicated inside each micro-batch only, so the vectors crossing
    the All2All inflate from U to sum(U_i).  Batch 0 split into N micro-batches of consecutive samples and by the key-centric sample clustering of Section V-C; every micro-batch goes through np_dedup."""
    from paper_2604_06956_amd import clustering as C
    b0 = batches[0]
    keys_dev = dbatch[0]["keys"]
    B.np_dedup(keys_dev, cfg.key_bits, out=dd, ws=ws_d)
    torch.cuda.synchronize()
    U = int(dd["num_unique"].item())
    inverse = dd["inverse"][:b0.n].cpu().numpy()
    counts = dd["counts"][:U].cpu().numpy()
    table = {}

    def sum_u(assign, N):
        tot = 0
        for m in range(N):
            pos, _, _ = C.micro_batch_lookups(b0.bag_offsets, cfg.batch, cfg.features, assign, m)
            if pos.size == 0:
                continue
            mk = keys_dev[torch.from_numpy(pos).to(keys_dev.device)].contiguous()
            B.np_dedup(mk, cfg.key_bits, out=dd, ws=ws_d)
            torch.cuda.synchronize()
            tot += int(dd["num_unique"].item())
        return tot

    for N in (1, 2, 4, 8, 16, 32):
        if cfg.batch < N:
            continue
        rec = {"consecutive": sum_u(C.consecutive_split(cfg.batch, N), N) / stats[0]["U"]}
        if N > 1 and (N == 8 or not args.cluster_only_8):
            t = time.perf_counter()
            assign = C.cluster_samples(b0.keys, b0.bag_offsets, cfg.batch, N, inverse=inverse, counts=counts)
            rec["clustering_host_s"] = time.perf_counter() - t
            rec["clustered"] = sum_u(assign, N) / stats[0]["U"]
        table[str(N)] = rec
    table["what"] = "sum over micro-batches of their distinct-key counts / the whole batch's U (batch 0)"
    return table


def n_steps_lookups(dbatch, args) -> int:
    return sum(dbatch[(args.warmup + i) % 2]["n"] for i in range(args.steps))


def _oracle_leg(cfg_tuple, keys, off, max_len, table_seed, table_dtype, wl_module_name="paper_2604_06956_amd.workloads"):
    """The five oracle steps on one slice of bags (its own little batch), timed; runs in the calling process."""
    import importlib
    wl = importlib.import_module(wl_module_name)
    from oracle import np_oracle as O
    dim, mode, num_shards, shard_fn, lr, eps = cfg_tuple
    nb = off.shape[0] - 1
    n = int(off[-1])
    touched = np.unique(keys)
    local = np.searchsorted(touched, keys).astype(np.int64)
    table = wl.table_init_rows(touched, dim, table_seed)
    if table_dtype == "bf16":
        table = O.f32_to_bf16_bits(table) if table.size < 1 << 16 else (
            ((table.view(np.uint32) + 0x7FFF + ((table.view(np.uint32) >> 16) & 1)) >> 16).astype(np.uint16))
    elif table_dtype == "f16":
        table = table.astype(np.float16)
    state = np.zeros(touched.shape[0], np.float32)
    rng = np.random.default_rng(1)
    seq = mode == 2
    if seq:
        dY = (rng.standard_normal((nb, max_len, dim)).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
    else:
        dY = rng.standard_normal((nb, dim)).astype(np.float32)
    t0 = time.perf_counter()
    unique, inverse, counts, occ_offsets, occ = O.dedup(local)
    t1 = time.perf_counter()
    send_keys, splits, send_offsets, sfu, uts = O.route(touched[unique], num_shards, shard_fn)
    l2s = O.compose(inverse, uts)
    t2 = time.perf_counter()
    O.lookup_fwd(table, unique[sfu], l2s, off, mode, max_len, O.BF16 if seq else O.F32)
    t3 = time.perf_counter()
    grads, _ = O.lookup_bwd(dY, O.BF16 if seq else O.F32, dim, mode, max_len, off, inverse, unique.shape[0], uts)
    t4 = time.perf_counter()
    if table_dtype == "bf16":
        O.sparse_adagrad_bf16(table, state, unique[sfu], grads, lr, eps)
    elif table_dtype == "f16":
        O.sparse_adagrad_f16(table.view(np.uint16), state, unique[sfu], grads, lr, eps)
    else:
        O.sparse_adagrad(table, state, unique[sfu], grads, lr, eps)
    t5 = time.perf_counter()
    return n, touched.shape[0], (t1 - t0, t2 - t1, t3 - t2, t4 - t3, t5 - t4)


_FORK_STATE = {}


def _oracle_worker(w: int):
    st = _FORK_STATE
    lo, hi = st["cuts"][w], st["cuts"][w + 1]
    off = st["off"][lo:hi + 1]
    keys = st["keys"][int(off[0]):int(off[-1])]
    t = time.perf_counter()
    n, u, per = _oracle_leg(st["cfg_tuple"], keys, (off - off[0]).astype(np.int32), st["max_len"], st["table_seed"], st["table_dtype"])
    return n, u, per, time.perf_counter() - t


def cpu_baseline(cfg, batch, wl, div: int, table_dtype: str = "f32"):
    """The CPU oracle, as it stands, on (the first 1/div of) batch 0: all five steps on a table that holds only the rows the
    sample touches (keys renumbered in order, which changes no result of the path).  Two legs: one thread over the whole
    sample; and one worker process per core, each running the same five steps on its own contiguous share of the bags (the
    oracle is single-threaded C, so this is how it uses the cores; per-share deduplication, as N workers would)."""
    import multiprocessing as mp
    from oracle import np_oracle as O
    O.build()
    nb = max(1, cfg.num_bags // max(div, 1))
    off = batch.bag_offsets[:nb + 1].astype(np.int64)
    n = int(off[-1])
    keys = batch.keys[:n]
    cfg_tuple = (cfg.dim, cfg.mode, cfg.num_shards, cfg.shard_fn, cfg.lr, cfg.eps)
    host_cores = os.cpu_count() or 1
    procs = max(1, min(host_cores, GPU_BOX_CPU_SHARE, nb))
    # ---- all cores: fork the workers before anything else in this process holds threads or a GPU context
    _FORK_STATE.update(cuts=[nb * w // procs for w in range(procs + 1)], off=off, keys=keys, cfg_tuple=cfg_tuple,
                       max_len=batch.max_len, table_seed=cfg.table_seed, table_dtype=table_dtype)
    t = time.perf_counter()
    if procs > 1:
        with mp.get_context("fork").Pool(procs) as pool:
            res = pool.map(_oracle_worker, range(procs))
    else:
        res = [_oracle_worker(0)]
    wall_all = time.perf_counter() - t
    busy = max(r[3] for r in res)
    # ---- one thread over the whole sample
    t = time.perf_counter()
    n1, u1, per1 = _oracle_leg(cfg_tuple, keys, off.astype(np.int32), batch.max_len, cfg.table_seed, table_dtype)
    wall_one = time.perf_counter() - t
    _FORK_STATE.clear()
    total1 = sum(per1)
    names = ("dedup", "route", "fwd", "bwd", "adagrad")
    return {"value": n / busy, "unit": "lookups/s", "cores": procs, "host_cores": host_cores, "kind": "oracle",
            "sample": f"first {nb} of {cfg.num_bags} bags of batch 0 ({n} lookups), all five steps, table holding only the touched "
                      f"rows; {procs} worker processes (one per core, at most {GPU_BOX_CPU_SHARE} on a one-GPU box), each the "
                      f"single-threaded C oracle (fp64 accumulation) on its contiguous share of the bags; value = lookups / the "
                      f"slowest worker's time, inputs in memory",
            "seconds": busy, "wall_seconds_with_process_start": wall_all,
            "one_thread": {"value": n1 / total1, "unit": "lookups/s", "cores": 1, "seconds": total1, "distinct_keys": u1,
                           "seconds_per_call": dict(zip(names, per1)), "wall_seconds_with_table_setup": wall_one}}


if __name__ == "__main__":
    sys.exit(main())
