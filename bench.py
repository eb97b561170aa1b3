#!/usr/bin/env python3
"""Benchmark of the sparse-embedding hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload large|skew|seq|dlrm|tiny]

One step = one pass of the whole path (np_dedup, np_route, np_lookup_fwd, np_lookup_bwd,
np_sparse_adagrad) over one synthetic batch, inputs already resident in HBM.  Consecutive steps alternate
between two batches (the second built with 30 % distinct-key overlap where the configuration asks for it),
and the Adagrad update stays live between steps.  Prints ONE JSON line:

  value       lookups per second over the whole five-call step
  roofline    the longest-running kernel: algorithmic bytes per launch / its mean duration (HIP events
              recorded by the library around every launch, on the launch stream) against 8 TB/s
  cpu_baseline  the CPU oracle timed on a bounded sample of the same batch on the host cores
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


# HBM-side bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by the copy-kernel
# calibration; see profiles/large_step_kernels.txt), keyed by (workload, kernel).  Static: bench.py cannot run
# the profiler on itself.
MEASURED_TRAFFIC = {("large", "bwd_main"): 14.59e9, ("large", "fwd_pool"): 9.52e9, ("large", "sparse_adagrad"): 8.38e9}

# the kernel that carries (nearly all of) each call's algorithmic bytes
KERNEL_OF_CALL = {"sparse_adagrad": "np_sparse_adagrad", "bwd_main": "np_lookup_bwd", "fwd_pool": "np_lookup_fwd",
                  "fwd_seq": "np_lookup_fwd"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="large")
    ap.add_argument("--table-dtype", choices=("f32", "bf16", "f16"), default="f32",
                    help="storage type of the table; bf16 / f16 run np_lookup_fwd_t / np_sparse_adagrad_t (not the headline)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-div", type=int, default=2)
    ap.add_argument("--fwp-report", action="store_true",
                    help="also dedup batch 0 split into N micro-batches of consecutive samples and report sum(U_i)/U")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus above 1 is not supported (no collectives are built; "
              "the All2All exchanges are represented by np_route's send buffer).", file=sys.stderr)
        return 2

    import torch
    from paper_2604_06956_amd import binding as B
    from paper_2604_06956_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")

    cfg = wl.config(args.workload)
    t_gen = time.time()
    b0 = wl.make_batch(cfg, 0, with_dy=False)
    b1 = wl.make_batch(cfg, 1, prev=b0, with_dy=False)
    batches = [b0, b1]
    stats = [wl.batch_stats(b.keys) for b in batches]
    K0, K1 = np.unique(b0.keys), np.unique(b1.keys)
    overlap = float(np.intersect1d(K0, K1, assume_unique=True).size / K1.size)
    gen_s = time.time() - t_gen

    R, D, S = cfg.num_rows, cfg.dim, cfg.num_shards
    seq = cfg.mode == wl.SEQ
    bf16_table = args.table_dtype != "f32"     # a 16-bit table, bf16 or fp16
    table = torch.empty((R, D), dtype={"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[args.table_dtype],
                        device=dev)
    state = torch.zeros(R, dtype=torch.float32, device=dev)
    if bf16_table:
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
    dd = dict(unique=torch.empty(n_max, dtype=i64, device=dev), inverse=torch.empty(n_max, dtype=i32, device=dev),
              counts=torch.empty(n_max, dtype=i32, device=dev), occ_offsets=torch.empty(n_max + 1, dtype=i32, device=dev),
              occ=torch.empty(n_max, dtype=i32, device=dev), num_unique=torch.zeros(1, dtype=i32, device=dev))
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

    def step(i: int) -> None:
        bt = dbatch[i % 2]
        n = bt["n"]
        main_stream = torch.cuda.current_stream()   # the recording stream while a graph is being captured
        B.np_dedup(bt["keys"], cfg.key_bits, out=dd, ws=ws_d)
        ev_dedup.record(main_stream)
        side_stream.wait_event(ev_dedup)
        with torch.cuda.stream(side_stream):
            B.np_route(dd["unique"], dd["num_unique"], cap, S, cfg.shard_fn, out=rr, ws=ws_r)
            ev_route.record(side_stream)
        # the table is local, so the forward reads it through the requester-side list (unique keys, inverse map);
        # gradients are produced in send order and applied with the send-ordered keys
        fwd_call(table, dd["unique"], dd["inverse"], bt["off"], n, cfg.mode, max_len, out_dtype,
                 num_list=dd["num_unique"], cap=cap, out=out)
        main_stream.wait_event(ev_route)
        B.np_lookup_bwd(bt["dY"], D, cfg.mode, max_len, bt["off"], n, dd["occ_offsets"], dd["occ"], dd["num_unique"], cap,
                        unique_to_send=rr["unique_to_send"], grads=grads, ws=ws_b)
        adagrad_call(table, state, rr["send_keys"], grads, dd["num_unique"], cap, cfg.lr, cfg.eps)

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
    lookups = sum(dbatch[(args.warmup + i) % 2]["n"] for i in range(args.steps))
    value = lookups / (t1 - t0)

    # ---- the variant with backward and update fused (np_lookup_bwd_adagrad): not the headline, reported beside it
    def step_fused(i: int) -> None:
        bt = dbatch[i % 2]
        n = bt["n"]
        B.np_dedup(bt["keys"], cfg.key_bits, out=dd, ws=ws_d)
        B.np_route(dd["unique"], dd["num_unique"], cap, S, cfg.shard_fn, out=rr, ws=ws_r)
        fwd_call(table, dd["unique"], dd["inverse"], bt["off"], n, cfg.mode, max_len, out_dtype,
                 num_list=dd["num_unique"], cap=cap, out=out)
        (B.np_lookup_bwd_adagrad_t if bf16_table else B.np_lookup_bwd_adagrad)(
            bt["dY"], cfg.mode, max_len, bt["off"], n, dd["occ_offsets"], dd["occ"], dd["unique"], dd["num_unique"], cap, table,
            state, cfg.lr, cfg.eps, ws=ws_b)

    fused = None
    if D <= 256:
        step_fused(0)
        B.np_prof_enable(True)
        torch.cuda.synchronize()
        tf0 = time.perf_counter()
        for i in range(args.steps):
            step_fused(args.warmup + i)
        torch.cuda.synchronize()
        fused_ms = (time.perf_counter() - tf0) * 1e3 / args.steps
        frec = B.np_prof_collect(65536)
        B.np_prof_enable(False)
        fk = {}
        for name, ms in frec:
            fk[name] = fk.get(name, 0.0) + ms / args.steps
        fused = {"ms_per_step": fused_ms, "lookups_per_s": n_steps_lookups(dbatch, args) / (fused_ms * 1e-3 * args.steps),
                 "bwd_update_ms": sum(v for k, v in fk.items() if k.startswith("bwd")),
                 "kernels_ms": {k: v for k, v in fk.items() if k.startswith("bwd")}}

    # ---- a worker that reads its own table by key needs no inverse map: np_dedup without it, forward over the raw
    # keys (idx = NULL); reported beside the headline, whose forward goes through (unique, inverse)
    def step_local(i: int) -> None:
        bt = dbatch[i % 2]
        n = bt["n"]
        main_stream = torch.cuda.current_stream()
        B.np_dedup(bt["keys"], cfg.key_bits, out=dd, ws=ws_d, want_inverse=False)
        ev_dedup.record(main_stream)
        side_stream.wait_event(ev_dedup)
        with torch.cuda.stream(side_stream):
            B.np_route(dd["unique"], dd["num_unique"], cap, S, cfg.shard_fn, out=rr, ws=ws_r)
            ev_route.record(side_stream)
        fwd_call(table, bt["keys"], None, bt["off"], n, cfg.mode, max_len, out_dtype, out=out)
        main_stream.wait_event(ev_route)
        B.np_lookup_bwd(bt["dY"], D, cfg.mode, max_len, bt["off"], n, dd["occ_offsets"], dd["occ"], dd["num_unique"], cap,
                        unique_to_send=rr["unique_to_send"], grads=grads, ws=ws_b)
        adagrad_call(table, state, rr["send_keys"], grads, dd["num_unique"], cap, cfg.lr, cfg.eps)

    for i in range(2):
        step_local(args.warmup + i)
    torch.cuda.synchronize()
    tl = time.perf_counter()
    for i in range(args.steps):
        step_local(args.warmup + i)
    torch.cuda.synchronize()
    local_ms = (time.perf_counter() - tl) * 1e3 / args.steps

    # ---- both sides of the sharded flow on the one GPU (what every GPU does around the three All2Alls): the owner
    # gathers the rows of the routed keys into the send buffer, the requester pools straight from that buffer through
    # lookup_to_send; backward and update as in the headline.  fp32 tables only.
    sharded_ms = None
    if not bf16_table:
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

        for i in range(2):
            step_sharded(args.warmup + i)
        torch.cuda.synchronize()
        ts = time.perf_counter()
        for i in range(args.steps):
            step_sharded(args.warmup + i)
        torch.cuda.synchronize()
        sharded_ms = (time.perf_counter() - ts) * 1e3 / args.steps
        del l2s, rows_buf

    # ---- the backward in two parts: its index work (np_lookup_bwd_prepare) behind np_route on the second stream, beside
    # the forward; the reduction (np_lookup_bwd_prepared) where np_lookup_bwd was.  Same bits; reported beside the headline.
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
            B.np_lookup_bwd_prepare(dy_dtype_code, D, cfg.mode, max_len, bt["off"], n, dd["occ_offsets"], dd["num_unique"], ws_b)
            ev_route.record(side_stream)
        fwd_call(table, dd["unique"], dd["inverse"], bt["off"], n, cfg.mode, max_len, out_dtype,
                 num_list=dd["num_unique"], cap=cap, out=out)
        main_stream.wait_event(ev_route)
        B.np_lookup_bwd_prepared(bt["dY"], D, cfg.mode, max_len, bt["off"], n, dd["occ_offsets"], dd["occ"], dd["num_unique"], cap,
                                 ws_b, unique_to_send=rr["unique_to_send"], grads=grads)
        adagrad_call(table, state, rr["send_keys"], grads, dd["num_unique"], cap, cfg.lr, cfg.eps)

    for i in range(2):
        step_split(args.warmup + i)
    torch.cuda.synchronize()
    tsp = time.perf_counter()
    for i in range(args.steps):
        step_split(args.warmup + i)
    torch.cuda.synchronize()
    split_ms = (time.perf_counter() - tsp) * 1e3 / args.steps

    # ---- the same K steps without event recording (what the events cost)
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    ms_per_step_noevents = (time.perf_counter() - t2) * 1e3 / args.steps

    # ---- and once more with one event pair per step: the spread over the steps (the two batches differ a little)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    marks[0].record()
    for i in range(args.steps):
        step(args.warmup + i)
        marks[i + 1].record()
    torch.cuda.synchronize()
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    step_spread = {"min_ms": per_step[0], "median_ms": per_step[len(per_step) // 2], "max_ms": per_step[-1]}

    # ---- the same step recorded into one HIP graph per batch and replayed (the library only enqueues kernels, so a
    # caller can do this; the launch-bound small workloads gain, configuration 5 does not)
    graphs = []
    for b in range(2):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            step(b)
        graphs.append(g)
    for i in range(2):
        graphs[(args.warmup + i) % 2].replay()
    torch.cuda.synchronize()
    t3 = time.perf_counter()
    for i in range(args.steps):
        graphs[(args.warmup + i) % 2].replay()
    torch.cuda.synchronize()
    graph_ms = (time.perf_counter() - t3) * 1e3 / args.steps

    kern = {}
    for name, ms in records:
        k = kern.setdefault(name, [0, 0.0])
        k[0] += 1
        k[1] += ms
    kernels = {k: {"launches_per_step": v[0] / args.steps, "ms_per_step": v[1] / args.steps, "avg_ms": v[1] / v[0]}
               for k, v in kern.items()}
    call_ms = {}
    for k, v in kernels.items():
        call = ("np_dedup" if k.startswith("dedup") else "np_route" if k.startswith("route") else
                "np_lookup_fwd" if k.startswith("fwd") else "np_lookup_bwd" if k.startswith("bwd") else "np_sparse_adagrad")
        call_ms[call] = call_ms.get(call, 0.0) + v["ms_per_step"]

    n_avg = float(np.mean([s["n"] for s in stats]))
    U_avg = float(np.mean([s["U"] for s in stats]))
    alg = algorithmic_bytes(int(n_avg), int(U_avg), cfg.num_bags, D, S, cfg.mode, max_len, 2 if bf16_table else 4)
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

    # ---- dual-buffer synchronisation of the two batches (Section IV-B), timed on its own: key-set intersection
    # plus the copy of the common rows from an active to a prefetch row buffer
    B.np_dedup(dbatch[0]["keys"], cfg.key_bits, out=dd, ws=ws_d)
    ua, na_ = dd["unique"][:cap].clone(), dd["num_unique"].clone()
    B.np_dedup(dbatch[1]["keys"], cfg.key_bits, out=dd, ws=ws_d)
    ub, nb_ = dd["unique"][:cap], dd["num_unique"]
    active = torch.empty((cap, D), dtype=torch.float32, device=dev)
    prefetch = torch.empty((cap, D), dtype=torch.float32, device=dev)
    isec = B.np_intersect(ua, na_, cap, ub, nb_, cap)
    B.np_sync_rows(active, isec["idx_a"], prefetch, isec["idx_b"], isec["num_common"], cap)
    torch.cuda.synchronize()
    B.np_prof_enable(True)
    reps = 5
    for _ in range(reps):
        B.np_intersect(ua, na_, cap, ub, nb_, cap, out=isec)
        B.np_sync_rows(active, isec["idx_a"], prefetch, isec["idx_b"], isec["num_common"], cap)
    torch.cuda.synchronize()
    sync_rec = B.np_prof_collect(1024)
    B.np_prof_enable(False)
    common = int(isec["num_common"].item())
    sync_k = {}
    for name, ms in sync_rec:
        sync_k[name] = sync_k.get(name, 0.0) + ms / reps
    dbsync = {"common_keys": common, "ms": sum(sync_k.values()), "kernels_ms": sync_k,
              "row_copy_GBps": 2 * common * 4 * D / (sync_k.get("sync_rows", 1e9) * 1e-3) / 1e9}
    del active, prefetch, ua

    fwp = None
    if args.fwp_report:
        # frozen-window micro-batching (Section V): keys are deduplicated inside each micro-batch only, so the
        # vectors crossing the All2All inflate from U to sum(U_i)
        fwp = {}
        keys0, off0 = dbatch[0]["keys"], batches[0].bag_offsets
        for N in (1, 2, 4, 8, 16, 32):
            tot, ms = 0, 0.0
            for i in range(N):
                s0, s1 = cfg.batch * i // N, cfg.batch * (i + 1) // N
                sl = [keys0[int(off0[f * cfg.batch + s0]):int(off0[f * cfg.batch + s1])] for f in range(cfg.features)]
                mk = torch.cat(sl).contiguous()
                if mk.numel() == 0:
                    continue
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                B.np_dedup(mk, cfg.key_bits, out=dd, ws=ws_d)
                e1.record()
                torch.cuda.synchronize()
                tot += int(dd["num_unique"].item())
                ms += e0.elapsed_time(e1)
            fwp[str(N)] = {"sum_unique": tot, "inflation": tot / stats[0]["U"], "dedup_ms_total": ms}

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(cfg, b0, wl, args.cpu_sample_div, args.table_dtype)

    line = {
        "metric": "embedding lookups/sec (fwd+bwd+update) and achieved HBM GB/s on 1 MI355X",
        "value": value,
        "unit": "lookups/s",
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
                     "traffic": None if bf16_table else MEASURED_TRAFFIC.get((cfg.name, dominant)),
                     "algorithmic_bytes_per_launch": alg[dom_call], "avg_launch_ms": dom_avg_ms,
                     "launches_timed": timed[dominant][0]},
        "cpu_baseline": cpu,
        "fwd_bwd_update": {"ms_per_step": fbu_ms, "lookups_per_s": n_avg / (fbu_ms * 1e-3) if fbu_ms > 0 else None,
                           "algorithmic_GBps": fbu_bytes / (fbu_ms * 1e-3) / 1e9 if fbu_ms > 0 else None,
                           "frac_of_peak": fbu_bytes / (fbu_ms * 1e-3) / 1e9 / HBM_PEAK_GBS if fbu_ms > 0 else None},
        "calls": {c: {"ms_per_step": call_ms.get(c, 0.0), "algorithmic_bytes": alg[c],
                      "algorithmic_GBps": alg[c] / (call_ms[c] * 1e-3) / 1e9 if call_ms.get(c, 0.0) > 0 else None}
                  for c in alg},
        "kernels": kernels,
        "streams": "np_route runs on a second stream beside np_lookup_fwd; its event times include that sharing",
        "prepared_bwd_step": {"ms_per_step": split_ms, "lookups_per_s": n_steps_lookups(dbatch, args) / (split_ms * 1e-3 * args.steps),
                              "what": "np_lookup_bwd_prepare behind np_route on the second stream, np_lookup_bwd_prepared after the forward"},
        "local_table_step": {"ms_per_step": local_ms, "lookups_per_s": n_steps_lookups(dbatch, args) / (local_ms * 1e-3 * args.steps),
                             "what": "np_dedup without the inverse map, forward over the raw keys; no events"},
        "sharded_flow_step": None if sharded_ms is None else {
            "ms_per_step": sharded_ms, "lookups_per_s": n_steps_lookups(dbatch, args) / (sharded_ms * 1e-3 * args.steps),
            "what": "owner-side row gather into the send buffer + requester-side pooling from it through lookup_to_send "
                    "(np_route with the composed map); backward and update as in the headline; no events"},
        "fused_bwd_update_step": fused,
        "dual_buffer_sync": dbsync,
        "frozen_window_dedup": fwp,
        "ms_per_step_without_events": ms_per_step_noevents,
        "step_time_spread": step_spread,
        "ms_per_step_with_events_on_every_launch": ms_per_step_all_events,
        "hip_graph_replay": {"ms_per_step": graph_ms, "lookups_per_s": n_steps_lookups(dbatch, args) / (graph_ms * 1e-3 * args.steps)},
        "stream_copy_GBps": copy_gbs,
        "input_generation_s": gen_s,
    }
    print(json.dumps(line))
    return 0


def n_steps_lookups(dbatch, args) -> int:
    return sum(dbatch[(args.warmup + i) % 2]["n"] for i in range(args.steps))


def cpu_baseline(cfg, batch, wl, div: int, table_dtype: str = "f32"):
    """The CPU oracle, as it stands, on the first 1/div of the batch's bags: the five steps on a table that holds
    only the rows the sample touches (keys renumbered in order, which changes no result of the path)."""
    from oracle import np_oracle as O
    O.build()
    nb = max(1, cfg.num_bags // div)
    off = batch.bag_offsets[:nb + 1].astype(np.int32)
    n = int(off[-1])
    keys = batch.keys[:n]
    touched = np.unique(keys)
    local = np.searchsorted(touched, keys).astype(np.int64)
    table = wl.table_init_rows(touched, cfg.dim, cfg.table_seed)
    if table_dtype == "bf16":
        import torch
        table = torch.from_numpy(table).bfloat16().view(torch.int16).numpy().view(np.uint16).copy()
    elif table_dtype == "f16":
        table = table.astype(np.float16)
    state = np.zeros(touched.shape[0], np.float32)
    rng = np.random.default_rng(1)
    seq = cfg.mode == wl.SEQ
    if seq:
        dY = (rng.standard_normal((nb, batch.max_len, cfg.dim)).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
    else:
        dY = rng.standard_normal((nb, cfg.dim)).astype(np.float32)
    t0 = time.perf_counter()
    unique, inverse, counts, occ_offsets, occ = O.dedup(local)
    t1 = time.perf_counter()
    send_keys, splits, send_offsets, sfu, uts = O.route(touched[unique], cfg.num_shards, cfg.shard_fn)
    l2s = O.compose(inverse, uts)
    t2 = time.perf_counter()
    O.lookup_fwd(table, unique[sfu], l2s, off, cfg.mode, batch.max_len, O.BF16 if seq else O.F32)
    t3 = time.perf_counter()
    grads, _ = O.lookup_bwd(dY, O.BF16 if seq else O.F32, cfg.dim, cfg.mode, batch.max_len, off, inverse, unique.shape[0], uts)
    t4 = time.perf_counter()
    if table_dtype == "bf16":
        O.sparse_adagrad_bf16(table, state, unique[sfu], grads, cfg.lr, cfg.eps)
    elif table_dtype == "f16":
        O.sparse_adagrad_f16(table.view(np.uint16), state, unique[sfu], grads, cfg.lr, cfg.eps)
    else:
        O.sparse_adagrad(table, state, unique[sfu], grads, cfg.lr, cfg.eps)
    t5 = time.perf_counter()
    total = t5 - t0
    return {"value": n / total, "unit": "lookups/s", "cores": 1, "kind": "oracle",
            "sample": f"first {nb} of {cfg.num_bags} bags of batch 0 ({n} lookups, {touched.shape[0]} distinct keys), all five "
                      f"steps, table holding only the touched rows; single-threaded C, fp64 accumulation",
            "seconds": total,
            "seconds_per_call": {"dedup": t1 - t0, "route": t2 - t1, "fwd": t3 - t2, "bwd": t4 - t3, "adagrad": t5 - t4}}


if __name__ == "__main__":
    sys.exit(main())
