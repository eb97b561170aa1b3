"""The five-call step recorded once into a HIP graph and replayed: the library enqueues kernels only (no allocation,
no host synchronisation, no memset nodes; the distinct-key count stays in device memory), so a caller can capture a
whole step and replay it on new batches of the same shape.  Every replay is compared bit for bit with the eager
calls on the same inputs, with unrelated eager work and synchronisations between the replays."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    import gpu_helpers
    return gpu_helpers


def _buffers(H, cfg, n, cap, max_len):
    import torch
    B = H.B
    D, S = cfg.dim, cfg.num_shards
    i32, i64, dev = torch.int32, torch.int64, "cuda"
    dd = dict(unique=torch.empty(n, dtype=i64, device=dev), inverse=torch.empty(n, dtype=i32, device=dev),
              counts=torch.empty(n, dtype=i32, device=dev), occ_offsets=torch.empty(n + 1, dtype=i32, device=dev),
              occ=torch.empty(n, dtype=i32, device=dev), num_unique=torch.zeros(1, dtype=i32, device=dev))
    rr = dict(send_keys=torch.empty(cap, dtype=i64, device=dev), splits=torch.empty(S, dtype=i32, device=dev),
              send_offsets=torch.empty(S + 1, dtype=i32, device=dev), send_from_unique=torch.empty(cap, dtype=i32, device=dev),
              unique_to_send=torch.empty(cap, dtype=i32, device=dev), lookup_to_send=torch.empty(n, dtype=i32, device=dev))
    ws = dict(d=torch.empty(max(B.np_dedup_workspace_bytes(n, cfg.key_bits), 256), dtype=torch.uint8, device=dev),
              r=torch.empty(max(B.np_route_workspace_bytes(cap, S), 256), dtype=torch.uint8, device=dev),
              b=torch.empty(max(B.np_lookup_bwd_workspace_bytes(cfg.num_bags, n, D, cfg.mode), 256), dtype=torch.uint8, device=dev))
    out = torch.empty((cfg.num_bags, D), dtype=torch.float32, device=dev)
    grads = torch.zeros((cap, D), dtype=torch.float32, device=dev)
    return dd, rr, ws, out, grads


def _step(H, cfg, keys, off, dY, n, cap, max_len, table, state, bufs):
    B = H.B
    dd, rr, ws, out, grads = bufs
    B.np_dedup(keys, cfg.key_bits, out=dd, ws=ws["d"])
    B.np_route(dd["unique"], dd["num_unique"], cap, cfg.num_shards, cfg.shard_fn, inverse=dd["inverse"], n=n, out=rr, ws=ws["r"])
    B.np_lookup_fwd(table, rr["send_keys"], rr["lookup_to_send"], off, n, cfg.mode, max_len, B.F32, num_list=dd["num_unique"],
                    cap=cap, out=out)
    B.np_lookup_bwd(dY, cfg.dim, cfg.mode, max_len, off, n, dd["occ_offsets"], dd["occ"], dd["num_unique"], cap,
                    unique_to_send=rr["unique_to_send"], grads=grads, ws=ws["b"])
    B.np_sparse_adagrad(table, state, rr["send_keys"], grads, dd["num_unique"], cap, cfg.lr, cfg.eps)


def _snapshot(H, bufs, table, state):
    dd, rr, _, out, grads = bufs
    U = int(dd["num_unique"].item())
    return dict(U=U, unique=H.host(dd["unique"])[:U].copy(), inverse=H.host(dd["inverse"]).copy(),
                send_keys=H.host(rr["send_keys"])[:U].copy(), splits=H.host(rr["splits"]).copy(), out=H.host(out).copy(),
                grads=H.host(grads)[:U].copy(), table=H.host(table).copy(), state=H.host(state).copy())


@pytest.mark.parametrize("name,row_div,batch_div", [("skew", 128, 16), ("tiny", 1, 1)])
def test_captured_step_replays_bit_exactly(H, name, row_div, batch_div):
    import torch
    wl, B = H.wl, H.B
    cfg = wl.config(name) if row_div == 1 else wl.scaled(wl.config(name), row_div, batch_div)
    R, D = cfg.num_rows, cfg.dim
    b0 = wl.make_batch(cfg, 0)
    # a second batch of the same shape (same bag offsets, so the same n) with other keys and gradients
    rng = np.random.default_rng(99)
    b1_keys = b0.keys[rng.permutation(b0.n)].copy()
    b1_keys[: b0.n // 3] = rng.integers(0, R, size=b0.n // 3)
    b1_dY = rng.standard_normal(b0.dY.shape).astype(np.float32)
    inputs = [(b0.keys, b0.dY), (b1_keys, b1_dY), (b0.keys, b1_dY)]
    n, cap, max_len = b0.n, b0.n, b0.max_len
    off = H.dev(b0.bag_offsets)

    # ---- eager sequence
    table = torch.empty((R, D), dtype=torch.float32, device="cuda")
    B.np_util_table_init(table, cfg.table_seed)
    state = torch.zeros(R, dtype=torch.float32, device="cuda")
    bufs = _buffers(H, cfg, n, cap, max_len)
    eager = []
    for keys, dY in inputs:
        _step(H, cfg, H.dev(keys), off, H.dev(dY), n, cap, max_len, table, state, bufs)
        torch.cuda.synchronize()
        eager.append(_snapshot(H, bufs, table, state))
    assert eager[0]["U"] != eager[1]["U"]          # the replays really see different distinct-key counts

    # ---- the same sequence as replays of one captured step
    table_g = torch.empty((R, D), dtype=torch.float32, device="cuda")
    B.np_util_table_init(table_g, cfg.table_seed)
    state_g = torch.zeros(R, dtype=torch.float32, device="cuda")
    bufs_g = _buffers(H, cfg, n, cap, max_len)
    keys_s = torch.zeros(n, dtype=torch.int64, device="cuda")
    dY_s = torch.zeros(b0.dY.shape, dtype=torch.float32, device="cuda")
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        _step(H, cfg, keys_s, off, dY_s, n, cap, max_len, table_g, state_g, bufs_g)
    torch.cuda.synchronize()
    # capture runs nothing: the table still holds the initial rows
    assert B.np_util_table_count_changed(table_g, cfg.table_seed) == 0
    scratch = torch.empty(1 << 20, dtype=torch.float32, device="cuda")
    for t, (keys, dY) in enumerate(inputs):
        keys_s.copy_(H.dev(keys))
        dY_s.copy_(H.dev(dY))
        graph.replay()
        torch.cuda.synchronize()
        got = _snapshot(H, bufs_g, table_g, state_g)
        for k, v in eager[t].items():
            if k == "U":
                assert got["U"] == v, (t, got["U"], v)
            else:
                assert got[k].tobytes() == v.tobytes(), f"replay {t}: {k} differs from the eager step"
        # unrelated eager work between replays: the library on other buffers, and a torch kernel
        other = B.np_dedup(H.dev(rng.integers(0, 1000, size=5000).astype(np.int64)), 10)
        scratch.normal_()
        torch.cuda.synchronize()
        assert int(other["num_unique"].item()) <= 1000


def test_two_steps_on_two_streams_do_not_interfere(H):
    """Two independent steps (own tables, buffers and workspaces) enqueued alternately call by call on two streams give
    the bits of the same steps run one after the other: the calls share no hidden state."""
    import torch
    wl, B = H.wl, H.B
    cfgs = [wl.scaled(wl.config("skew"), 128, 16), wl.scaled(wl.config("dlrm"), 64, 16)]
    work = []
    for cfg in cfgs:
        b = wl.make_batch(cfg, 0)
        work.append(dict(cfg=cfg, keys=H.dev(b.keys), off=H.dev(b.bag_offsets), dY=H.dev(b.dY), n=b.n, cap=b.n, max_len=b.max_len))

    def fresh(w):
        cfg = w["cfg"]
        table = torch.empty((cfg.num_rows, cfg.dim), dtype=torch.float32, device="cuda")
        B.np_util_table_init(table, cfg.table_seed)
        state = torch.zeros(cfg.num_rows, dtype=torch.float32, device="cuda")
        return table, state, _buffers(H, cfg, w["n"], w["cap"], w["max_len"])

    # one after the other on the current stream
    ref = []
    for w in work:
        table, state, bufs = fresh(w)
        for _ in range(2):
            _step(H, w["cfg"], w["keys"], w["off"], w["dY"], w["n"], w["cap"], w["max_len"], table, state, bufs)
        torch.cuda.synchronize()
        ref.append(_snapshot(H, bufs, table, state))

    # interleaved call by call on two streams
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    live = [fresh(w) for w in work]
    torch.cuda.synchronize()

    def calls(w, table, state, bufs):
        cfg, n, cap, max_len = w["cfg"], w["n"], w["cap"], w["max_len"]
        dd, rr, ws, out, grads = bufs
        yield lambda: B.np_dedup(w["keys"], cfg.key_bits, out=dd, ws=ws["d"])
        yield lambda: B.np_route(dd["unique"], dd["num_unique"], cap, cfg.num_shards, cfg.shard_fn, inverse=dd["inverse"], n=n, out=rr,
                                 ws=ws["r"])
        yield lambda: B.np_lookup_fwd(table, rr["send_keys"], rr["lookup_to_send"], w["off"], n, cfg.mode, max_len, B.F32,
                                      num_list=dd["num_unique"], cap=cap, out=out)
        yield lambda: B.np_lookup_bwd(w["dY"], cfg.dim, cfg.mode, max_len, w["off"], n, dd["occ_offsets"], dd["occ"], dd["num_unique"],
                                      cap, unique_to_send=rr["unique_to_send"], grads=grads, ws=ws["b"])
        yield lambda: B.np_sparse_adagrad(table, state, rr["send_keys"], grads, dd["num_unique"], cap, cfg.lr, cfg.eps)

    for _ in range(2):
        its = [calls(w, *lv) for w, lv in zip(work, live)]
        for pair in zip(*its):
            for st, call in zip(streams, pair):
                with torch.cuda.stream(st):
                    call()
    torch.cuda.synchronize()
    for w, lv, want in zip(work, live, ref):
        table, state, bufs = lv
        got = _snapshot(H, bufs, table, state)
        for k, v in want.items():
            if k == "U":
                assert got["U"] == v
            else:
                assert got[k].tobytes() == v.tobytes(), f"{w['cfg'].name}: {k} differs when run beside another step"


def test_two_host_threads_issue_steps_concurrently(H):
    """The same two independent steps issued from two host threads at once, each on a stream of its own."""
    import threading

    import torch
    wl, B = H.wl, H.B
    cfgs = [wl.scaled(wl.config("skew"), 128, 16), wl.scaled(wl.config("large"), 2048, 64)]
    work = []
    for cfg in cfgs:
        b = wl.make_batch(cfg, 0)
        work.append(dict(cfg=cfg, keys=H.dev(b.keys), off=H.dev(b.bag_offsets), dY=H.dev(b.dY), n=b.n, cap=b.n, max_len=b.max_len))

    def fresh(w):
        cfg = w["cfg"]
        table = torch.empty((cfg.num_rows, cfg.dim), dtype=torch.float32, device="cuda")
        B.np_util_table_init(table, cfg.table_seed)
        state = torch.zeros(cfg.num_rows, dtype=torch.float32, device="cuda")
        return table, state, _buffers(H, cfg, w["n"], w["cap"], w["max_len"])

    reps = 5
    ref = []
    for w in work:
        table, state, bufs = fresh(w)
        for _ in range(reps):
            _step(H, w["cfg"], w["keys"], w["off"], w["dY"], w["n"], w["cap"], w["max_len"], table, state, bufs)
        torch.cuda.synchronize()
        ref.append(_snapshot(H, bufs, table, state))

    live = [fresh(w) for w in work]
    torch.cuda.synchronize()
    errors = []
    gate = threading.Barrier(2)

    def run(w, lv):
        try:
            torch.cuda.set_device(0)
            st = torch.cuda.Stream()
            gate.wait(timeout=60)
            with torch.cuda.stream(st):
                for _ in range(reps):
                    _step(H, w["cfg"], w["keys"], w["off"], w["dY"], w["n"], w["cap"], w["max_len"], *lv)
            st.synchronize()
        except Exception as e:  # noqa: BLE001  (reported by the main thread)
            errors.append(repr(e))

    threads = [threading.Thread(target=run, args=(w, lv)) for w, lv in zip(work, live)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=120)
    assert not errors, errors
    torch.cuda.synchronize()
    for w, lv, want in zip(work, live, ref):
        table, state, bufs = lv
        got = _snapshot(H, bufs, table, state)
        for k, v in want.items():
            if k == "U":
                assert got["U"] == v
            else:
                assert got[k].tobytes() == v.tobytes(), f"{w['cfg'].name}: {k} differs when issued from a second thread"
