"""GPU parity of the dual-buffer synchronisation (Section IV-B): np_intersect and np_sync_rows against the
oracle, bit for bit, and the pipelined run of two overlapping batches (prefetch before the update, update on
the active buffer, synchronise the intersection, forward from the prefetch buffer) against the sequential run
on the table (Proposition 1)."""
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


def _gpu_intersect(H, a, b, pad=37):
    import torch
    abuf = np.zeros(a.size + pad, np.int64)
    abuf[:a.size] = a
    bbuf = np.zeros(b.size + pad, np.int64)
    bbuf[:b.size] = b
    r = H.B.np_intersect(H.dev(abuf), H.dev(np.array([a.size], np.int32)), abuf.size, H.dev(bbuf),
                         H.dev(np.array([b.size], np.int32)), bbuf.size)
    torch.cuda.synchronize()
    c = int(r["num_common"].item())
    return H.host(r["idx_a"])[:c], H.host(r["idx_b"])[:c], r


@pytest.mark.parametrize("na,nb,hi", [(1, 1, 2), (1000, 800, 3000), (5000, 1, 100), (1, 5000, 100), (300000, 250000, 10 ** 6),
                                      (2050, 2047, 2 ** 40), (700000, 700000, 2 ** 33)])
def test_intersect_bit_exact(H, na, nb, hi):
    rng = np.random.default_rng(na + nb)
    a = np.unique(rng.integers(0, hi, size=na)).astype(np.int64)
    b = np.unique(rng.integers(0, hi, size=nb)).astype(np.int64)
    ia, ib, _ = _gpu_intersect(H, a, b)
    ra, rb = H.O.intersect(a, b)
    assert np.array_equal(ia, ra) and np.array_equal(ib, rb)


def test_intersect_uneven_densities(H):
    """Slices of A far longer than the staged window (dense A, sparse B), and far shorter (the reverse); B spanning
    several tiles and more than one batch of tiles per chunk."""
    rng = np.random.default_rng(5)
    dense = np.arange(0, 3_000_000, dtype=np.int64)
    sparse = np.unique(rng.integers(0, 3_000_000, size=9000)).astype(np.int64)
    for a, b in ((dense, sparse), (sparse, dense), (dense[::3], dense[::5]),
                 (np.concatenate([dense[:5000], dense[2_900_000:]]), sparse)):
        ia, ib, _ = _gpu_intersect(H, a, b)
        ra, rb = H.O.intersect(a, b)
        assert np.array_equal(ia, ra) and np.array_equal(ib, rb)


def test_intersect_degenerate(H):
    a = np.arange(0, 5000, 2, dtype=np.int64)
    ia, ib, _ = _gpu_intersect(H, a, a)
    assert np.array_equal(ia, np.arange(a.size)) and np.array_equal(ib, np.arange(a.size))
    ia, ib, _ = _gpu_intersect(H, a, a + 1)
    assert ia.size == 0
    ia, ib, _ = _gpu_intersect(H, a, np.empty(0, np.int64))
    assert ia.size == 0
    ia, ib, _ = _gpu_intersect(H, np.empty(0, np.int64), a)
    assert ia.size == 0


@pytest.mark.parametrize("dim", [4, 16, 64, 128, 512])
def test_sync_rows_bit_copy(H, dim):
    import torch
    rng = np.random.default_rng(dim)
    src = rng.standard_normal((3000, dim)).astype(np.float32)
    dst0 = rng.standard_normal((4000, dim)).astype(np.float32)
    m = 1700
    si = rng.choice(3000, size=m, replace=False).astype(np.int32)
    di = rng.choice(4000, size=m, replace=False).astype(np.int32)
    ref = dst0.copy()
    H.O.sync_rows(src, si, ref, di)
    d = H.dev(dst0)
    pad = np.zeros(64, np.int32)
    H.B.np_sync_rows(H.dev(src), H.dev(np.concatenate([si, pad])), d, H.dev(np.concatenate([di, pad])),
                     H.dev(np.array([m], np.int32)), m + 64)
    torch.cuda.synchronize()
    assert H.host(d).tobytes() == ref.tobytes()


def _pipeline_check(H, cfg):
    """Two consecutive batches: sequential on the table vs dual-buffer pipeline on compact row buffers."""
    import torch
    B, O, wl = H.B, H.O, H.wl
    R, D = cfg.num_rows, cfg.dim
    b1 = wl.make_batch(cfg, 0)
    b2 = wl.make_batch(cfg, 1, prev=b1)
    table = torch.empty((R, D), dtype=torch.float32, device="cuda")
    B.np_util_table_init(table, cfg.table_seed)
    state = torch.zeros(R, dtype=torch.float32, device="cuda")
    k1, off1, dY1 = H.dev(b1.keys), H.dev(b1.bag_offsets), H.dev(b1.dY)
    k2, off2 = H.dev(b2.keys), H.dev(b2.bag_offsets)
    d1 = B.np_dedup(k1, cfg.key_bits)
    d2 = B.np_dedup(k2, cfg.key_bits)
    torch.cuda.synchronize()
    U1, U2 = int(d1["num_unique"].item()), int(d2["num_unique"].item())
    empty_off = H.dev(np.array([0], np.int32))
    # both buffers are filled from the table as it is BEFORE batch 1 updates it
    _, active = B.np_lookup_fwd(table, d1["unique"], None, empty_off, 0, 0, num_list=d1["num_unique"], cap=U1, want_rows=True,
                                out=torch.empty((0, D), dtype=torch.float32, device="cuda"))
    _, prefetch = B.np_lookup_fwd(table, d2["unique"], None, empty_off, 0, 0, num_list=d2["num_unique"], cap=U2, want_rows=True,
                                  out=torch.empty((0, D), dtype=torch.float32, device="cuda"))
    stale = prefetch.clone()
    iota1 = torch.arange(U1, dtype=torch.int64, device="cuda")
    iota2 = torch.arange(U2, dtype=torch.int64, device="cuda")
    astate = torch.zeros(U1, dtype=torch.float32, device="cuda")
    # batch 1: gradients once, applied to the active buffer (pipeline) and to the table (sequential reference)
    g1 = B.np_lookup_bwd(dY1, D, cfg.mode, 1, off1, b1.n, d1["occ_offsets"], d1["occ"], d1["num_unique"], U1)
    B.np_sparse_adagrad(active, astate, iota1, g1, d1["num_unique"], U1, cfg.lr, cfg.eps)
    B.np_sparse_adagrad(table, state, d1["unique"], g1, d1["num_unique"], U1, cfg.lr, cfg.eps)
    seq, _ = B.np_lookup_fwd(table, d2["unique"], d2["inverse"], off2, b2.n, cfg.mode)
    # synchronise the intersection, then batch 2 reads the prefetch buffer
    isec = B.np_intersect(d1["unique"], d1["num_unique"], U1, d2["unique"], d2["num_unique"], U2)
    B.np_sync_rows(active, isec["idx_a"], prefetch, isec["idx_b"], isec["num_common"], min(U1, U2))
    dbp, _ = B.np_lookup_fwd(prefetch, iota2, d2["inverse"], off2, b2.n, cfg.mode)
    old, _ = B.np_lookup_fwd(stale, iota2, d2["inverse"], off2, b2.n, cfg.mode)
    torch.cuda.synchronize()
    C = int(isec["num_common"].item())
    ra, rb = O.intersect(H.host(d1["unique"])[:U1], H.host(d2["unique"])[:U2])
    assert C == ra.size > 0
    assert np.array_equal(H.host(isec["idx_a"])[:C], ra) and np.array_equal(H.host(isec["idx_b"])[:C], rb)
    assert torch.equal(dbp, seq)                       # Proposition 1: exactly W_{t+1}
    assert not torch.equal(old, seq)                   # without the synchronisation the read is stale
    # rows of the prefetch buffer outside the intersection kept their bits
    keep = np.ones(U2, bool)
    keep[rb] = False
    assert H.host(prefetch)[keep].tobytes() == H.host(stale)[keep].tobytes()
    return C, U1, U2


def test_pipeline_tiny_config(H):
    _pipeline_check(H, H.wl.config("tiny"))


def test_pipeline_scaled_large_config_with_30pct_overlap(H):
    C, U1, U2 = _pipeline_check(H, H.wl.scaled(H.wl.config("large"), 2000, 64))
    assert abs(C / U2 - 0.30) < 0.01


def _two_stream_pipeline(H, cfg):
    """The inter-batch pipeline with the prefetch of B_t on a second stream, issued BEFORE B_{t-1}'s update (Section IV-B,
    Proposition 1).  `master` stands for the copy of the table that prefetches read (the DRAM tier of the paper): it still
    holds W_t while B_{t-1}'s update runs on the active buffer, so the prefetched rows of the common keys are stale until
    the synchronisation overwrites them.  The sequential reference runs on a clone of the table, one stream, update first."""
    import torch
    B, wl = H.B, H.wl
    R, D = cfg.num_rows, cfg.dim
    b1 = wl.make_batch(cfg, 0)
    b2 = wl.make_batch(cfg, 1, prev=b1)
    master = torch.empty((R, D), dtype=torch.float32, device="cuda")
    B.np_util_table_init(master, cfg.table_seed)
    table_seq = master.clone()
    state_seq = torch.zeros(R, dtype=torch.float32, device="cuda")
    k1, off1, dY1 = H.dev(b1.keys), H.dev(b1.bag_offsets), H.dev(b1.dY)
    k2, off2 = H.dev(b2.keys), H.dev(b2.bag_offsets)
    d1 = B.np_dedup(k1, cfg.key_bits)
    d2 = B.np_dedup(k2, cfg.key_bits)
    torch.cuda.synchronize()
    U1, U2 = int(d1["num_unique"].item()), int(d2["num_unique"].item())
    empty_off = H.dev(np.array([0], np.int32))
    none_out = torch.empty((0, D), dtype=torch.float32, device="cuda")
    iota1 = torch.arange(U1, dtype=torch.int64, device="cuda")
    iota2 = torch.arange(U2, dtype=torch.int64, device="cuda")
    # everything the streams touch exists before the first enqueue (no allocation between the event-ordered calls)
    active = torch.empty((U1, D), dtype=torch.float32, device="cuda")
    prefetch = torch.empty((U2, D), dtype=torch.float32, device="cuda")
    astate = torch.zeros(U1, dtype=torch.float32, device="cuda")
    g1 = torch.empty((U1, D), dtype=torch.float32, device="cuda")
    ws_b = torch.empty(max(B.np_lookup_bwd_workspace_bytes(cfg.num_bags, b1.n, D, cfg.mode), 256), dtype=torch.uint8, device="cuda")
    isec = dict(idx_a=torch.empty(min(U1, U2), dtype=torch.int32, device="cuda"), idx_b=torch.empty(min(U1, U2), dtype=torch.int32, device="cuda"),
                num_common=torch.zeros(1, dtype=torch.int32, device="cuda"))
    ws_i = torch.empty(max(int(B.lib.np_intersect_workspace_bytes(U2)), 256), dtype=torch.uint8, device="cuda")
    out_dbp = torch.empty((cfg.num_bags, D), dtype=torch.float32, device="cuda")
    main = torch.cuda.current_stream()
    side = torch.cuda.Stream()                       # default priority
    ev_ready, ev_prefetched = torch.cuda.Event(), torch.cuda.Event()
    # B_{t-1}'s rows are in the active buffer (its own prefetch, long done)
    B.np_lookup_fwd(master, d1["unique"], None, empty_off, 0, 0, num_list=d1["num_unique"], cap=U1, out=none_out, rows_out=active)
    ev_ready.record(main)
    # ---- second stream: B_t's prefetch, enqueued before B_{t-1}'s backward and update
    side.wait_event(ev_ready)
    with torch.cuda.stream(side):
        B.np_lookup_fwd(master, d2["unique"], None, empty_off, 0, 0, num_list=d2["num_unique"], cap=U2, out=none_out, rows_out=prefetch)
        ev_prefetched.record(side)
    # ---- main stream: B_{t-1}'s backward and update on the active buffer, beside the prefetch
    B.np_lookup_bwd(dY1, D, cfg.mode, 1, off1, b1.n, d1["occ_offsets"], d1["occ"], d1["num_unique"], U1, grads=g1, ws=ws_b)
    B.np_sparse_adagrad(active, astate, iota1, g1, d1["num_unique"], U1, cfg.lr, cfg.eps)
    B.np_intersect(d1["unique"], d1["num_unique"], U1, d2["unique"], d2["num_unique"], U2, out=isec, ws=ws_i)
    main.wait_event(ev_prefetched)                   # the synchronisation needs both the update and the prefetch
    B.np_sync_rows(active, isec["idx_a"], prefetch, isec["idx_b"], isec["num_common"], min(U1, U2))
    B.np_lookup_fwd(prefetch, iota2, d2["inverse"], off2, b2.n, cfg.mode, out=out_dbp)
    torch.cuda.synchronize()
    # ---- sequential reference: update the table, then read it
    B.np_sparse_adagrad(table_seq, state_seq, d1["unique"], g1, d1["num_unique"], U1, cfg.lr, cfg.eps)
    seq, _ = B.np_lookup_fwd(table_seq, d2["unique"], d2["inverse"], off2, b2.n, cfg.mode)
    # what the prefetch alone would have given (rows of W_t): must differ, or the test shows nothing
    _, stale = B.np_lookup_fwd(master, d2["unique"], None, empty_off, 0, 0, num_list=d2["num_unique"], cap=U2, want_rows=True, out=none_out)
    old, _ = B.np_lookup_fwd(stale, iota2, d2["inverse"], off2, b2.n, cfg.mode)
    torch.cuda.synchronize()
    assert int(isec["num_common"].item()) > 0
    assert torch.equal(out_dbp, seq)
    assert not torch.equal(old, seq)
    # the oracle's sequential result for the same two batches.  The rows batch 2 reads: the oracle's update of W_t with the
    # same gradient rows, held to the update's own tolerance (measured against |w| + |step|: a pooled sum of updated rows
    # can cancel to nothing, so the sum's own magnitude is no yardstick for the update's rounding); the pooled sums: the
    # oracle's forward over exactly the rows the prefetch buffer holds, to the forward's tolerance.
    u1, u2 = H.host(d1["unique"])[:U1], H.host(d2["unique"])[:U2]
    tref = wl.table_init_rows(np.arange(R), D, cfg.table_seed)
    before = tref.copy()
    sref = np.zeros(R, np.float32)
    H.O.sparse_adagrad(tref, sref, u1, H.host(g1)[:U1], cfg.lr, cfg.eps)
    rows = H.host(prefetch)[:U2]
    step = np.abs(tref[u2].astype(np.float64) - before[u2])
    H.assert_close(rows, tref[u2], np.abs(before[u2]) + step, H.RTOL_F32, "rows of the synchronised prefetch buffer")
    fresh = np.setdiff1d(u2, u1)
    assert rows[np.searchsorted(u2, fresh)].tobytes() == before[fresh].tobytes()     # keys outside K(B_{t-1}): W_t bit for bit
    ref, _, ab = H.O.lookup_fwd(rows, np.arange(U2), H.host(d2["inverse"])[:b2.n], b2.bag_offsets, cfg.mode, want_abs=True)
    H.assert_close(H.host(out_dbp), ref, ab, H.RTOL_F32, "forward from the synchronised prefetch buffer")


def test_two_stream_pipeline_tiny_config(H):
    _two_stream_pipeline(H, H.wl.config("tiny"))


def test_two_stream_pipeline_scaled_large_config(H):
    _two_stream_pipeline(H, H.wl.scaled(H.wl.config("large"), 2000, 64))
