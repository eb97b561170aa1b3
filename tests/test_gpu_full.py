"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration bench.py times
(preallocated buffers, U-sized capacity, two consecutive batches with the update left live).

The tables are 10-205 GB, so the oracle works on a table that holds only the rows a batch touches: the
oracle's key list is the position of each send slot's key in the sorted distinct-key set, which leaves every
result of the path unchanged.  Integer outputs are compared bit for bit and in full; values are compared in
full against the oracle; that no row outside the batch changed is shown by counting, on the device, the rows
of the whole table that differ from the stateless initialiser."""
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


def _full_check(H, name, steps):
    import torch
    wl, O, B = H.wl, H.O, H.B
    cfg = wl.config(name)
    R, D, S = cfg.num_rows, cfg.dim, cfg.num_shards
    seq = cfg.mode == wl.SEQ
    dt = O.BF16 if seq else O.F32
    table = torch.empty((R, D), dtype=torch.float32, device="cuda")
    state = torch.zeros(R, dtype=torch.float32, device="cuda")
    B.np_util_table_init(table, cfg.table_seed)
    assert B.np_util_table_count_changed(table, cfg.table_seed) == 0
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1234 + cfg.index)
    known_keys = np.empty(0, np.int64)     # keys touched so far (sorted) and the rows / states the GPU holds for them
    known_rows = np.empty((0, D), np.float32)
    known_state = np.empty(0, np.float32)
    prev = None
    touched_all = np.empty(0, np.int64)
    for t in range(steps):
        H.progress(f"[{name}] step {t}: generating")
        batch = wl.make_batch(cfg, t, prev=prev, with_dy=False)
        prev = batch
        n, Bn, max_len = batch.n, cfg.num_bags, batch.max_len
        shape = (Bn, max_len, D) if seq else (Bn, D)
        dY = torch.randn(shape, dtype=torch.float32, device="cuda", generator=gen)
        if seq:
            dY = dY.bfloat16()
        keys_d, off_d = H.dev(batch.keys), H.dev(batch.bag_offsets)
        # ---- oracle integer outputs first (they size the device buffers exactly as bench.py does)
        unique, inverse, counts, occ_offsets, occ = O.dedup(batch.keys)
        U = unique.shape[0]
        send_keys, splits, send_offsets, sfu, uts = O.route(unique, S, cfg.shard_fn)
        l2s = O.compose(inverse, uts)
        cap = U + 1024
        H.progress(f"[{name}] step {t}: n={n} U={U} hottest={counts.max()} -> GPU")
        d = B.np_dedup(keys_d, cfg.key_bits)
        i32, i64 = torch.int32, torch.int64
        rr = dict(send_keys=torch.empty(cap, dtype=i64, device="cuda"), splits=torch.empty(S, dtype=i32, device="cuda"),
                  send_offsets=torch.empty(S + 1, dtype=i32, device="cuda"),
                  send_from_unique=torch.empty(cap, dtype=i32, device="cuda"),
                  unique_to_send=torch.empty(cap, dtype=i32, device="cuda"),
                  lookup_to_send=torch.empty(n, dtype=i32, device="cuda"))
        B.np_route(d["unique"], d["num_unique"], cap, S, cfg.shard_fn, inverse=d["inverse"], n=n, out=rr)
        out, _ = B.np_lookup_fwd(table, rr["send_keys"], rr["lookup_to_send"], off_d, n, cfg.mode, max_len,
                                 B.BF16 if seq else B.F32, num_list=d["num_unique"], cap=cap)
        # the forward exactly as bench.py issues it (requester-side list: distinct keys + inverse map): same rows in the
        # same order, so the same bits
        out_b, _ = B.np_lookup_fwd(table, d["unique"], d["inverse"], off_d, n, cfg.mode, max_len, B.BF16 if seq else B.F32,
                                   num_list=d["num_unique"], cap=cap)
        assert torch.equal(out, out_b)
        del out_b
        grads = B.np_lookup_bwd(dY, D, cfg.mode, max_len, off_d, n, d["occ_offsets"], d["occ"], d["num_unique"], cap,
                                unique_to_send=rr["unique_to_send"])
        grads2 = B.np_lookup_bwd(dY, D, cfg.mode, max_len, off_d, n, d["occ_offsets"], d["occ"], d["num_unique"], cap,
                                 unique_to_send=rr["unique_to_send"])
        B.np_sparse_adagrad(table, state, rr["send_keys"], grads, d["num_unique"], cap, cfg.lr, cfg.eps)
        torch.cuda.synchronize()
        g = dict(dedup=d, route=rr)
        ref = dict(unique=unique, inverse=inverse, counts=counts, occ_offsets=occ_offsets, occ=occ, send_keys=send_keys,
                   splits=splits, send_offsets=send_offsets, send_from_unique=sfu, unique_to_send=uts, lookup_to_send=l2s)
        assert H.assert_int_outputs_equal(g, ref, n, S) == U
        assert torch.equal(grads[:U], grads2[:U])                       # deterministic at full size
        del grads2
        # ---- the table as the oracle must see it: initial rows, overwritten by every earlier update
        H.progress(f"[{name}] step {t}: oracle values")
        table_c = wl.table_init_rows(unique, D, cfg.table_seed)
        state_c = np.zeros(U, np.float32)
        if known_keys.size:
            both = np.intersect1d(known_keys, unique, assume_unique=True)
            assert both.size > 0
            table_c[np.searchsorted(unique, both)] = known_rows[np.searchsorted(known_keys, both)]
            state_c[np.searchsorted(unique, both)] = known_state[np.searchsorted(known_keys, both)]
        list_c = sfu.astype(np.int64)                                    # send slot -> row of the compact table
        out_ref, _, ab = O.lookup_fwd(table_c, list_c, l2s, batch.bag_offsets, cfg.mode, max_len, dt, want_abs=not seq)
        if seq:
            assert H.host(out).tobytes() == out_ref.tobytes()
        else:
            H.assert_close(H.host(out), out_ref, ab, H.RTOL_F32, f"{name} step {t} forward")
        del out_ref, ab
        dy_h = H.host(dY)
        g_ref, gab = O.lookup_bwd(dy_h, dt, D, cfg.mode, max_len, batch.bag_offsets, inverse, U, uts, want_abs=True)
        g_gpu = H.host(grads)[:U]
        H.assert_close(g_gpu, g_ref, gab, H.RTOL_F32, f"{name} step {t} gradients")
        del g_ref, gab, dy_h
        before = table_c.copy()
        O.sparse_adagrad(table_c, state_c, list_c, g_gpu, cfg.lr, cfg.eps)
        rows_gpu = H.host(table[H.dev(unique)])
        st_gpu = H.host(state[H.dev(unique)])
        delta = np.abs(table_c.astype(np.float64) - before)
        H.assert_close(rows_gpu, table_c, np.abs(before) + delta, H.RTOL_F32, f"{name} step {t} updated rows")
        H.assert_close(st_gpu, state_c, np.abs(state_c), H.RTOL_F32, f"{name} step {t} state")
        # ---- Eq. (2): nothing outside the batches moved, anywhere in the table
        touched_all = np.union1d(touched_all, unique)
        rows_all = H.host(table[H.dev(touched_all)])
        init_all = wl.table_init_rows(touched_all, D, cfg.table_seed)
        changed_touched = int(np.any(rows_all.view(np.uint32) != init_all.view(np.uint32), axis=1).sum())
        assert B.np_util_table_count_changed(table, cfg.table_seed) == changed_touched
        assert int(torch.count_nonzero(state).item()) == int(np.count_nonzero(H.host(state[H.dev(touched_all)])))
        # remember the GPU's own rows for the next step (keeps rounding differences from leaking across steps)
        if t + 1 < steps:
            known_rows, known_keys = rows_all, touched_all
            known_state = H.host(state[H.dev(touched_all)])
        del init_all
        H.progress(f"[{name}] step {t}: ok")


@pytest.mark.timeout(600)
def test_full_dlrm(H):
    _full_check(H, "dlrm", steps=2)


@pytest.mark.timeout(600)
def test_full_skew(H):
    _full_check(H, "skew", steps=2)


@pytest.mark.timeout(900)
def test_full_seq(H):
    _full_check(H, "seq", steps=1)


@pytest.mark.timeout(1100)
def test_full_large_two_batches_with_overlap(H):
    """Configuration 5: two consecutive batches with 30 % distinct-key overlap; the second lookup must read the
    rows the first update wrote (Proposition 1)."""
    _full_check(H, "large", steps=2)
