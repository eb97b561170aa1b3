"""The staleness-free guarantee (Proposition 1, Eq. (2)): the parameters batch B_{t+1} reads are exactly
W_{t+1}.  Two overlapping batches run as lookup -> update -> lookup must equal the sequential result, an
emulated dual-buffer pipeline (prefetch before the update, then overwrite the intersection) must equal it
bitwise, and a pipeline that skips the overwrite must not."""
import numpy as np
import pytest

from paper_2604_06956_amd import workloads as wl


def _two_batches(seed=0, R=400, D=8, B=60):
    rng = np.random.default_rng(seed)
    table = rng.standard_normal((R, D)).astype(np.float32) * 0.01
    state = np.zeros(R, np.float32)
    batches = []
    for t in range(2):
        lens = rng.integers(1, 8, size=B)
        off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        keys = rng.zipf(1.3, size=int(off[-1])) % R
        dY = rng.standard_normal((B, D)).astype(np.float32)
        batches.append((keys.astype(np.int64), off, dY))
    return table, state, batches


def test_sequential_two_batches_and_untouched_rows(oracle):
    table, state, batches = _two_batches()
    t0 = table.copy()
    (k1, off1, dY1), (k2, off2, dY2) = batches
    r1 = oracle.step(table, state, k1, off1, dY1, oracle.F32, 0, 1, 8, oracle.SHARD_HASH, 0.01, 1e-8)
    t1 = table.copy()
    K1, K2 = np.unique(k1), np.unique(k2)
    assert np.intersect1d(K1, K2).size > 0
    # Eq. (2), first case: rows outside K(B_1) are bit-unchanged; rows inside moved
    out1 = np.setdiff1d(np.arange(table.shape[0]), K1)
    assert t1[out1].tobytes() == t0[out1].tobytes()
    assert np.all(np.any(t1[K1] != t0[K1], axis=1))
    # the forward of batch 1 read W_1, the forward of batch 2 reads W_2 = the updated table
    f1, _, _ = oracle.lookup_fwd(t0, k1, None, off1, 0)
    assert r1["out"].tobytes() == f1.tobytes()
    r2 = oracle.step(table, state, k2, off2, dY2, oracle.F32, 0, 1, 8, oracle.SHARD_HASH, 0.01, 1e-8)
    f2, _, _ = oracle.lookup_fwd(t1, k2, None, off2, 0)
    assert r2["out"].tobytes() == f2.tobytes()
    stale, _, _ = oracle.lookup_fwd(t0, k2, None, off2, 0)
    assert stale.tobytes() != f2.tobytes()             # reading W_1 for batch 2 would be visible


def test_dual_buffer_emulation_equals_sequential(oracle):
    table, state, batches = _two_batches(seed=1)
    (k1, off1, dY1), (k2, off2, dY2) = batches
    K1 = np.unique(k1)
    u2, inv2, *_ = oracle.dedup(k2)
    # prefetch buffer: rows of K(B_2) copied BEFORE batch 1 updates the table
    _, prefetch, _ = oracle.lookup_fwd(table, u2, None, np.array([0, 0], np.int32), 0, want_rows=True)
    oracle.step(table, state, k1, off1, dY1, oracle.F32, 0, 1, 8, oracle.SHARD_HASH, 0.01, 1e-8)
    # synchronise the intersection from the active copy (Section IV-B)
    both = np.intersect1d(K1, u2)
    synced = prefetch.copy()
    synced[np.searchsorted(u2, both)] = table[both]
    ident = np.arange(u2.size, dtype=np.int64)
    seq, _, _ = oracle.lookup_fwd(table, u2, inv2, off2, 0)
    dbp, _, _ = oracle.lookup_fwd(synced, ident, inv2, off2, 0)
    assert seq.tobytes() == dbp.tobytes()
    broken, _, _ = oracle.lookup_fwd(prefetch, ident, inv2, off2, 0)      # overwrite skipped: stale
    assert broken.tobytes() != seq.tobytes()


def test_overlap_construction_hits_target():
    cfg = wl.scaled(wl.config("large"), 2000, 64)
    b1 = wl.make_batch(cfg, 0, with_dy=False)
    b2 = wl.make_batch(cfg, 1, prev=b1, with_dy=False)
    K1, K2 = np.unique(b1.keys), np.unique(b2.keys)
    rho = np.intersect1d(K1, K2).size / K2.size
    assert abs(rho - 0.30) < 0.005
    # substitution keeps the multiplicity structure: same n, same bag layout
    raw = wl.make_batch(wl.Config(**{**cfg.__dict__, "overlap": None}), 1, with_dy=False)
    assert raw.n == b2.n and np.array_equal(raw.bag_offsets, b2.bag_offsets)
    assert np.array_equal(np.sort(np.unique(raw.keys, return_counts=True)[1]),
                          np.sort(np.unique(b2.keys, return_counts=True)[1]))
