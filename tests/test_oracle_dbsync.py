"""Pins for the oracle's dual-buffer synchronisation (Section IV-B: intersection of the compact key sets of
two consecutive batches, then copies of the intersecting vectors from the active to the prefetch buffer;
Proposition 1: afterwards the prefetch buffer holds exactly W_{t+1} for the keys of the next batch)."""
import numpy as np
import pytest
from hypothesis import given, settings, strategies as st


def _check(oracle, a, b):
    ia, ib = oracle.intersect(a, b)
    common, ra, rb = np.intersect1d(a, b, assume_unique=True, return_indices=True)     # library routine
    assert np.array_equal(ia, ra) and np.array_equal(ib, rb)
    assert np.array_equal(a[ia], common) and np.array_equal(b[ib], common)


def test_intersect_vs_numpy(oracle):
    rng = np.random.default_rng(0)
    for na, nb, hi in ((1000, 800, 3000), (1, 500, 100), (500, 1, 100), (2000, 2000, 2 ** 40)):
        a = np.unique(rng.integers(0, hi, size=na)).astype(np.int64)
        b = np.unique(rng.integers(0, hi, size=nb)).astype(np.int64)
        _check(oracle, a, b)


def test_intersect_special_cases(oracle):
    a = np.arange(0, 100, 2, dtype=np.int64)
    ia, ib = oracle.intersect(a, a)                                    # identical sets: identity pairs
    assert np.array_equal(ia, np.arange(50)) and np.array_equal(ib, np.arange(50))
    ia, ib = oracle.intersect(a, a + 1)                                # disjoint
    assert ia.size == 0 and ib.size == 0
    ia, ib = oracle.intersect(a, np.empty(0, np.int64))                # one side empty
    assert ia.size == 0
    ia, ib = oracle.intersect(np.array([1, 5, 9], np.int64), np.array([0, 5, 6, 9, 12], np.int64))
    assert ia.tolist() == [1, 2] and ib.tolist() == [1, 3]
    big = np.array([2 ** 40, 2 ** 40 + 1, 2 ** 62], np.int64)           # keys that differ only above bit 32
    ia, ib = oracle.intersect(big, np.array([1, 2 ** 40 + 1, 2 ** 62], np.int64))
    assert ia.tolist() == [1, 2] and ib.tolist() == [1, 2]


@settings(max_examples=50, deadline=None)
@given(st.sets(st.integers(0, 300), max_size=80), st.sets(st.integers(0, 300), max_size=80))
def test_intersect_property(oracle, sa, sb):
    a = np.array(sorted(sa), dtype=np.int64)
    b = np.array(sorted(sb), dtype=np.int64)
    _check(oracle, a, b)


def test_sync_rows_is_a_bit_copy(oracle):
    rng = np.random.default_rng(1)
    src = rng.standard_normal((50, 12)).astype(np.float32)
    dst0 = rng.standard_normal((70, 12)).astype(np.float32)
    si = rng.choice(50, size=20, replace=False).astype(np.int32)
    di = rng.choice(70, size=20, replace=False).astype(np.int32)
    dst = dst0.copy()
    oracle.sync_rows(src, si, dst, di)
    ref = dst0.copy()
    ref[di] = src[si]                                                    # library routine
    assert dst.tobytes() == ref.tobytes()
    rest = np.setdiff1d(np.arange(70), di)
    assert dst[rest].tobytes() == dst0[rest].tobytes()


def test_dual_buffer_pipeline_equals_sequential(oracle):
    """Prefetch the vectors of B_2 before B_1 updates, run B_1 on its active buffer, synchronise the intersection,
    then run B_2's forward from the prefetch buffer: bitwise equal to the sequential run (Proposition 1); without
    the synchronisation the result differs."""
    rng = np.random.default_rng(2)
    R, D, B = 500, 8, 80
    table = (rng.standard_normal((R, D)) * 0.01).astype(np.float32)
    state = np.zeros(R, np.float32)
    batches = []
    for _ in range(2):
        lens = rng.integers(1, 7, size=B)
        off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
        keys = (rng.zipf(1.3, size=int(off[-1])) % R).astype(np.int64)
        batches.append((keys, off, rng.standard_normal((B, D)).astype(np.float32)))
    (k1, off1, dY1), (k2, off2, _) = batches
    u1, inv1, *_ = oracle.dedup(k1)
    u2, inv2, *_ = oracle.dedup(k2)
    iota1 = np.arange(u1.size, dtype=np.int64)
    iota2 = np.arange(u2.size, dtype=np.int64)
    # both buffers are filled from the table as it is before B_1's update
    _, active, _ = oracle.lookup_fwd(table, u1, None, np.array([0, 0], np.int32), 0, want_rows=True)
    _, prefetch, _ = oracle.lookup_fwd(table, u2, None, np.array([0, 0], np.int32), 0, want_rows=True)
    astate = np.zeros(u1.size, np.float32)
    # B_1 on the active buffer
    g1, _ = oracle.lookup_bwd(dY1, oracle.F32, D, 0, 1, off1, inv1, u1.size)
    oracle.sparse_adagrad(active, astate, iota1, g1, 0.01, 1e-8)
    # sequential reference: B_1 on the table itself
    oracle.sparse_adagrad(table, state, u1, g1, 0.01, 1e-8)
    seq, _, _ = oracle.lookup_fwd(table, u2, inv2, off2, 0)
    stale, _, _ = oracle.lookup_fwd(prefetch, iota2, inv2, off2, 0)
    assert stale.tobytes() != seq.tobytes()
    ia, ib = oracle.intersect(u1, u2)
    assert ia.size > 0
    oracle.sync_rows(active, ia, prefetch, ib)
    dbp, _, _ = oracle.lookup_fwd(prefetch, iota2, inv2, off2, 0)
    assert dbp.tobytes() == seq.tobytes()
