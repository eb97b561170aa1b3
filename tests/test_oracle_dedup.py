"""Pins for the oracle's dedup (Section IV-A, "Key Routing": keys are deduplicated first).

The oracle sorts (key, position) pairs; these tests hold it against numpy's own unique/argsort
routines, against invariants that any correct dedup satisfies, and against hand-written cases.
"""
import numpy as np
import pytest
from hypothesis import given, settings, strategies as st


def _check_invariants(keys, unique, inverse, counts, occ_offsets, occ):
    n = keys.shape[0]
    U = unique.shape[0]
    assert np.array_equal(unique[inverse], keys)                    # inverse reconstructs the input
    assert np.all(np.diff(unique) > 0)                              # strictly ascending
    assert counts.sum() == n and np.all(counts >= 1)
    assert occ_offsets[0] == 0 and occ_offsets[U] == n
    assert np.array_equal(np.diff(occ_offsets), counts)
    assert np.array_equal(np.sort(occ), np.arange(n))               # a permutation
    ks = keys[occ]
    assert np.all(np.diff(ks) >= 0)
    same = np.diff(ks) == 0
    assert np.all(np.diff(occ)[same] > 0)                           # positions ascend inside a key
    for u in (0, U // 2, U - 1):
        seg = occ[occ_offsets[u]:occ_offsets[u + 1]]
        assert np.all(keys[seg] == unique[u])


def _vs_numpy(keys, res):
    unique, inverse, counts, occ_offsets, occ = res
    u, inv, c = np.unique(keys, return_inverse=True, return_counts=True)
    assert np.array_equal(unique, u)
    assert np.array_equal(inverse, inv.astype(np.int32))
    assert np.array_equal(counts, c.astype(np.int32))
    assert np.array_equal(occ, np.argsort(keys, kind="stable").astype(np.int32))
    assert np.array_equal(occ_offsets, np.concatenate([[0], np.cumsum(c)]).astype(np.int32))


def test_hand_case(oracle):
    keys = np.array([7, 3, 7, 7, 1, 3], dtype=np.int64)
    unique, inverse, counts, occ_offsets, occ = oracle.dedup(keys)
    assert unique.tolist() == [1, 3, 7]
    assert inverse.tolist() == [2, 1, 2, 2, 0, 1]
    assert counts.tolist() == [1, 2, 3]
    assert occ_offsets.tolist() == [0, 1, 3, 6]
    assert occ.tolist() == [4, 1, 5, 0, 2, 3]


@pytest.mark.parametrize("n,hi", [(1, 10), (2, 2), (1000, 50), (5000, 10 ** 6), (20000, 2 ** 40)])
def test_random_vs_numpy(oracle, n, hi):
    rng = np.random.default_rng(n + hi % 97)
    keys = rng.integers(0, hi, size=n, dtype=np.int64)
    res = oracle.dedup(keys)
    _vs_numpy(keys, res)
    _check_invariants(keys, *res)


def test_special_cases(oracle):
    # empty
    unique, inverse, counts, occ_offsets, occ = oracle.dedup(np.empty(0, np.int64))
    assert unique.size == 0 and inverse.size == 0 and occ_offsets.tolist() == [0]
    # all equal
    keys = np.full(777, 42, np.int64)
    unique, inverse, counts, occ_offsets, occ = oracle.dedup(keys)
    assert unique.tolist() == [42] and counts.tolist() == [777]
    assert np.array_equal(occ, np.arange(777)) and not inverse.any()
    # all distinct: inverse is the rank
    rng = np.random.default_rng(5)
    keys = rng.permutation(1000).astype(np.int64) * 3
    unique, inverse, counts, occ_offsets, occ = oracle.dedup(keys)
    assert np.array_equal(unique, np.arange(1000) * 3)
    assert np.array_equal(inverse, keys // 3)
    assert np.all(counts == 1)
    # keys that need more than 32 bits, including neighbours that differ only in the high word
    keys = np.array([2 ** 40 + 1, 1, 2 ** 40, 2 ** 33 + 1, 1, 2 ** 62], dtype=np.int64)
    res = oracle.dedup(keys)
    _vs_numpy(keys, res)


def test_zipf_batch(oracle):
    from paper_2604_06956_amd import workloads as wl
    b = wl.make_batch(wl.config("tiny"), 0, with_dy=False)
    res = oracle.dedup(b.keys)
    _vs_numpy(b.keys, res)
    _check_invariants(b.keys, *res)


@settings(max_examples=60, deadline=None)
@given(st.lists(st.integers(min_value=0, max_value=2 ** 62), min_size=0, max_size=200))
def test_property(oracle, xs):
    keys = np.array(xs, dtype=np.int64)
    res = oracle.dedup(keys)
    if keys.size:
        _vs_numpy(keys, res)
        _check_invariants(keys, *res)
    else:
        assert res[0].size == 0


def test_owner_side_second_dedup(oracle):
    """Section IV-A, "Embedding Retrieval": the owner dedups again over keys from several sources.
    Each source segment is already unique; the union equals a dedup of everything at once."""
    rng = np.random.default_rng(11)
    segs = [np.unique(rng.integers(0, 500, size=200)) for _ in range(4)]
    cat = np.concatenate(segs).astype(np.int64)
    unique, inverse, counts, _, _ = oracle.dedup(cat)
    assert np.array_equal(unique, np.unique(cat))
    assert counts.max() <= 4
    # idempotent on unique input
    u2, inv2, c2, _, _ = oracle.dedup(unique)
    assert np.array_equal(u2, unique) and np.array_equal(inv2, np.arange(unique.size)) and np.all(c2 == 1)
