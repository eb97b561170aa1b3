"""Pins for the oracle's routing (Section IV-A: deduplicated keys are partitioned into buckets by
the table-sharding rule; the buckets are the key All2All payload)."""
import os

import numpy as np
import pytest

M64 = (1 << 64) - 1
C = 0x9E3779B97F4A7C15


def _unmix(a: int) -> int:
    """Undo the routing hash step by step with exact integers: each stage is a bijection of 64-bit
    words (xor-shift by s >= 22 is undone by two more applications; an odd multiplier has an inverse)."""
    cinv = pow(C, -1, 1 << 64)
    a ^= a >> 29
    a ^= a >> 58
    a = (a * cinv) & M64
    a ^= a >> 32
    a = (a * cinv) & M64
    return a


def test_mix_is_a_bijection_with_known_inverse(oracle):
    rng = np.random.default_rng(1)
    xs = [0, 1, 2, 1535, 1536, 2 ** 31, 2 ** 32, 2 ** 63, M64] + [int(x) for x in rng.integers(0, 2 ** 63, 200)]
    for x in xs:
        assert _unmix(oracle.mix(x)) == x
    assert oracle.mix(0) == 0


def test_mix_spreads_sequential_keys(oracle):
    """Consecutive row ids must land on shards uniformly (chi-square far below a loose bound)."""
    S = 1536
    n = 1536 * 200
    sh = np.array([oracle.shard(k, S, oracle.SHARD_HASH) for k in range(n)])
    counts = np.bincount(sh, minlength=S)
    chi2 = ((counts - n / S) ** 2 / (n / S)).sum()
    assert chi2 < S + 6 * np.sqrt(2 * S)          # mean S-1, sd sqrt(2(S-1))
    # strided ids (what a modulo rule maps to one shard) spread as well
    sh = np.array([oracle.shard(k * S, S, oracle.SHARD_HASH) for k in range(n // 4)])
    counts = np.bincount(sh, minlength=S)
    chi2 = ((counts - n / 4 / S) ** 2 / (n / 4 / S)).sum()
    assert chi2 < S + 6 * np.sqrt(2 * S)


def test_mix_golden(oracle):
    """Regression guard: values written once by tests/golden/make_mix_golden.py (which calls only the oracle)."""
    path = os.path.join(os.path.dirname(__file__), "golden", "mix_golden.txt")
    rows = [ln.split() for ln in open(path) if ln.strip() and not ln.startswith("#")]
    assert len(rows) >= 8
    for k, v in rows:
        assert oracle.mix(int(k, 16)) == int(v, 16)


def test_shard_mod_is_plain_modulo(oracle):
    for k in [0, 1, 7, 8, 9, 12345678901234]:
        assert oracle.shard(k, 8, oracle.SHARD_MOD) == k % 8


def _check(oracle, unique, S, fn):
    send_keys, splits, send_offsets, sfu, uts = oracle.route(unique, S, fn)
    U = unique.shape[0]
    sh = np.array([oracle.shard(int(k), S, fn) for k in unique], dtype=np.int64)
    assert splits.sum() == U                                            # per-shard splits sum to the unique count
    assert np.array_equal(splits, np.bincount(sh, minlength=S))
    assert np.array_equal(send_offsets, np.concatenate([[0], np.cumsum(splits)]))
    assert np.array_equal(sfu, np.argsort(sh, kind="stable"))          # library routine
    assert np.array_equal(send_keys, unique[sfu])
    assert np.array_equal(uts[sfu], np.arange(U)) and np.array_equal(sfu[uts], np.arange(U))
    assert np.array_equal(send_keys[uts], unique)
    for s in range(S):
        seg = send_keys[send_offsets[s]:send_offsets[s + 1]]
        assert np.all(np.diff(seg) > 0)                                 # ascending inside a bucket
        assert all(oracle.shard(int(k), S, fn) == s for k in seg[:3])
    return send_keys, splits


@pytest.mark.parametrize("S,fn", [(8, 0), (8, 1), (64, 1), (1536, 1), (1, 0), (1, 1), (3, 0)])
def test_route_vs_numpy(oracle, S, fn):
    rng = np.random.default_rng(S * 2 + fn)
    unique = np.unique(rng.integers(0, 10 ** 7, size=4000)).astype(np.int64)
    _check(oracle, unique, S, fn)


def test_route_special_cases(oracle):
    # one shard: identity
    unique = np.arange(0, 100, 3, dtype=np.int64)
    send_keys, splits, send_offsets, sfu, uts = oracle.route(unique, 1, oracle.SHARD_MOD)
    assert np.array_equal(send_keys, unique) and splits.tolist() == [unique.size]
    assert np.array_equal(sfu, np.arange(unique.size)) and np.array_equal(uts, np.arange(unique.size))
    # modulo rule with keys 0..S-1: one per shard, in place
    unique = np.arange(8, dtype=np.int64)
    send_keys, splits, _, sfu, _ = oracle.route(unique, 8, oracle.SHARD_MOD)
    assert splits.tolist() == [1] * 8 and np.array_equal(send_keys, unique)
    # hand case, S = 3 modulo
    unique = np.array([1, 3, 4, 6, 8], dtype=np.int64)
    send_keys, splits, send_offsets, sfu, uts = oracle.route(unique, 3, oracle.SHARD_MOD)
    assert send_keys.tolist() == [3, 6, 1, 4, 8]
    assert splits.tolist() == [2, 2, 1] and send_offsets.tolist() == [0, 2, 4, 5]
    assert sfu.tolist() == [1, 3, 0, 2, 4] and uts.tolist() == [2, 0, 3, 1, 4]
    # empty
    send_keys, splits, send_offsets, _, _ = oracle.route(np.empty(0, np.int64), 4, oracle.SHARD_HASH)
    assert send_keys.size == 0 and splits.tolist() == [0] * 4 and send_offsets.tolist() == [0] * 5


def test_compose(oracle):
    rng = np.random.default_rng(3)
    keys = rng.integers(0, 300, size=2000).astype(np.int64)
    unique, inverse, *_ = oracle.dedup(keys)
    send_keys, _, _, _, uts = oracle.route(unique, 16, oracle.SHARD_HASH)
    l2s = oracle.compose(inverse, uts)
    assert np.array_equal(send_keys[l2s], keys)      # every lookup finds its own key in the send buffer
