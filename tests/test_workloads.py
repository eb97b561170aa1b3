"""Sanity of the synthetic input generators (no method arithmetic lives there)."""
import numpy as np
import pytest

from paper_2604_06956_amd import workloads as wl


@pytest.mark.parametrize("R,alpha", [(1000, 1.05), (10 ** 7, 1.2), (3 * 10 ** 7, 1.5)])
def test_zipf_head_frequencies_and_tail_mass(R, alpha):
    z = wl.BoundedZipf(R, alpha)
    rng = np.random.default_rng(0)
    n = 400_000
    r = z.sample(rng, n)
    assert r.min() >= 1 and r.max() <= R
    p = z.pmf_head()
    for rank in (1, 2, 5, 20):
        got = np.mean(r == rank)
        assert abs(got - p[rank - 1]) < 5 * np.sqrt(p[rank - 1] / n) + 1e-4
    if R > z.M:
        exact_tail = np.sum(np.arange(z.M + 1, R + 1, dtype=np.float64) ** -alpha)
        assert abs(exact_tail - z.tail_mass) / exact_tail < 1e-6
        assert abs(np.mean(r > z.M) - z.tail_mass / z.total_mass) < 5e-3


def test_rank_permutation_is_a_bijection():
    for R in (1000, 99991, 100000):
        ids = wl.ranks_to_ids(np.arange(1, R + 1), R, 12345)
        assert np.array_equal(np.sort(ids), np.arange(R))


def test_table_init_range_and_determinism():
    rows = np.array([0, 1, 5, 799_999_999])
    a = wl.table_init_rows(rows, 64, 7)
    b = wl.table_init_rows(rows[::-1].copy(), 64, 7)[::-1]
    assert a.dtype == np.float32 and np.array_equal(a, b)
    assert a.min() >= -0.01 and a.max() < 0.01
    big = wl.table_init_rows(np.arange(4000), 64, 7)
    assert abs(big.mean()) < 1e-4 and abs(big.std() - 0.02 / np.sqrt(12)) < 1e-4
    assert not np.array_equal(a, wl.table_init_rows(rows, 64, 8))


def test_configs_match_the_benchmark_definition():
    t = wl.config("tiny")
    assert (t.num_rows, t.dim, t.num_bags, t.num_shards, t.key_bits) == (100_000, 16, 2048, 8, 17)
    d = wl.config("dlrm")
    assert len(d.table_rows) == 26 and min(d.table_rows) >= 10 ** 4 and max(d.table_rows) <= 10 ** 7
    assert d.num_bags == 16384 * 26 and d.mode == wl.POOL_MEAN
    s = wl.config("seq")
    assert s.num_rows == 200_000_000 and s.dim == 128 and s.mode == wl.SEQ
    k = wl.config("skew")
    assert k.num_rows == 200_000_000 and k.num_shards == 1536
    L = wl.config("large")
    assert L.num_rows == 800_000_000 and L.num_bags == 131072 * 40 and L.key_bits == 30 and L.overlap == 0.30


def test_tiny_batch_shape_and_stats():
    cfg = wl.config("tiny")
    b = wl.make_batch(cfg, 0)
    assert b.bag_offsets.shape == (2049,) and b.bag_offsets[-1] == b.n and b.dY.shape == (2048, 16)
    lens = np.diff(b.bag_offsets)
    assert lens.min() >= 1 and lens.max() <= 20
    st = wl.batch_stats(b.keys)
    assert 0.25 < st["U_over_n"] < 0.40 and 1500 < st["hottest"] < 3200
    assert b.keys.min() >= 0 and b.keys.max() < cfg.num_rows
    b_again = wl.make_batch(cfg, 0)
    assert np.array_equal(b.keys, b_again.keys) and np.array_equal(b.dY, b_again.dY)


def test_seq_batch_shares_lengths_across_features():
    cfg = wl.scaled(wl.config("seq"), 1000, 256)
    b = wl.make_batch(cfg, 0)
    lens = np.diff(b.bag_offsets).reshape(cfg.features, cfg.batch)
    assert np.all(lens == lens[0]) and lens.min() >= 200 and lens.max() <= 1000
    assert b.dY.shape == (cfg.num_bags, b.max_len, cfg.dim)
    assert np.array_equal(wl.round_to_bf16(b.dY), b.dY)
    base = cfg.table_base
    for f in range(cfg.features):
        seg = b.keys[b.bag_offsets[f * cfg.batch]:b.bag_offsets[(f + 1) * cfg.batch]]
        assert seg.min() >= base[f] and seg.max() < base[f] + cfg.table_rows[f]
