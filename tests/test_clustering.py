"""Key-centric sample clustering (Section V-C): host-side preprocessing for frozen-window micro-batches.

The paper names the step and its goal (samples that share keys go to the same micro-batch, so that deduplication inside a
micro-batch removes more) but gives no algorithm, so the grouping itself has nothing to be compared with (parity unpinned).
What is fixed and checked here: the result is a balanced partition of the samples, it is deterministic, it lowers the
objective sum_i U_i against the consecutive split where the samples do fall into groups that share keys, and it does not
raise it on independent samples.  Proposition 2 (the gradient does not depend on the partition) is checked on the GPU in
tests/test_gpu_microbatch.py."""
import numpy as np
import pytest

from paper_2604_06956_amd import clustering as C
from paper_2604_06956_amd import workloads as wl


def _planted(cfg, batch, groups, seed):
    """Keys of `batch` with every key of moderate multiplicity made private to one of `groups` sample populations (the
    samples are assigned to populations at random, so the consecutive split mixes them)."""
    rng = np.random.default_rng(seed)
    group = rng.integers(0, groups, size=cfg.batch)
    samp = C.sample_of_lookup(batch.bag_offsets, cfg.batch)
    keys = batch.keys.copy()
    _, inv, cnt = np.unique(keys, return_inverse=True, return_counts=True)
    mid = cnt[inv] < cfg.batch // 4
    keys[mid] = (keys[mid] + group[samp[mid]] * 7919) % cfg.num_rows
    return keys


@pytest.fixture(scope="module")
def case():
    cfg = wl.scaled(wl.config("large"), 400, 32)          # 4096 samples x 40 features
    return cfg, wl.make_batch(cfg, 0, with_dy=False)


@pytest.mark.parametrize("N", [1, 2, 3, 4, 8, 16, 32, 48])
def test_partition_is_balanced_and_deterministic(case, N):
    cfg, b = case
    a = C.cluster_samples(b.keys, b.bag_offsets, cfg.batch, N)
    assert a.shape == (cfg.batch,) and a.dtype == np.int32 and a.min() >= 0 and a.max() < max(N, 1)
    sizes = np.bincount(a, minlength=N)
    assert sizes.sum() == cfg.batch and sizes.max() - sizes.min() <= 1
    assert np.array_equal(a, C.cluster_samples(b.keys, b.bag_offsets, cfg.batch, N))
    # the micro-batches together hold every lookup exactly once
    seen = np.zeros(b.n, np.int32)
    for m in range(N):
        pos, off, bags = C.micro_batch_lookups(b.bag_offsets, cfg.batch, cfg.features, a, m)
        seen[pos] += 1
        assert off[0] == 0 and off[-1] == pos.size and np.all(np.diff(off) == np.diff(b.bag_offsets)[bags])
    assert (seen == 1).all()


def test_passing_the_dedup_outputs_changes_nothing(case):
    cfg, b = case
    _, inv, cnt = np.unique(b.keys, return_inverse=True, return_counts=True)
    a0 = C.cluster_samples(b.keys, b.bag_offsets, cfg.batch, 8)
    a1 = C.cluster_samples(b.keys, b.bag_offsets, cfg.batch, 8, inverse=inv.astype(np.int32), counts=cnt.astype(np.int32))
    assert np.array_equal(a0, a1)


@pytest.mark.parametrize("N", [2, 4, 8, 16])
def test_lowers_the_objective_where_samples_share_keys_in_groups(case, N):
    cfg, b = case
    keys = _planted(cfg, b, groups=16, seed=N)
    U = np.unique(keys).size
    base = C.sum_unique(keys, b.bag_offsets, cfg.batch, cfg.features, C.consecutive_split(cfg.batch, N), N)
    got = C.sum_unique(keys, b.bag_offsets, cfg.batch, cfg.features, C.cluster_samples(keys, b.bag_offsets, cfg.batch, N), N)
    assert got >= U                                      # never below one copy of every key
    assert (got - U) < 0.6 * (base - U), (N, base / U, got / U)   # at least 40 % of the duplication is gone


@pytest.mark.parametrize("N", [2, 8, 32])
def test_does_not_raise_the_objective_on_independent_samples(case, N):
    cfg, b = case
    base = C.sum_unique(b.keys, b.bag_offsets, cfg.batch, cfg.features, C.consecutive_split(cfg.batch, N), N)
    got = C.sum_unique(b.keys, b.bag_offsets, cfg.batch, cfg.features, C.cluster_samples(b.keys, b.bag_offsets, cfg.batch, N), N)
    assert got <= base


def test_consecutive_split_and_degenerate_inputs():
    assert np.array_equal(C.consecutive_split(10, 3), [0, 0, 0, 0, 1, 1, 1, 2, 2, 2])
    off = np.array([0, 1, 2, 3, 4], np.int32)
    keys = np.array([5, 5, 6, 7], np.int64)
    assert np.array_equal(C.cluster_samples(keys, off, 4, 1), np.zeros(4, np.int32))
    a = C.cluster_samples(keys, off, 4, 2)
    assert sorted(np.bincount(a, minlength=2)) == [2, 2] and a[0] == a[1]     # the two samples that share key 5 stay together
