"""Pins for the oracle's backward (Section II-A: gradients are aggregated at the owner; Eq. (2) sums the
per-sample gradients of a key over the batch; Proposition 2: any partition into micro-batches sums to
the same gradient)."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F


def _case(seed, R=120, D=8, B=41, maxL=9):
    rng = np.random.default_rng(seed)
    lens = rng.integers(0, maxL + 1, size=B)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    keys = rng.integers(0, R, size=int(off[-1])).astype(np.int64)
    dY = rng.standard_normal((B, D)).astype(np.float32)
    return off, keys, dY


@pytest.mark.parametrize("mode", [0, 1])
def test_vs_autograd_and_brute_force(oracle, mode):
    R, D = 120, 8
    off, keys, dY = _case(10 + mode)
    unique, inverse, counts, *_ = oracle.dedup(keys)
    g, ab = oracle.lookup_bwd(dY, oracle.F32, D, mode, 1, off, inverse, unique.size, None, want_abs=True)
    # library routine: autograd through embedding_bag on a dense weight
    w = torch.zeros(R, D, dtype=torch.float64, requires_grad=True)
    out = F.embedding_bag(torch.from_numpy(keys), w, torch.from_numpy(off[:-1].astype(np.int64)),
                          mode="sum" if mode == 0 else "mean")
    out.backward(torch.from_numpy(dY).double())
    dense = w.grad.numpy()
    assert np.allclose(g, dense[unique], rtol=1e-6, atol=1e-7)
    untouched = np.setdiff1d(np.arange(R), unique)
    assert not dense[untouched].any()
    # brute force
    ref = np.zeros((unique.size, D))
    refabs = np.zeros((unique.size, D))
    for b in range(len(off) - 1):
        L = off[b + 1] - off[b]
        for j in range(off[b], off[b + 1]):
            wj = 1.0 / L if mode == 1 else 1.0
            for d in range(D):
                ref[inverse[j], d] += wj * float(dY[b, d])
                refabs[inverse[j], d] += abs(wj * float(dY[b, d]))
    assert np.array_equal(g, ref.astype(np.float32))
    assert np.allclose(ab, refabs, rtol=1e-12)


def test_ones_gradient_gives_counts_and_single_occurrence_is_a_copy(oracle):
    off, keys, dY = _case(20)
    unique, inverse, counts, *_ = oracle.dedup(keys)
    g, _ = oracle.lookup_bwd(np.ones_like(dY), oracle.F32, 8, 0, 1, off, inverse, unique.size)
    assert np.array_equal(g, np.repeat(counts[:, None], 8, 1).astype(np.float32))
    g, _ = oracle.lookup_bwd(dY, oracle.F32, 8, 0, 1, off, inverse, unique.size)
    bag_of = np.repeat(np.arange(len(off) - 1), np.diff(off))
    for u in np.nonzero(counts == 1)[0]:
        j = int(np.nonzero(inverse == u)[0][0])
        assert g[u].tobytes() == dY[bag_of[j]].tobytes()


@pytest.mark.parametrize("mode", [0, 1])
def test_mass_conservation(oracle, mode):
    off, keys, dY = _case(30 + mode, B=200)
    unique, inverse, *_ = oracle.dedup(keys)
    g, _ = oracle.lookup_bwd(dY, oracle.F32, 8, mode, 1, off, inverse, unique.size)
    lens = np.diff(off).astype(np.float64)
    wsum = lens if mode == 0 else (lens > 0).astype(np.float64)      # L * w
    assert np.allclose(g.astype(np.float64).sum(0), (wsum[:, None] * dY.astype(np.float64)).sum(0), atol=1e-4)


def test_send_order_placement(oracle):
    off, keys, dY = _case(40)
    unique, inverse, *_ = oracle.dedup(keys)
    _, _, _, sfu, uts = oracle.route(unique, 8, oracle.SHARD_HASH)
    g, _ = oracle.lookup_bwd(dY, oracle.F32, 8, 0, 1, off, inverse, unique.size)
    gs, _ = oracle.lookup_bwd(dY, oracle.F32, 8, 0, 1, off, inverse, unique.size, uts)
    assert gs.tobytes() == g[sfu].tobytes()


def test_partition_invariance(oracle):
    """Proposition 2: split the bags into N micro-batches any way; per-key gradients add up to the
    whole-batch gradient.  Integer-valued dY makes every sum exact, so equality is bitwise."""
    rng = np.random.default_rng(50)
    off, keys, _ = _case(50, B=64)
    B = len(off) - 1
    dY = rng.integers(-8, 9, size=(B, 8)).astype(np.float32)
    unique, inverse, *_ = oracle.dedup(keys)
    whole, _ = oracle.lookup_bwd(dY, oracle.F32, 8, 0, 1, off, inverse, unique.size)
    for N in (2, 4, 7):
        part = rng.integers(0, N, size=B)
        acc = np.zeros((unique.size, 8), np.float64)
        for i in range(N):
            bags = np.nonzero(part == i)[0]
            lens = np.diff(off)[bags]
            moff = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
            mkeys = np.concatenate([keys[off[b]:off[b + 1]] for b in bags] + [np.empty(0, np.int64)]).astype(np.int64)
            mu, minv, *_ = oracle.dedup(mkeys)
            mg, _ = oracle.lookup_bwd(dY[bags], oracle.F32, 8, 0, 1, moff, minv, mu.size)
            acc[np.searchsorted(unique, mu)] += mg
        assert np.array_equal(acc.astype(np.float32), whole)


def test_seq_mode_bf16_and_padding_ignored(oracle):
    rng = np.random.default_rng(60)
    B, D, R = 9, 16, 40
    lens = rng.integers(0, 7, size=B)
    max_len = int(lens.max())
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    keys = rng.integers(0, R, size=int(off[-1])).astype(np.int64)
    dY32 = torch.randn(B, max_len, D, generator=torch.Generator().manual_seed(1))
    dYb = dY32.bfloat16()
    bits = dYb.view(torch.int16).numpy().astype(np.uint16).copy()
    for b in range(B):                                   # poison the padding: it must never be read
        bits[b, lens[b]:] = 0x7FC0
    unique, inverse, *_ = oracle.dedup(keys)
    g, _ = oracle.lookup_bwd(bits, oracle.BF16, D, 2, max_len, off, inverse, unique.size)
    assert np.isfinite(g).all()
    # library routine: autograd through a plain embedding of the flattened lookups
    w = torch.zeros(R, D, dtype=torch.float64, requires_grad=True)
    e = F.embedding(torch.from_numpy(keys), w)
    up = torch.cat([dYb[b, :lens[b]].double() for b in range(B)])
    e.backward(up)
    assert np.allclose(g, w.grad.numpy()[unique], rtol=1e-6, atol=1e-7)
