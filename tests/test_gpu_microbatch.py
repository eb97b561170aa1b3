"""Frozen-window micro-batching and the owner-side merge on the GPU (Section V-A, Proposition 2; Section IV-A,
"Embedding Retrieval": the owner deduplicates again over the keys of all sources).

A batch is split into N micro-batches.  Each runs np_dedup and np_lookup_bwd on its own; nothing is updated
in between (the frozen window).  The owner then deduplicates the concatenation of the per-micro-batch key
lists and reduces the concatenated gradient rows per key: with one "bag" per concatenated row that is
np_lookup_bwd again.  One np_sparse_adagrad follows.  The result must equal the whole-batch gradient: exactly
for integer-valued upstream gradients, within tolerance otherwise, whatever the partition."""
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


def _split(batch, cfg, N, rng):
    """Partition the bags into N micro-batches (random assignment = an arbitrary clustering of the samples)."""
    Bn = cfg.num_bags
    part = rng.integers(0, N, size=Bn)
    lens = np.diff(batch.bag_offsets)
    out = []
    for i in range(N):
        bags = np.nonzero(part == i)[0]
        off = np.concatenate([[0], np.cumsum(lens[bags])]).astype(np.int32)
        sel = np.concatenate([np.arange(batch.bag_offsets[b], batch.bag_offsets[b + 1]) for b in bags] + [np.empty(0, np.int64)])
        out.append((bags, off, batch.keys[sel.astype(np.int64)]))
    return out


def _split_by_samples(batch, cfg, assign, N):
    """Micro-batches of whole samples (all the bags of a sample go together), e.g. the clustering's result."""
    from paper_2604_06956_amd import clustering as C
    out = []
    for i in range(N):
        pos, off, bags = C.micro_batch_lookups(batch.bag_offsets, cfg.batch, cfg.features, assign, i)
        out.append((bags, off, batch.keys[pos]))
    return out


def _microbatch_grads(H, cfg, batch, dY, N, seed, parts=None):
    """-> merged unique keys, merged gradient rows (numpy), sum of micro-batch unique counts."""
    import torch
    B = H.B
    D = cfg.dim
    rng = np.random.default_rng(seed)
    if parts is None:
        parts = _split(batch, cfg, N, rng)
    key_lists, grad_lists, total_u = [], [], 0
    for bags, off, keys in parts:
        if keys.size == 0:
            continue
        d = B.np_dedup(H.dev(keys), cfg.key_bits)
        torch.cuda.synchronize()
        U = int(d["num_unique"].item())
        g = B.np_lookup_bwd(H.dev(dY[bags]), D, cfg.mode, 1, H.dev(off), keys.size, d["occ_offsets"], d["occ"], d["num_unique"], U)
        key_lists.append(d["unique"][:U])
        grad_lists.append(g[:U])
        total_u += U
    # owner side: second dedup over the keys of all micro-batches, then a per-key reduction of their gradient rows
    cat_keys = torch.cat(key_lists)
    cat_grads = torch.cat(grad_lists).contiguous()
    m = cat_keys.numel()
    d = B.np_dedup(cat_keys, cfg.key_bits)
    torch.cuda.synchronize()
    U = int(d["num_unique"].item())
    one_per_bag = torch.arange(m + 1, dtype=torch.int32, device="cuda")
    merged = B.np_lookup_bwd(cat_grads, D, B.POOL_SUM, 1, one_per_bag, m, d["occ_offsets"], d["occ"], d["num_unique"], U)
    torch.cuda.synchronize()
    return H.host(d["unique"])[:U], H.host(merged)[:U], total_u


@pytest.mark.parametrize("N", [1, 2, 4, 16])
def test_partition_invariance_exact_with_integer_gradients(H, N):
    import torch
    cfg = H.wl.config("tiny")
    batch = H.wl.make_batch(cfg, 0)
    rng = np.random.default_rng(7)
    dY = rng.integers(-8, 9, size=(cfg.num_bags, cfg.dim)).astype(np.float32)
    unique, inverse, *_ = H.O.dedup(batch.keys)
    whole, _ = H.O.lookup_bwd(dY, H.O.F32, cfg.dim, 0, 1, batch.bag_offsets, inverse, unique.size)
    keys, grads, total_u = _microbatch_grads(H, cfg, batch, dY, N, seed=N)
    assert np.array_equal(keys, unique)
    assert grads.tobytes() == whole.tobytes()            # Proposition 2: the same gradient, bit for bit
    assert total_u >= unique.size                        # dedup inside small micro-batches removes fewer keys


def test_partition_invariance_and_single_update(H):
    """Real-valued gradients on a scaled configuration 5 batch, N = 8: merged gradients within tolerance of the
    fp64 whole-batch sums, then ONE update equals the update of the whole batch."""
    import torch
    cfg = H.wl.scaled(H.wl.config("large"), 4000, 128)
    batch = H.wl.make_batch(cfg, 0)
    unique, inverse, *_ = H.O.dedup(batch.keys)
    U = unique.size
    whole, ab = H.O.lookup_bwd(batch.dY, H.O.F32, cfg.dim, 0, 1, batch.bag_offsets, inverse, U, want_abs=True)
    keys, grads, total_u = _microbatch_grads(H, cfg, batch, batch.dY, 8, seed=3)
    assert np.array_equal(keys, unique)
    H.assert_close(grads, whole, ab, H.RTOL_F32, "merged micro-batch gradients")
    assert total_u > U
    # one update after the frozen window
    R, D = cfg.num_rows, cfg.dim
    table = torch.empty((R, D), dtype=torch.float32, device="cuda")
    H.B.np_util_table_init(table, cfg.table_seed)
    state = torch.zeros(R, dtype=torch.float32, device="cuda")
    H.B.np_sparse_adagrad(table, state, H.dev(unique), H.dev(grads), H.dev(np.array([U], np.int32)), U, cfg.lr, cfg.eps)
    torch.cuda.synchronize()
    tref = H.wl.table_init_rows(np.arange(R), D, cfg.table_seed)
    before = tref.copy()
    sref = np.zeros(R, np.float32)
    H.O.sparse_adagrad(tref, sref, unique, grads, cfg.lr, cfg.eps)
    delta = np.abs(tref[unique].astype(np.float64) - before[unique])
    H.assert_close(H.host(table)[unique], tref[unique], np.abs(before[unique]) + delta, H.RTOL_F32, "single update")
    rest = np.ones(R, bool)
    rest[unique] = False
    assert H.host(table)[rest].tobytes() == before[rest].tobytes()


@pytest.mark.parametrize("name,N", [("tiny", 2), ("tiny", 8), ("scaled_large", 4), ("scaled_large", 32)])
def test_clustered_micro_batches_give_the_whole_batch_gradient(H, name, N):
    """Key-centric sample clustering (Section V-C) changes which samples share a micro-batch, nothing else: with integer
    upstream gradients the accumulated gradient equals the whole-batch one bit for bit (Proposition 2), and the number
    of vectors crossing the All2All, sum(U_i), does not exceed that of the consecutive split."""
    from paper_2604_06956_amd import clustering as C
    wl = H.wl
    cfg = wl.config("tiny") if name == "tiny" else wl.scaled(wl.config("large"), 400, 32)
    batch = wl.make_batch(cfg, 0)
    rng = np.random.default_rng(N)
    dY = rng.integers(-8, 9, size=(cfg.num_bags, cfg.dim)).astype(np.float32)
    unique, inverse, counts, *_ = H.O.dedup(batch.keys)
    whole, _ = H.O.lookup_bwd(dY, H.O.F32, cfg.dim, 0, 1, batch.bag_offsets, inverse, unique.size)
    totals = {}
    for kind, assign in (("clustered", C.cluster_samples(batch.keys, batch.bag_offsets, cfg.batch, N, inverse=inverse, counts=counts)),
                         ("consecutive", C.consecutive_split(cfg.batch, N))):
        keys, grads, totals[kind] = _microbatch_grads(H, cfg, batch, dY, N, seed=0, parts=_split_by_samples(batch, cfg, assign, N))
        assert np.array_equal(keys, unique), kind
        assert grads.tobytes() == whole.tobytes(), kind
    assert unique.size <= totals["clustered"] <= totals["consecutive"]
