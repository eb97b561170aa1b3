"""The owner's side of "Embedding Retrieval" on the GPU (Section IV-A): the owner receives one deduplicated key list
from every source, deduplicates again over their concatenation, reads every distinct row ONCE, and hands each source
the vectors of its keys.  With S_src sources emulated on the one GPU:

    cat = [list_0 | list_1 | ... ]                    np_dedup(cat)           -> unique_o, inverse_o
    rows_o = table[unique_o]                           np_lookup_fwd(rows_out) -> one gather of U_o rows
    back_s[i] = rows_o[inverse_o[off_s + i]]           np_sync_rows            -> source s's slice of the reply

Every source's reply must equal table[list_s] bit for bit, the owner's key set must be the union of the lists, and
merging is idempotent: merging the merged list again (alone, or together with any of the lists) changes nothing."""
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


def _source_lists(H, cfg, batch, num_src, rng):
    """Each source holds a share of the samples and sends the ascending distinct keys of its share."""
    import torch
    part = rng.integers(0, num_src, size=cfg.num_bags)
    lists = []
    for s in range(num_src):
        bags = np.nonzero(part == s)[0]
        sel = np.concatenate([np.arange(batch.bag_offsets[b], batch.bag_offsets[b + 1]) for b in bags] + [np.empty(0, np.int64)])
        keys = batch.keys[sel.astype(np.int64)]
        if keys.size == 0:
            lists.append(np.empty(0, np.int64))
            continue
        d = H.B.np_dedup(H.dev(keys), cfg.key_bits)
        torch.cuda.synchronize()
        lists.append(H.host(d["unique"])[:int(d["num_unique"].item())].copy())
    return lists


def _owner_merge(H, cfg, table, lists):
    """-> unique_o (numpy), per-source reply rows (numpy), the owner's row buffer (device), U_o."""
    import torch
    B = H.B
    D = cfg.dim
    cat = np.concatenate(lists)
    m = cat.size
    d = B.np_dedup(H.dev(cat), cfg.key_bits)
    torch.cuda.synchronize()
    U = int(d["num_unique"].item())
    no_bags = H.dev(np.array([0], np.int32))
    _, rows_o = B.np_lookup_fwd(table, d["unique"], None, no_bags, 0, B.POOL_SUM, num_list=d["num_unique"], cap=U, want_rows=True,
                                out=torch.empty((0, D), dtype=torch.float32, device="cuda"))
    replies, off = [], 0
    for ls in lists:
        k = ls.size
        back = torch.full((max(k, 1), D), float("nan"), dtype=torch.float32, device="cuda")
        if k:
            sl = d["inverse"][off:off + k].contiguous()
            B.np_sync_rows(rows_o, sl, back, torch.arange(k, dtype=torch.int32, device="cuda"), H.dev(np.array([k], np.int32)), k)
        replies.append(back[:k])
        off += k
    torch.cuda.synchronize()
    return H.host(d["unique"])[:U].copy(), [H.host(r) for r in replies], rows_o, U, d


@pytest.mark.parametrize("name,num_src", [("tiny", 3), ("tiny", 8), ("scaled_large", 4), ("scaled_large", 16)])
def test_rows_back_per_source_bit_exact(H, name, num_src):
    import torch
    wl, O = H.wl, H.O
    cfg = wl.config("tiny") if name == "tiny" else wl.scaled(wl.config("large"), 4000, 128)
    batch = wl.make_batch(cfg, 0, with_dy=False)
    R, D = cfg.num_rows, cfg.dim
    table = torch.empty((R, D), dtype=torch.float32, device="cuda")
    H.B.np_util_table_init(table, cfg.table_seed)
    lists = _source_lists(H, cfg, batch, num_src, np.random.default_rng(num_src))
    unique_o, replies, rows_o, U, d = _owner_merge(H, cfg, table, lists)
    cat = np.concatenate(lists)
    # the oracle on the same concatenation: second dedup, one row per distinct key, rows handed back through inverse
    ru, rinv, rcounts, _, _ = O.dedup(cat)
    assert np.array_equal(unique_o, ru)
    assert np.array_equal(unique_o, np.unique(batch.keys))                      # the union of the lists = the batch's key set
    assert np.array_equal(H.host(d["inverse"])[:cat.size], rinv)
    assert np.array_equal(H.host(d["counts"])[:U], rcounts)                      # how many sources asked for each key
    tref = wl.table_init_rows(ru, D, cfg.table_seed)                             # the rows of the distinct keys, in key order
    _, rows_ref, _ = O.lookup_fwd(tref, np.arange(ru.size), None, np.array([0], np.int32), 0, want_rows=True)
    assert H.host(rows_o)[:U].tobytes() == rows_ref.tobytes()                    # gathered once, U_o rows
    off = 0
    for s, ls in enumerate(lists):
        want = rows_ref[rinv[off:off + ls.size]]
        assert replies[s].tobytes() == want.tobytes(), f"source {s}"
        assert replies[s].tobytes() == wl.table_init_rows(ls, D, cfg.table_seed).tobytes()   # = table[list_s] by definition
        off += ls.size


def test_merge_is_idempotent(H):
    import torch
    wl = H.wl
    cfg = wl.scaled(wl.config("large"), 4000, 128)
    batch = wl.make_batch(cfg, 0, with_dy=False)
    table = torch.empty((cfg.num_rows, cfg.dim), dtype=torch.float32, device="cuda")
    H.B.np_util_table_init(table, cfg.table_seed)
    lists = _source_lists(H, cfg, batch, 6, np.random.default_rng(1))
    unique_o, _, rows_o, U, _ = _owner_merge(H, cfg, table, lists)
    # merging the merged list alone: same keys, every key once, identity inverse, the same rows
    again, replies, rows_again, U2, d2 = _owner_merge(H, cfg, table, [unique_o])
    assert U2 == U and np.array_equal(again, unique_o)
    assert np.array_equal(H.host(d2["inverse"])[:U], np.arange(U, dtype=np.int32))
    assert (H.host(d2["counts"])[:U] == 1).all()
    assert H.host(rows_again)[:U].tobytes() == H.host(rows_o)[:U].tobytes()
    assert replies[0].tobytes() == H.host(rows_o)[:U].tobytes()
    # merging it together with lists it already contains adds nothing
    more, _, rows_more, U3, _ = _owner_merge(H, cfg, table, [unique_o, lists[0], lists[3]])
    assert U3 == U and np.array_equal(more, unique_o)
    assert H.host(rows_more)[:U].tobytes() == H.host(rows_o)[:U].tobytes()
