"""The whole path at the largest batch the interface accepts: n = 2^31 - 2^20 - 1 lookups (index arithmetic next to the
int32 limit, 8.4 M tiles, a key with 8.4 M occurrences).  No CPU oracle finishes at this size, so every output is held
to properties that determine it completely, evaluated with plain torch operations on the device, and to closed forms
that are exact in fp32: all-ones upstream gradients make every gradient row equal the key's multiplicity (all
multiplicities stay below 2^24), small-integer table rows make every pooled value an exactly representable sum."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

N_MAX = 2**31 - 1 - 2**20


@pytest.fixture(scope="module")
def H():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    import gpu_helpers
    return gpu_helpers


def test_sizes_beyond_the_limit_are_refused(H):
    import torch
    B = H.B
    k = torch.zeros(8, dtype=torch.int64, device="cuda")
    i = torch.zeros(9, dtype=torch.int32, device="cuda")
    L = B.lib
    st = torch.cuda.current_stream().cuda_stream
    ws = torch.zeros(1024, dtype=torch.uint8, device="cuda")
    rc = L.np_dedup(k.data_ptr(), N_MAX + 1, 30, k.data_ptr(), i.data_ptr(), i.data_ptr(), i.data_ptr(), i.data_ptr(), i.data_ptr(),
                    ws.data_ptr(), 1 << 62, st)
    assert rc == -3
    f = torch.zeros(8, dtype=torch.float32, device="cuda")
    rc = L.np_lookup_bwd(f.data_ptr(), 0, 4, 0, 1, i.data_ptr(), 1, N_MAX + 1, i.data_ptr(), i.data_ptr(), i.data_ptr(), 8, 0,
                         f.data_ptr(), ws.data_ptr(), 1 << 62, st)
    assert rc == -3
    torch.cuda.synchronize()


def _all(t) -> bool:
    """Truth of a device-side check as a plain bool (kept out of the assert expression: pytest's failure report would
    otherwise try to explain a comparison of tensors with billions of elements)."""
    return bool(t.all())


def _rows(t, idx, step=1 << 24):
    """t[idx] for a 2-D t, in pieces: torch's row gather refuses to launch beyond some tens of millions of rows."""
    import torch
    return torch.cat([t[idx[i:i + step]] for i in range(0, idx.numel(), step)])


def _chunks(n, step=1 << 28):
    for lo in range(0, n, step):
        yield lo, min(n, lo + step)


@pytest.mark.timeout(900)
def test_whole_path_at_the_largest_batch(H):
    import torch
    B = H.B
    n, D, R, S, L = N_MAX, 4, 1 << 28, 1536, 8
    dev = "cuda"
    gen = torch.Generator(device=dev)
    gen.manual_seed(20260406)
    H.progress(f"[maxsize] n={n}: generating")
    keys = torch.randint(0, R, (n,), generator=gen, device=dev, dtype=torch.int64)
    hot = 123456789 % R
    keys[::256] = hot                                        # one key with n/256 = 8.4 M occurrences (< 2^24)
    nb = (n + L - 1) // L
    off = torch.arange(nb + 1, device=dev, dtype=torch.int64).mul_(L).clamp_(max=n).to(torch.int32)

    # ---------------------------------------------------------------- np_dedup
    d = B.np_dedup(keys, 28)
    torch.cuda.synchronize()
    U = int(d["num_unique"].item())
    H.progress(f"[maxsize] dedup done, U={U}")
    unique, inverse, counts, occ_offsets, occ = d["unique"][:U], d["inverse"], d["counts"][:U], d["occ_offsets"][:U + 1], d["occ"]
    ok = _all(unique[1:] > unique[:-1]) and int(unique[0]) >= 0 and int(unique[-1]) < R  # ascending, distinct
    assert ok
    assert int(counts.sum(dtype=torch.int64)) == n and int(counts.min()) >= 1
    assert int(occ_offsets[0]) == 0 and int(occ_offsets[U]) == n
    ok = _all(occ_offsets[1:] - occ_offsets[:-1] == counts)
    assert ok
    seen = torch.zeros(n, dtype=torch.bool, device=dev)
    prev_key = prev_pos = None
    for lo, hi in _chunks(n):
        ok = _all(unique[inverse[lo:hi].long()] == keys[lo:hi])  # inverse rebuilds the keys
        assert ok
        o = occ[lo:hi].long()
        assert int(o.min()) >= 0 and int(o.max()) < n
        seen[o] = True
        k = keys[o]                                                                                    # keys in occurrence order
        nondecr = k[1:] >= k[:-1]
        stable = (k[1:] > k[:-1]) | (o[1:] > o[:-1])                                                   # positions ascend inside a key
        ok = bool(nondecr.all()) and bool(stable.all())
        assert ok
        if prev_key is not None:
            assert int(k[0]) > prev_key or (int(k[0]) == prev_key and int(o[0]) > prev_pos)
        prev_key, prev_pos = int(k[-1]), int(o[-1])
        # the segment boundaries sit where the key changes: position p starts a segment iff it is an occ_offsets entry
        del o, k, nondecr, stable
    ok = bool(seen.all())  # occ is a permutation
    assert ok
    del seen
    heads = keys[occ[occ_offsets[:U].long()].long()]
    ok = _all(heads == unique)  # segment u holds key unique[u]
    assert ok
    del heads
    hot_u = int(torch.searchsorted(unique, torch.tensor([hot], device=dev))[0])
    assert int(unique[hot_u]) == hot and int(counts[hot_u]) >= n // 256
    assert int(counts.max()) < (1 << 24)
    H.progress("[maxsize] dedup properties ok")

    # ---------------------------------------------------------------- np_route (key mod S)
    cap = U + 8
    r = B.np_route(d["unique"], d["num_unique"], cap, S, B.SHARD_MOD)
    torch.cuda.synchronize()
    send_keys, splits, send_offsets = r["send_keys"][:U], r["splits"], r["send_offsets"]
    sfu, uts = r["send_from_unique"][:U], r["unique_to_send"][:U]
    assert int(splits.sum(dtype=torch.int64)) == U
    ok = int(send_offsets[0]) == 0 and int(send_offsets[S]) == U and _all(send_offsets[1:] - send_offsets[:-1] == splits)
    assert ok
    sh = send_keys % S
    ok = _all((sh[1:] > sh[:-1]) | ((sh[1:] == sh[:-1]) & (send_keys[1:] > send_keys[:-1])))  # grouped, stable
    assert ok
    ok = _all(torch.bincount(sh, minlength=S) == splits)
    assert ok
    ok = _all(send_keys[uts.long()] == unique) and _all(unique[sfu.long()] == send_keys)
    assert ok
    del sh
    H.progress("[maxsize] route properties ok")

    # ---------------------------------------------------------------- np_lookup_fwd: table[r, :] = r mod 7
    table = (torch.arange(R, device=dev) % 7).to(torch.float32).unsqueeze(1).expand(R, D).contiguous()
    state = torch.zeros(R, dtype=torch.float32, device=dev)
    out, _ = B.np_lookup_fwd(table, d["unique"], d["inverse"], off, n, B.POOL_SUM, num_list=d["num_unique"], cap=cap)
    torch.cuda.synchronize()
    full = n // L
    want = (keys[: full * L] % 7).view(full, L).sum(dim=1).to(torch.float32)
    ok = _all(out[:full] == want.unsqueeze(1))
    assert ok
    if nb > full:
        tail = float((keys[full * L:] % 7).sum())
        ok = _all(out[full] == tail)
        assert ok
    del out, want
    H.progress("[maxsize] forward ok")

    # ---------------------------------------------------------------- np_lookup_bwd: dY = 1 -> every row equals the multiplicity
    dY = torch.ones((nb, D), dtype=torch.float32, device=dev)
    grads = B.np_lookup_bwd(dY, D, B.POOL_SUM, 1, off, n, d["occ_offsets"], d["occ"], d["num_unique"], cap,
                            unique_to_send=r["unique_to_send"])
    torch.cuda.synchronize()
    want_g = counts[sfu.long()].to(torch.float32)                       # row of send slot p belongs to unique[sfu[p]]
    ok = _all(grads[:U] == want_g.unsqueeze(1))
    assert ok
    H.progress("[maxsize] backward ok")

    # ---------------------------------------------------------------- np_sparse_adagrad: closed form of the first step
    lr, eps = 0.01, 1e-8
    B.np_sparse_adagrad(table, state, r["send_keys"], grads, d["num_unique"], cap, lr, eps)
    torch.cuda.synchronize()
    H.progress("[maxsize] update ran")
    c = counts.to(torch.float64)
    w0 = (unique % 7).to(torch.float64)
    w_ref = w0 - lr * c / (c + eps)
    got = _rows(table, unique)
    ok = _all(got[:, 0:1] == got)  # the four columns move together
    assert ok
    err_w = float((got[:, 0].double() - w_ref).abs().sub_(2e-6 * w_ref.abs()).max())
    assert err_w <= 1e-7, err_w
    st = state[unique].double()
    err_s = float(((st - c * c).abs() / (c * c)).max())
    assert err_s <= 1e-6, err_s
    H.progress("[maxsize] updated rows ok")
    init = (torch.arange(R, device=dev) % 7).to(torch.float32)
    changed = int((table[:, 0] != init).sum())
    touched = int(torch.count_nonzero(state))
    assert changed == U and touched == U, (changed, touched, U)     # rows outside the batch untouched
    H.progress("[maxsize] update ok")
