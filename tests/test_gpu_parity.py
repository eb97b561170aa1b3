"""GPU parity: every C-ABI call against the CPU oracle, element by element, on seeded inputs that span
several tiles and ragged tails, plus the degenerate cases of each step.  Integer outputs must be bit
exact; values must be within 1e-5 (fp32) / 1e-2 (bf16) of the oracle, measured against the sum of the
absolute terms of each element."""
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


# ------------------------------------------------------------------------------------------ harness

def test_table_init_matches_the_numpy_generator(H):
    import torch
    for R, D in ((1000, 16), (777, 64), (50, 128)):
        t = torch.empty((R, D), dtype=torch.float32, device="cuda")
        H.B.np_util_table_init(t, 7)
        ref = H.wl.table_init_rows(np.arange(R), D, 7)
        assert H.host(t).tobytes() == ref.tobytes()


def test_gather_yardstick_reads_the_rows_it_says(H):
    """np_util_gather_rate against its definition: row read i = hash(i, seed) mod-scaled into num_rows, sums of 64 reads."""
    import torch
    rng = np.random.default_rng(3)
    R, n, seed = 1000, 64 * 37, 5
    src = rng.integers(-3, 4, size=(R + 50, 64)).astype(np.float32)         # small integers: the sums are exact in any order
    out = torch.full((n // 64, 64), -1.0, dtype=torch.float32, device="cuda")
    H.B.np_util_gather_rate(H.dev(src), R, n, seed, out)
    torch.cuda.synchronize()
    i = np.arange(n, dtype=np.uint64)
    h = (i * 2654435761 + seed) & 0xFFFFFFFF
    h ^= h >> 16
    h = (h * 0x7feb352d) & 0xFFFFFFFF
    h ^= h >> 15
    h = (h * 0x846ca68b) & 0xFFFFFFFF
    h ^= h >> 16
    rows = ((h * R) >> 32).astype(np.int64)
    assert rows.max() < R
    want = src[rows].reshape(n // 64, 64, 64).sum(axis=1)
    assert np.array_equal(H.host(out), want)


# ------------------------------------------------------------------------------------------ dedup

def _keys_case(name):
    import zlib
    rng = np.random.default_rng(zlib.crc32(name.encode()))
    if name == "one":
        return np.array([5], np.int64), 3
    if name == "all_equal":
        return np.full(10000, 123456, np.int64), 17
    if name == "all_distinct":
        return rng.permutation(50000).astype(np.int64), 16
    if name == "wave_edges":
        return rng.integers(0, 50, size=64 * 16 * 4 + 1).astype(np.int64), 6
    if name == "tile_minus_1":
        return rng.integers(0, 1 << 20, size=4095).astype(np.int64), 20
    if name == "tile_exact":
        return rng.integers(0, 1 << 20, size=4096).astype(np.int64), 20
    if name == "tile_plus_1":
        return rng.integers(0, 1 << 20, size=4097).astype(np.int64), 20
    if name == "multi_chunk":
        return rng.integers(0, 1 << 27, size=5_000_000).astype(np.int64), 27
    if name == "bits_1":
        return rng.integers(0, 2, size=30000).astype(np.int64), 1
    if name == "bits_32":      # the widest key that still sorts as 32 bits: values with the top bit set
        k = rng.integers(0, 1 << 32, size=150000).astype(np.int64)
        k[:100] = (1 << 32) - 1
        k[100:200] = 1 << 31
        k[200:300] = 0
        return k, 32
    if name == "bits_33":
        return rng.integers(0, 1 << 33, size=200000).astype(np.int64), 33
    if name == "bits_40_dups":
        base = rng.integers(0, 1 << 40, size=3000).astype(np.int64)
        return base[rng.integers(0, 3000, size=100000)], 40
    if name == "bits_63":
        base = rng.integers(0, (1 << 63) - 1, size=5000).astype(np.int64)
        return base[rng.integers(0, 5000, size=60000)], 63
    if name == "bits_32_many_tiles":   # 2048 bins: staging shares the counters' LDS; several tiles per chunk
        k = rng.integers(0, 1 << 32, size=3_000_001).astype(np.int64)
        k[rng.random(k.size) < 0.2] = (1 << 32) - 7
        return k, 32
    if name == "bits_40_many_tiles":   # 64-bit sort keys (separate key and position arrays), several tiles per chunk
        base = rng.integers(0, 1 << 40, size=400_000).astype(np.int64)
        return base[rng.integers(0, base.size, size=2_500_003)], 40
    if name == "hot_key":
        k = rng.integers(0, 1 << 28, size=300000).astype(np.int64)
        k[rng.random(300000) < 0.4] = 77777777
        return k, 28
    raise KeyError(name)


DEDUP_CASES = ["one", "all_equal", "all_distinct", "wave_edges", "tile_minus_1", "tile_exact", "tile_plus_1",
               "multi_chunk", "bits_1", "bits_32", "bits_33", "bits_40_dups", "bits_63", "hot_key", "bits_32_many_tiles",
               "bits_40_many_tiles"]


@pytest.mark.parametrize("case", DEDUP_CASES)
def test_dedup_bit_exact(H, case):
    keys, bits = _keys_case(case)
    g, _ = H.gpu_dedup(keys, bits)
    H.assert_dedup_equal(g, keys)


@pytest.fixture
def tile_ordered_emit(H):
    """Forces np_dedup's tile-ordered way of writing the inverse map (taken on its own only for batches of millions of
    lookups) for every size; the outputs are the same bits either way."""
    old = H.B.np_tune_get("emit_order_min_n")
    H.B.np_tune_set("emit_order_min_n", 0)
    yield
    H.B.np_tune_set("emit_order_min_n", old)


@pytest.mark.parametrize("case", DEDUP_CASES + ["tile1024_minus_1", "tile1024_exact", "tile1024_plus_1", "hot_runs",
                                                "hot_runs_wide_keys", "counts_around_33", "keys_34_each"])
def test_dedup_bit_exact_with_the_tile_ordered_inverse_map(H, tile_ordered_emit, case):
    if case == "hot_runs_wide_keys":    # 64-bit sort keys: popular keys beside cold ones
        rng = np.random.default_rng(7)
        keys = rng.integers(0, 1 << 40, size=300_001).astype(np.int64)
        pick = rng.random(keys.size)
        keys[pick < 0.25] = (1 << 39) + 5
        keys[(pick >= 0.25) & (pick < 0.40)] = 3
        hot = rng.integers(0, 1 << 40, size=500)
        sel = (pick >= 0.40) & (pick < 0.70)
        keys[sel] = hot[rng.integers(0, hot.size, size=int(sel.sum()))]
        bits = 40
    elif case == "counts_around_33":    # keys with 31 .. 35 lookups each, shuffled
        rng = np.random.default_rng(33)
        reps = np.repeat(np.arange(31, 36), 400)
        keys = np.repeat(rng.permutation(1 << 20)[:reps.size].astype(np.int64), reps)
        keys = keys[rng.permutation(keys.size)]
        bits = 20
    elif case == "keys_34_each":    # 100 000 keys with 34 lookups each, shuffled: no segment fills a tile, every tile holds ~30 heads
        rng = np.random.default_rng(34)
        keys = np.repeat(np.arange(100_000, dtype=np.int64) * 7919 % (1 << 24), 34)
        keys = keys[rng.permutation(keys.size)]
        bits = 24
    elif case.startswith("tile1024"):
        rng = np.random.default_rng(len(case))
        keys = rng.integers(0, 300, size=1024 * 3 + {"minus_1": -1, "exact": 0, "plus_1": 1}[case.split("_", 1)[1]]).astype(np.int64)
        bits = 9
    elif case == "hot_runs":    # several keys whose segments cover whole tiles, beside many cold keys, ragged end
        rng = np.random.default_rng(99)
        keys = rng.integers(0, 1 << 22, size=700_001).astype(np.int64)
        pick = rng.random(keys.size)
        keys[pick < 0.30] = 12345
        keys[(pick >= 0.30) & (pick < 0.45)] = 4_000_000
        keys[(pick >= 0.45) & (pick < 0.50)] = 0
        bits = 22
    else:
        keys, bits = _keys_case(case)
    g, _ = H.gpu_dedup(keys, bits)
    H.assert_dedup_equal(g, keys)
    d = H.B.np_dedup(H.dev(keys), bits, want_inverse=False)      # without the inverse map the chunked kernel runs: same bits
    import torch
    torch.cuda.synchronize()
    U = g["U"]
    for name, k in (("unique", U), ("counts", U), ("occ_offsets", U + 1), ("occ", keys.shape[0])):
        assert H.host(d[name])[:k].tobytes() == g[name].tobytes(), name


def test_tunables(H):
    B = H.B
    assert B.np_tune_get("no_such_knob") == -1
    with pytest.raises(B.NestPipeError):
        B.np_tune_set("no_such_knob", 1)
    with pytest.raises(B.NestPipeError):
        B.np_tune_set("emit_order_min_n", -5)
    old = B.np_tune_get("bwd_order_min_dy_bytes")
    assert old == 256 << 20
    B.np_tune_set("bwd_order_min_dy_bytes", 12345)
    assert B.np_tune_get("bwd_order_min_dy_bytes") == 12345
    B.np_tune_set("bwd_order_min_dy_bytes", old)


def test_dedup_empty(H):
    import torch
    d = H.B.np_dedup(torch.empty(0, dtype=torch.int64, device="cuda"), 10)
    torch.cuda.synchronize()
    assert int(d["num_unique"].item()) == 0 and int(d["occ_offsets"][0].item()) == 0


def test_dedup_is_deterministic(H):
    keys, bits = _keys_case("hot_key")
    a, _ = H.gpu_dedup(keys, bits)
    b, _ = H.gpu_dedup(keys, bits)
    for k in ("unique", "inverse", "counts", "occ_offsets", "occ"):
        assert a[k].tobytes() == b[k].tobytes()


def test_dedup_without_inverse(H):
    """The inverse map is optional: the other outputs do not change, and a buffer passed in its place stays untouched."""
    import torch
    keys, bits = _keys_case("multi_chunk")
    full, _ = H.gpu_dedup(keys, bits)
    d = H.B.np_dedup(H.dev(keys), bits, want_inverse=False)
    torch.cuda.synchronize()
    assert d["inverse"] is None
    U = int(d["num_unique"].item())
    assert U == full["U"]
    n = keys.shape[0]
    for name, k in (("unique", U), ("counts", U), ("occ_offsets", U + 1), ("occ", n)):
        assert H.host(d[name])[:k].tobytes() == full[name].tobytes(), name


# ------------------------------------------------------------------------------------------ route

@pytest.mark.parametrize("S,fn", [(1, 0), (3, 1), (7, 0), (8, 0), (8, 1), (64, 1), (1000, 0), (1535, 1), (1536, 1), (4095, 0), (4096, 1)])
@pytest.mark.parametrize("U", [1, 4097, 300000])
def test_route_bit_exact(H, S, fn, U):
    import torch
    rng = np.random.default_rng(S * 7 + fn + U)
    unique = np.unique(rng.integers(0, 1 << 33, size=U)).astype(np.int64)
    U = unique.shape[0]
    inv = rng.integers(0, U, size=2 * U + 3).astype(np.int32)
    cap = U + 100                                       # the host bound may exceed the device count
    ubuf = np.zeros(cap, np.int64)
    ubuf[:U] = unique
    r = H.B.np_route(H.dev(ubuf), H.dev(np.array([U], np.int32)), cap, S, fn, inverse=H.dev(inv), n=inv.shape[0])
    torch.cuda.synchronize()
    send_keys, splits, send_offsets, sfu, uts = H.O.route(unique, S, fn)
    assert np.array_equal(H.host(r["send_keys"])[:U], send_keys)
    assert np.array_equal(H.host(r["splits"])[:S], splits)
    assert np.array_equal(H.host(r["send_offsets"])[:S + 1], send_offsets)
    assert np.array_equal(H.host(r["send_from_unique"])[:U], sfu)
    assert np.array_equal(H.host(r["unique_to_send"])[:U], uts)
    assert np.array_equal(H.host(r["lookup_to_send"])[:inv.shape[0]], H.O.compose(inv, uts))


def test_route_zero_keys(H):
    import torch
    r = H.B.np_route(torch.zeros(16, dtype=torch.int64, device="cuda"), H.dev(np.array([0], np.int32)), 16, 8, 1)
    torch.cuda.synchronize()
    assert not H.host(r["splits"]).any() and not H.host(r["send_offsets"]).any()


# ------------------------------------------------------------------------------------------ forward

def _bags(rng, B, max_l, R, allow_empty=True):
    lens = rng.integers(0 if allow_empty else 1, max_l + 1, size=B)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    keys = rng.integers(0, R, size=int(off[-1])).astype(np.int64)
    return off, keys


@pytest.mark.parametrize("dim", [4, 8, 16, 48, 64, 128, 256, 512, 768, 1024])
@pytest.mark.parametrize("mode", [0, 1])
def test_fwd_pooled(H, dim, mode):
    import torch
    rng = np.random.default_rng(dim * 3 + mode)
    R, Bn = 3000, 1237
    table = rng.standard_normal((R, dim)).astype(np.float32)
    off, keys = _bags(rng, Bn, 70 if dim <= 128 else 9, R)
    unique, inverse, *_ = H.O.dedup(keys)
    ref, _, ab = H.O.lookup_fwd(table, unique, inverse, off, mode, want_abs=True)
    out, _ = H.B.np_lookup_fwd(H.dev(table), H.dev(unique), H.dev(inverse), H.dev(off), keys.shape[0], mode)
    torch.cuda.synchronize()
    H.assert_close(H.host(out), ref, ab, H.RTOL_F32, f"fwd pooled dim={dim} mode={mode}")
    empty = np.diff(off) == 0
    assert not H.host(out)[empty].any()
    # direct path (no slot indirection) and bf16 output
    out2, _ = H.B.np_lookup_fwd(H.dev(table), H.dev(keys), None, H.dev(off), keys.shape[0], mode)
    torch.cuda.synchronize()
    assert H.host(out2).tobytes() == H.host(out).tobytes()
    out3, _ = H.B.np_lookup_fwd(H.dev(table), H.dev(unique), H.dev(inverse), H.dev(off), keys.shape[0], mode, out_dtype=H.B.BF16)
    torch.cuda.synchronize()
    H.assert_close(H.O.bf16_bits_to_f32(H.host(out3)), ref, ab, H.RTOL_BF16, "fwd pooled bf16")


@pytest.mark.parametrize("dim", [16, 128, 512])
def test_fwd_seq_bit_exact_and_rows_out(H, dim):
    import torch
    rng = np.random.default_rng(dim)
    R, Bn = 5000, 211
    table = rng.standard_normal((R, dim)).astype(np.float32)
    off, keys = _bags(rng, Bn, 37, R)
    max_len = int(np.diff(off).max())
    unique, inverse, *_ = H.O.dedup(keys)
    U = unique.shape[0]
    for dt in (H.B.BF16, H.B.F32):
        ref, rows, _ = H.O.lookup_fwd(table, unique, inverse, off, 2, max_len, dt, want_rows=True)
        out = torch.full((Bn, max_len, dim), 7.0, dtype=torch.bfloat16 if dt == H.B.BF16 else torch.float32, device="cuda")
        out, rows_g = H.B.np_lookup_fwd(H.dev(table), H.dev(unique), H.dev(inverse), H.dev(off), keys.shape[0], 2, max_len, dt,
                                        num_list=H.dev(np.array([U], np.int32)), cap=U + 5, want_rows=True, out=out)
        torch.cuda.synchronize()
        assert H.host(out).tobytes() == ref.tobytes()                 # a copy / one rounding: bit exact, zero padding
        assert H.host(rows_g)[:U].tobytes() == rows.tobytes()


@pytest.mark.parametrize("dim,mode", [(16, 0), (64, 1), (128, 2), (520, 0)])
def test_fwd_in_two_stages_like_the_sharded_flow(H, dim, mode):
    """Owner side: rows_out = table[send_keys] (the payload of the embedding All2All).  Requester side: pooling straight
    from that buffer through lookup_to_send (list_keys = NULL: the slot is the row).  Same rows in the same order as the
    one-call forward, so the same bits; and equal to the oracle's forward over the identity key list."""
    import torch
    rng = np.random.default_rng(dim + mode)
    R, Bn, S = 4000, 700, 64
    table = rng.standard_normal((R, dim)).astype(np.float32)
    off, keys = _bags(rng, Bn, 30, R)
    max_len = max(1, int(np.diff(off).max()))
    n = keys.shape[0]
    d = H.B.np_dedup(H.dev(keys), 12)
    r = H.B.np_route(d["unique"], d["num_unique"], n, S, 1, inverse=d["inverse"], n=n)
    dt = H.B.BF16 if mode == 2 else H.B.F32
    tab = H.dev(table)
    one, rows = H.B.np_lookup_fwd(tab, r["send_keys"], r["lookup_to_send"], H.dev(off), n, mode, max_len, dt,
                                  num_list=d["num_unique"], cap=n, want_rows=True)
    two, _ = H.B.np_lookup_fwd(rows, None, r["lookup_to_send"], H.dev(off), n, mode, max_len, dt)
    torch.cuda.synchronize()
    U = int(d["num_unique"].item())
    assert H.host(two).tobytes() == H.host(one).tobytes()
    l2s = H.host(r["lookup_to_send"])[:n]
    ref, _, ab = H.O.lookup_fwd(H.host(rows)[:U], np.arange(U, dtype=np.int64), l2s, off, mode, max_len, dt, want_abs=mode != 2)
    if mode == 2:
        assert H.host(two).tobytes() == ref.tobytes()
    else:
        H.assert_close(H.host(two), ref, ab, H.RTOL_F32, "requester-side pooling")


# ------------------------------------------------------------------------------------------ backward

def _bwd_case(rng, dim, Bn, max_l, R, hot=0.0):
    off, keys = _bags(rng, Bn, max_l, R)
    if hot > 0:
        keys[rng.random(keys.shape[0]) < hot] = 3
    dY = rng.standard_normal((Bn, dim)).astype(np.float32)
    return off, keys, dY


@pytest.mark.parametrize("dim", [4, 16, 64, 128, 256, 512, 1024])
@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("hot", [0.0, 0.5])
def test_bwd_pooled(H, dim, mode, hot):
    import torch
    rng = np.random.default_rng(dim + mode * 5 + int(hot * 10))
    Bn = 3001 if dim <= 128 else 400
    off, keys, dY = _bwd_case(rng, dim, Bn, 11, 2000, hot)
    n = keys.shape[0]
    g, d = H.gpu_dedup(keys, 11)
    unique, inverse, counts, _, _ = H.assert_dedup_equal(g, keys)
    U = unique.shape[0]
    _, _, _, _, uts = H.O.route(unique, 16, 1)
    ref, ab = H.O.lookup_bwd(dY, 0, dim, mode, 1, off, inverse, U, uts, want_abs=True)
    grads = H.B.np_lookup_bwd(H.dev(dY), dim, mode, 1, H.dev(off), n, d["occ_offsets"], d["occ"], d["num_unique"], n,
                              unique_to_send=H.dev(uts))
    torch.cuda.synchronize()
    got = H.host(grads)[:U]
    H.assert_close(got, ref, ab, H.RTOL_F32, f"bwd dim={dim} mode={mode} hot={hot}")
    # deterministic: a second run gives the same bits
    grads2 = H.B.np_lookup_bwd(H.dev(dY), dim, mode, 1, H.dev(off), n, d["occ_offsets"], d["occ"], d["num_unique"], n,
                               unique_to_send=H.dev(uts))
    torch.cuda.synchronize()
    assert H.host(grads2)[:U].tobytes() == got.tobytes()
    if mode == 0:
        # unit gradient: every key receives exactly its multiplicity; unique order when no permutation is given
        ones = torch.ones((Bn, dim), dtype=torch.float32, device="cuda")
        gc = H.B.np_lookup_bwd(ones, dim, 0, 1, H.dev(off), n, d["occ_offsets"], d["occ"], d["num_unique"], n)
        torch.cuda.synchronize()
        assert np.array_equal(H.host(gc)[:U], np.repeat(counts[:, None], dim, 1).astype(np.float32))


@pytest.mark.parametrize("knob", ["bwd_row_index", "bwd_singles_by_bag"])
@pytest.mark.parametrize("dim,mode", [(16, 0), (64, 1), (256, 0), (512, 1), (72, 2), (128, 2)])
def test_bwd_variants_give_the_same_bits(H, knob, dim, mode):
    """np_tune_set switches between ways of doing the same reduction; the gradients must not change by a bit (and are the
    oracle's within tolerance).  Pooled modes with fp32 upstream gradients, sequence mode with bf16 ones; empty bags, a
    popular key, and keys with a single lookup are all present."""
    import torch
    rng = np.random.default_rng(dim * 7 + mode)
    seq = mode == 2
    Bn, R = (97, 900) if seq else (3001, 2500)
    off, keys = _bags(rng, Bn, 300 if seq else 11, R)
    keys[rng.random(keys.shape[0]) < 0.3] = 7
    n = keys.shape[0]
    max_len = int(np.diff(off).max()) if seq else 1
    if seq:
        dY = H.wl.round_to_bf16(rng.standard_normal((Bn, max_len, dim)).astype(np.float32))
        dYd = H.bf16_dev(dY)
        dY_ref, dt = H.host(dYd), 1
    else:
        dY = rng.standard_normal((Bn, dim)).astype(np.float32)
        dYd, dY_ref, dt = H.dev(dY), dY, 0
    g, d = H.gpu_dedup(keys, 12)
    unique, inverse, *_ = H.assert_dedup_equal(g, keys)
    U = unique.shape[0]
    _, _, _, _, uts = H.O.route(unique, 16, 1)
    ref, ab = H.O.lookup_bwd(dY_ref, dt, dim, mode, max_len, off, inverse, U, uts, want_abs=True)
    old = H.B.np_tune_get(knob)
    got = {}
    try:
        for v in (0, 1):
            H.B.np_tune_set(knob, v)
            grads = H.B.np_lookup_bwd(dYd, dim, mode, max_len, H.dev(off), n, d["occ_offsets"], d["occ"], d["num_unique"], n,
                                      unique_to_send=H.dev(uts))
            torch.cuda.synchronize()
            got[v] = H.host(grads)[:U].copy()
    finally:
        H.B.np_tune_set(knob, old)
    assert got[0].tobytes() == got[1].tobytes()
    H.assert_close(got[1], ref, ab, H.RTOL_F32, f"bwd {knob} dim={dim} mode={mode}")


@pytest.mark.parametrize("dim,Bn,mode", [(64, 1_100_000, 0), (1024, 70_000, 1)])
def test_bwd_with_an_upstream_gradient_larger_than_the_last_level_cache(H, dim, Bn, mode):
    """Above 256 MB of dY the backward runs its tiles in the locality order (long segments sorted by relative position,
    one range per die); popular keys give it segments of many tiles to order."""
    import torch
    rng = np.random.default_rng(dim)
    lens = rng.integers(0, 6, size=Bn)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    n = int(off[-1])
    keys = rng.integers(0, 200_000, size=n).astype(np.int64)
    hot = rng.random(n)
    keys[hot < 0.25] = 5
    keys[(hot >= 0.25) & (hot < 0.35)] = 77
    keys[(hot >= 0.35) & (hot < 0.37)] = 4242
    dY = rng.standard_normal((Bn, dim)).astype(np.float32)
    assert dY.nbytes > 256 << 20
    g, d = H.gpu_dedup(keys, 18)
    unique, inverse, counts, _, _ = H.assert_dedup_equal(g, keys)
    U = unique.shape[0]
    assert counts.max() > 100 * 256
    ref, ab = H.O.lookup_bwd(dY, 0, dim, mode, 1, off, inverse, U, None, want_abs=True)
    dYd = H.dev(dY)
    grads = H.B.np_lookup_bwd(dYd, dim, mode, 1, H.dev(off), n, d["occ_offsets"], d["occ"], d["num_unique"], U)
    torch.cuda.synchronize()
    H.assert_close(H.host(grads)[:U], ref, ab, H.RTOL_F32, f"bwd ordered dim={dim}")
    grads2 = H.B.np_lookup_bwd(dYd, dim, mode, 1, H.dev(off), n, d["occ_offsets"], d["occ"], d["num_unique"], U)
    torch.cuda.synchronize()
    assert torch.equal(grads[:U], grads2[:U])
    # the same in two parts: the index work first, the reduction on the prepared workspace
    ws = torch.empty(H.B.np_lookup_bwd_workspace_bytes(Bn, n, dim, mode), dtype=torch.uint8, device="cuda")
    H.B.np_lookup_bwd_prepare(H.B.F32, dim, mode, 1, H.dev(off), n, d["occ_offsets"], d["occ"], d["num_unique"], ws)
    grads3 = H.B.np_lookup_bwd_prepared(dYd, dim, mode, 1, H.dev(off), n, d["occ_offsets"], d["occ"], d["num_unique"], U, ws)
    torch.cuda.synchronize()
    assert torch.equal(grads[:U], grads3[:U])


@pytest.mark.parametrize("dim,mode", [(16, 0), (64, 1), (256, 0), (20, 0), (24, 1), (40, 0), (136, 1)])
def test_bwd_pooled_bf16_upstream_gradient(H, dim, mode):
    """Pooled modes with the upstream gradient stored in bf16 (read exactly, accumulated in fp32)."""
    import torch
    rng = np.random.default_rng(dim * 7 + mode)
    off, keys, dY = _bwd_case(rng, dim, 2500, 13, 3000, 0.3)
    dYb = H.wl.round_to_bf16(dY)
    n = keys.shape[0]
    g, d = H.gpu_dedup(keys, 12)
    unique, inverse, *_ = H.assert_dedup_equal(g, keys)
    U = unique.shape[0]
    dev_dy = H.bf16_dev(dYb)
    ref, ab = H.O.lookup_bwd(H.host(dev_dy), 1, dim, mode, 1, off, inverse, U, None, want_abs=True)
    grads = H.B.np_lookup_bwd(dev_dy, dim, mode, 1, H.dev(off), n, d["occ_offsets"], d["occ"], d["num_unique"], n)
    torch.cuda.synchronize()
    H.assert_close(H.host(grads)[:U], ref, ab, H.RTOL_F32, f"bwd pooled bf16 dY dim={dim} mode={mode}")
    ref32, _ = H.O.lookup_bwd(dYb, 0, dim, mode, 1, off, inverse, U, None)
    assert np.array_equal(ref, ref32)          # the oracle reads bf16 exactly


@pytest.mark.parametrize("dim", [16, 128, 24, 72, 36])
def test_bwd_seq_bf16(H, dim):
    import torch
    rng = np.random.default_rng(dim + 99)
    Bn, R = 97, 900
    off, keys = _bags(rng, Bn, 300, R)
    max_len = int(np.diff(off).max())
    n = keys.shape[0]
    dY = H.wl.round_to_bf16(rng.standard_normal((Bn, max_len, dim)).astype(np.float32))
    dYt = H.bf16_dev(dY)
    bits = H.host(dYt).copy()
    lens = np.diff(off)
    poisoned = bits.copy()
    for b in range(Bn):
        poisoned[b, lens[b]:] = 0x7FC0                                   # NaN in the padding must never be read
    dYp = torch.from_numpy(poisoned.view(np.int16)).cuda().view(torch.bfloat16)
    g, d = H.gpu_dedup(keys, 10)
    unique, inverse, *_ = H.assert_dedup_equal(g, keys)
    U = unique.shape[0]
    ref, ab = H.O.lookup_bwd(bits, 1, dim, 2, max_len, off, inverse, U, None, want_abs=True)
    grads = H.B.np_lookup_bwd(dYp, dim, 2, max_len, H.dev(off), n, d["occ_offsets"], d["occ"], d["num_unique"], n)
    torch.cuda.synchronize()
    H.assert_close(H.host(grads)[:U], ref, ab, H.RTOL_F32, f"bwd seq dim={dim}")


def test_bwd_bf16_gradient_at_an_8_byte_aligned_base(H):
    """A bf16 dY whose base is 8- but not 16-byte aligned takes the 8-byte loads and gives the same bits as the aligned
    copy (which takes the 16-byte ones)."""
    import torch
    dim = 64
    rng = np.random.default_rng(4242)
    off, keys, dY = _bwd_case(rng, dim, 1800, 11, 2500, 0.3)
    n = keys.shape[0]
    g, d = H.gpu_dedup(keys, 12)
    dev_dy = H.bf16_dev(H.wl.round_to_bf16(dY))
    store = torch.zeros(dev_dy.numel() + 16, dtype=torch.bfloat16, device="cuda")
    base = store.data_ptr()
    shift = 4 if base % 16 == 0 else 0                      # elements; 4 bf16 = 8 bytes
    odd = store[shift:shift + dev_dy.numel()].view(dev_dy.shape)
    odd.copy_(dev_dy)
    assert odd.data_ptr() % 16 == 8
    args = (dim, 0, 1, H.dev(off), n, d["occ_offsets"], d["occ"], d["num_unique"], n)
    g_al = H.B.np_lookup_bwd(dev_dy, *args)
    g_odd = H.B.np_lookup_bwd(odd, *args)
    torch.cuda.synchronize()
    U = int(d["num_unique"].item())
    assert torch.equal(g_al[:U], g_odd[:U])


# ------------------------------------------------------------------------------------------ update

@pytest.mark.parametrize("dim", [4, 16, 64, 128, 512, 1024])
def test_adagrad(H, dim):
    import torch
    rng = np.random.default_rng(dim + 1)
    R, U = 20000, 6000
    t0 = (rng.standard_normal((R, dim)) * 0.01).astype(np.float32)
    s0 = (rng.random(R) * 0.1).astype(np.float32)
    s0[::3] = 0
    keys = np.sort(rng.choice(R, size=U, replace=False)).astype(np.int64)
    keys = keys[rng.permutation(U)]
    grads = rng.standard_normal((U, dim)).astype(np.float32)
    grads[5] = 0.0
    s0[keys[5]] = 0.0
    tr, sr = t0.copy(), s0.copy()
    H.O.sparse_adagrad(tr, sr, keys, grads, 0.01, 1e-8)
    tg, sg = H.dev(t0), H.dev(s0)
    gbuf = np.zeros((U + 50, dim), np.float32)
    gbuf[:U] = grads
    kbuf = np.zeros(U + 50, np.int64)
    kbuf[:U] = keys
    H.B.np_sparse_adagrad(tg, sg, H.dev(kbuf), H.dev(gbuf), H.dev(np.array([U], np.int32)), U + 50, 0.01, 1e-8)
    torch.cuda.synchronize()
    tgot, sgot = H.host(tg), H.host(sg)
    delta = np.abs(tr.astype(np.float64) - t0)
    H.assert_close(tgot[keys], tr[keys], np.abs(t0[keys]) + delta[keys], H.RTOL_F32, "updated rows")
    H.assert_close(sgot[keys], sr[keys], np.abs(sr[keys]), H.RTOL_F32, "updated state")
    rest = np.setdiff1d(np.arange(R), keys)
    assert tgot[rest].tobytes() == t0[rest].tobytes() and sgot[rest].tobytes() == s0[rest].tobytes()
    assert tgot[keys[5]].tobytes() == t0[keys[5]].tobytes() and sgot[keys[5]] == 0.0   # zero gradient: no change, no NaN


# ------------------------------------------------------------------------------------------ whole step

def _dense_step_check(H, cfg, steps=2):
    """Runs `steps` consecutive batches through the five calls on a dense table small enough for the oracle.
    Every call is held against the oracle on the same inputs: the integer outputs bit for bit, the forward
    against the table as the previous update left it (the staleness-free read of Proposition 1), the
    gradients against the fp64 sums, and the update against the oracle's update of the same gradient rows."""
    import torch
    R, D = cfg.num_rows, cfg.dim
    table_ref = H.wl.table_init_rows(np.arange(R), D, cfg.table_seed)
    state_ref = np.zeros(R, np.float32)
    table = torch.empty((R, D), dtype=torch.float32, device="cuda")
    H.B.np_util_table_init(table, cfg.table_seed)
    state = torch.zeros(R, dtype=torch.float32, device="cuda")
    prev = None
    seq = cfg.mode == H.wl.SEQ
    dt = H.O.BF16 if seq else H.O.F32
    for t in range(steps):
        batch = H.wl.make_batch(cfg, t, prev=prev)
        prev = batch
        g = H.gpu_step(cfg, batch, table, state)
        dy_ref = H.host(g["dY"]) if seq else batch.dY
        unique, inverse, counts, occ_offsets, occ = H.O.dedup(batch.keys)
        send_keys, splits, send_offsets, sfu, uts = H.O.route(unique, cfg.num_shards, cfg.shard_fn)
        l2s = H.O.compose(inverse, uts)
        ref = dict(unique=unique, inverse=inverse, counts=counts, occ_offsets=occ_offsets, occ=occ, send_keys=send_keys,
                   splits=splits, send_offsets=send_offsets, send_from_unique=sfu, unique_to_send=uts, lookup_to_send=l2s)
        U = H.assert_int_outputs_equal(g, ref, batch.n, cfg.num_shards)
        out_ref, _, ab = H.O.lookup_fwd(table_ref, send_keys, l2s, batch.bag_offsets, cfg.mode, batch.max_len, dt, want_abs=True)
        if seq:
            assert H.host(g["out"]).tobytes() == out_ref.tobytes()
        else:
            H.assert_close(H.host(g["out"]), out_ref, ab, H.RTOL_F32, f"step {t} forward")
        grads_ref, gab = H.O.lookup_bwd(dy_ref, dt, D, cfg.mode, batch.max_len, batch.bag_offsets, inverse, U, uts, want_abs=True)
        grads_gpu = H.host(g["grads"])[:U]
        H.assert_close(grads_gpu, grads_ref, gab, H.RTOL_F32, f"step {t} gradients")
        before_t, before_s = table_ref.copy(), state_ref.copy()
        H.O.sparse_adagrad(table_ref, state_ref, send_keys, grads_gpu, cfg.lr, cfg.eps)
        tg, sg = H.host(table), H.host(state)
        K = unique
        delta = np.abs(table_ref[K].astype(np.float64) - before_t[K])
        H.assert_close(tg[K], table_ref[K], np.abs(before_t[K]) + delta, H.RTOL_F32, f"step {t} updated rows")
        H.assert_close(sg[K], state_ref[K], np.abs(state_ref[K]), H.RTOL_F32, f"step {t} state")
        rest = np.ones(R, bool)
        rest[K] = False
        assert tg[rest].tobytes() == before_t[rest].tobytes()           # Eq. (2): keys outside the batch are untouched
        assert sg[rest].tobytes() == before_s[rest].tobytes()
        assert np.all(np.any(tg[K] != before_t[K], axis=1) | ~np.any(grads_gpu[uts] != 0, axis=1))
        # continue from the GPU's own table so that rounding differences do not leak into the next step's checks
        table_ref[:] = tg
        state_ref[:] = sg


def test_step_tiny_config_two_batches(H):
    """Configuration 1 at full size, two consecutive batches with shared hot keys: lookup -> update -> lookup
    equals the sequential oracle (Proposition 1)."""
    _dense_step_check(H, H.wl.config("tiny"), steps=2)


@pytest.mark.parametrize("name,row_div,batch_div", [("dlrm", 400, 64), ("seq", 4000, 128), ("skew", 4000, 64),
                                                    ("large", 8000, 256)])
def test_step_scaled_configs(H, name, row_div, batch_div):
    _dense_step_check(H, H.wl.scaled(H.wl.config(name), row_div, batch_div), steps=2)


def _random_config(H, rng, case):
    """A small random configuration of the path: every structural parameter drawn independently."""
    wl = H.wl
    mode = int(rng.integers(0, 3))
    dim = int(rng.choice([4, 8, 12, 16, 32, 36, 64, 72, 128, 256, 520]))
    tables = int(rng.integers(1, 4))
    rows = tuple(int(rng.integers(64, 20000)) for _ in range(tables))
    law, args = [("uniform", (1, int(rng.integers(2, 40)))), ("poisson", (int(rng.integers(1, 9)),)),
                 ("fixed", (int(rng.integers(1, 33)),)), ("poisson_clip", (4, 1, 64))][int(rng.integers(0, 4))]
    if mode == wl.SEQ:
        law, args = "seq_uniform", (1, int(rng.integers(2, 60)))
    S = int(rng.choice([1, 2, 7, 8, 64, 100, 1536, 4096]))
    return wl.Config(f"random{case}", 1 + case % 5, rows, dim, int(rng.integers(1, 300)), int(rng.integers(1, 6)), law, args,
                     float(rng.choice([0.0, 0.8, 1.05, 1.5])), S, int(rng.integers(0, 2)), mode, table_seed=100 + case)


@pytest.mark.parametrize("block", range(4))
def test_step_random_small_configurations(H, block):
    """Sixty small configurations with independently drawn modes, widths, table counts, length laws, skews and shard
    counts, two consecutive batches each, every call against the oracle."""
    rng = np.random.default_rng(777 + block)
    for case in range(block * 15, block * 15 + 15):
        cfg = _random_config(H, rng, case)
        H.progress(f"[random step] {cfg}")
        _dense_step_check(H, cfg, steps=2)


@pytest.mark.parametrize("mode", [0, 1, 2])
def test_step_with_no_lookups(H, mode):
    """A batch whose bags are all empty: zero distinct keys, zero splits, zero (or zero-padded) outputs, no gradient
    row written, table and state untouched."""
    import torch
    B = H.B
    Bn, D, S, R, max_len = 300, 32, 16, 500, 3
    keys = torch.empty(0, dtype=torch.int64, device="cuda")
    off = torch.zeros(Bn + 1, dtype=torch.int32, device="cuda")
    table = torch.randn((R, D), device="cuda")
    state = torch.rand(R, device="cuda")
    t0, s0 = table.clone(), state.clone()
    d = B.np_dedup(keys, 9)
    r = B.np_route(d["unique"], d["num_unique"], 0, S, 1, inverse=d["inverse"], n=0)
    dt = B.BF16 if mode == 2 else B.F32
    out = torch.full((Bn, max_len, D) if mode == 2 else (Bn, D), 7.0, dtype=torch.bfloat16 if mode == 2 else torch.float32,
                     device="cuda")
    B.np_lookup_fwd(table, r["send_keys"], r["lookup_to_send"], off, 0, mode, max_len, dt, num_list=d["num_unique"], cap=0, out=out)
    dY = torch.randn(out.shape, device="cuda").to(out.dtype)
    grads = torch.full((4, D), 3.0, device="cuda")
    B.np_lookup_bwd(dY, D, mode, max_len, off, 0, d["occ_offsets"], d["occ"], d["num_unique"], 0,
                    unique_to_send=r["unique_to_send"], grads=grads)
    B.np_sparse_adagrad(table, state, r["send_keys"], grads, d["num_unique"], 0, 0.01, 1e-8)
    B.np_lookup_bwd_adagrad(dY, mode, max_len, off, 0, d["occ_offsets"], d["occ"], d["unique"], d["num_unique"], 0, table, state,
                            0.01, 1e-8)
    torch.cuda.synchronize()
    assert int(d["num_unique"].item()) == 0 and int(d["occ_offsets"][0].item()) == 0
    assert not H.host(r["splits"]).any() and not H.host(r["send_offsets"]).any()
    assert not H.host(out).any()
    assert torch.equal(grads, torch.full((4, D), 3.0, device="cuda"))
    assert torch.equal(table, t0) and torch.equal(state, s0)


@pytest.mark.parametrize("mode", [0, 1])
def test_one_very_long_bag_between_an_empty_and_a_short_one(H, mode):
    """Forward and backward with a 100,000-lookup bag (one group walks it; its mean weight is 1e-5)."""
    import torch
    rng = np.random.default_rng(41 + mode)
    R, D = 3000, 32
    lens = np.array([0, 100_000, 5, 0, 1], np.int64)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    n = int(off[-1])
    keys = rng.integers(0, R, size=n).astype(np.int64)
    keys[-1] = R - 1
    keys[0] = 0
    table = rng.standard_normal((R, D)).astype(np.float32)
    dY = rng.standard_normal((lens.size, D)).astype(np.float32)
    g, d = H.gpu_dedup(keys, 12)
    unique, inverse, *_ = H.assert_dedup_equal(g, keys)
    U = unique.shape[0]
    ref, _, ab = H.O.lookup_fwd(table, unique, inverse, off, mode, want_abs=True)
    out, _ = H.B.np_lookup_fwd(H.dev(table), d["unique"], d["inverse"], H.dev(off), n, mode)
    gref, gab = H.O.lookup_bwd(dY, 0, D, mode, 1, off, inverse, U, None, want_abs=True)
    grads = H.B.np_lookup_bwd(H.dev(dY), D, mode, 1, H.dev(off), n, d["occ_offsets"], d["occ"], d["num_unique"], U)
    torch.cuda.synchronize()
    H.assert_close(H.host(out), ref, ab, H.RTOL_F32, "forward, long bag")
    H.assert_close(H.host(grads)[:U], gref, gab, H.RTOL_F32, "backward, long bag")


@pytest.mark.parametrize("words", [1, 255, 256, 1025, 4096 * 16384 // 16 + 3, (1 << 22) + 777])
def test_stream_copy_yardstick_copies_every_word(H, words):
    """The bandwidth yardstick is a real copy: every 16-byte word arrives, nothing past the end is touched (slabs per
    block with a ragged last slab, a tail shorter than one round of loads)."""
    import torch
    src = torch.arange(words * 4 + 8, dtype=torch.int32, device="cuda")
    dst = torch.full_like(src, -1)
    H.B.np_util_stream_copy(dst[: words * 4], src[: words * 4])
    torch.cuda.synchronize()
    assert torch.equal(dst[: words * 4], src[: words * 4])
    assert bool((dst[words * 4:] == -1).all())


def test_binding_refuses_tensors_of_the_wrong_element_type(H):
    import torch
    B = H.B
    keys32 = torch.arange(100, dtype=torch.int32, device="cuda")
    with pytest.raises(TypeError):
        B.np_dedup(keys32, 10)
    table64 = torch.zeros((8, 4), dtype=torch.float64, device="cuda")
    off = torch.tensor([0, 2], dtype=torch.int32, device="cuda")
    keys = torch.tensor([1, 2], dtype=torch.int64, device="cuda")
    with pytest.raises(TypeError):
        B.np_lookup_fwd(table64, keys, None, off, 2, B.POOL_SUM)
    with pytest.raises(TypeError):
        B.np_lookup_fwd_t(table64, keys, None, off, 2, B.POOL_SUM)
    with pytest.raises(ValueError):
        B.np_dedup(torch.arange(100, dtype=torch.int64), 10)          # host tensor


def test_batch_precondition_check(H):
    import torch
    B = H.B
    rng = np.random.default_rng(77)
    R, nb = 5000, 3000
    lens = rng.integers(0, 9, nb)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    n = int(off[-1])
    keys = rng.integers(0, R, n).astype(np.int64)
    assert B.np_util_check_batch(H.dev(keys), R, H.dev(off)) == (0, 0, 0, 0)
    bad = keys.copy()
    bad[[5, 700, n - 1]] = [-1, R, R + 5]
    assert B.np_util_check_batch(H.dev(bad), R, H.dev(off)) == (3, 0, 0, 0)
    off2 = off.copy()
    off2[100] = off2[101] + 1          # one decreasing step (off2[99] <= off2[100] still holds or not: count both ways)
    want_steps = int(np.sum(np.diff(off2.astype(np.int64)) < 0))
    assert want_steps >= 1
    assert B.np_util_check_batch(H.dev(keys), R, H.dev(off2)) == (0, want_steps, 0, 0)
    off3 = off.copy()
    off3[0] = 1
    off3[-1] = n + 2
    got = B.np_util_check_batch(H.dev(keys), R, H.dev(off3))
    assert got[2] == 1 and got[3] == 1
    assert B.np_util_check_batch(None, R, H.dev(np.zeros(1, np.int32))) == (0, 0, 0, 0)
    assert B.np_util_check_batch(H.dev(keys), R, None)[0] == 0


@pytest.mark.parametrize("dim,mode,bf16", [(4, 0, False), (16, 1, False), (64, 0, False), (64, 1, True), (128, 2, True), (24, 2, True),
                                           (520, 0, False)])
@pytest.mark.parametrize("row_index", [0, 1])
def test_bwd_in_two_parts_equals_the_single_call(H, dim, mode, bf16, row_index):
    """np_lookup_bwd_prepare on a second stream, ordered by an event, then np_lookup_bwd_prepared: the bits of np_lookup_bwd,
    also when the prepared workspace is used for two different gradients in a row; with and without the row index."""
    import torch
    B = H.B
    old = B.np_tune_get("bwd_row_index")
    B.np_tune_set("bwd_row_index", row_index)
    try:
        _two_parts(H, dim, mode, bf16)
    finally:
        B.np_tune_set("bwd_row_index", old)


def _two_parts(H, dim, mode, bf16):
    import torch
    B = H.B
    rng = np.random.default_rng(dim * 3 + mode)
    Bn = 700
    off, keys = _bags(rng, Bn, 40, 3000)
    keys[rng.random(keys.shape[0]) < 0.4] = 11                       # one key with a long chain of tiles
    n = keys.shape[0]
    max_len = int(np.diff(off).max()) if mode == 2 else 1
    shape = (Bn, max_len, dim) if mode == 2 else (Bn, dim)
    g, d = H.gpu_dedup(keys, 12)
    U = int(d["num_unique"].item())
    offd = H.dev(off)
    ws = torch.empty(B.np_lookup_bwd_workspace_bytes(Bn, n, dim, mode), dtype=torch.uint8, device="cuda")
    side = torch.cuda.Stream()
    ready = torch.cuda.Event()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        B.np_lookup_bwd_prepare(B.BF16 if bf16 else B.F32, dim, mode, max_len, offd, n, d["occ_offsets"], d["occ"], d["num_unique"], ws)
        ready.record(side)
    torch.cuda.current_stream().wait_event(ready)
    for rep in range(2):
        dY = torch.from_numpy(rng.standard_normal(shape).astype(np.float32)).cuda()
        if bf16:
            dY = dY.bfloat16()
        want = B.np_lookup_bwd(dY, dim, mode, max_len, offd, n, d["occ_offsets"], d["occ"], d["num_unique"], n)
        got = B.np_lookup_bwd_prepared(dY, dim, mode, max_len, offd, n, d["occ_offsets"], d["occ"], d["num_unique"], n, ws)
        torch.cuda.synchronize()
        assert torch.equal(want[:U], got[:U]), rep


def test_bwd_prepare_checks_its_arguments(H):
    import torch
    B, L = H.B, H.B.lib
    off = torch.tensor([0, 2, 5], dtype=torch.int32, device="cuda")
    oo = torch.tensor([0, 3, 5], dtype=torch.int32, device="cuda")
    nu = torch.tensor([2], dtype=torch.int32, device="cuda")
    oc = torch.tensor([0, 2, 4, 1, 3], dtype=torch.int32, device="cuda")
    need = B.np_lookup_bwd_workspace_bytes(2, 5, 8, 0)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    st = torch.cuda.current_stream().cuda_stream
    assert L.np_lookup_bwd_prepare(0, 8, 0, 1, off.data_ptr(), 2, 5, oo.data_ptr(), oc.data_ptr(), nu.data_ptr(), ws.data_ptr(), need, st) == 0
    assert L.np_lookup_bwd_prepare(0, 8, 0, 1, off.data_ptr(), 2, 5, oo.data_ptr(), oc.data_ptr(), nu.data_ptr(), ws.data_ptr(), need - 1, st) == -2
    assert L.np_lookup_bwd_prepare(0, 6, 0, 1, off.data_ptr(), 2, 5, oo.data_ptr(), oc.data_ptr(), nu.data_ptr(), ws.data_ptr(), need, st) == -3
    assert L.np_lookup_bwd_prepare(7, 8, 0, 1, off.data_ptr(), 2, 5, oo.data_ptr(), oc.data_ptr(), nu.data_ptr(), ws.data_ptr(), need, st) == -1
    assert L.np_lookup_bwd_prepare(0, 8, 0, 1, 0, 2, 5, oo.data_ptr(), oc.data_ptr(), nu.data_ptr(), ws.data_ptr(), need, st) == -1
    assert L.np_lookup_bwd_prepare(0, 8, 0, 1, off.data_ptr(), 2, 0, oo.data_ptr(), oc.data_ptr(), nu.data_ptr(), 0, 0, st) == 0     # no lookups
    assert L.np_lookup_bwd_prepare(0, 8, 0, 1, off.data_ptr(), 2, 5, oo.data_ptr(), 0, nu.data_ptr(), ws.data_ptr(), need, st) == -1    # no occ
    torch.cuda.synchronize()
