"""The fused backward + update entry point (np_lookup_bwd_adagrad) against the two separate calls: the same
sums in the same order and the same update arithmetic, so table and state must come out bit-identical; and
against the oracle within tolerance."""
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


def _run_both(H, table0, state0, keys, off, dY, mode, max_len, key_bits):
    import torch
    B = H.B
    D = table0.shape[1]
    n = keys.shape[0]
    kd, od = H.dev(keys), H.dev(off)
    d = B.np_dedup(kd, key_bits)
    torch.cuda.synchronize()
    U = int(d["num_unique"].item())
    t1, s1 = H.dev(table0), H.dev(state0)
    g = B.np_lookup_bwd(dY, D, mode, max_len, od, n, d["occ_offsets"], d["occ"], d["num_unique"], U)
    B.np_sparse_adagrad(t1, s1, d["unique"], g, d["num_unique"], U, 0.01, 1e-8)
    t2, s2 = H.dev(table0), H.dev(state0)
    B.np_lookup_bwd_adagrad(dY, mode, max_len, od, n, d["occ_offsets"], d["occ"], d["unique"], d["num_unique"], U, t2, s2, 0.01, 1e-8)
    torch.cuda.synchronize()
    return t1, s1, t2, s2, d, U, g


@pytest.mark.parametrize("dim", [4, 16, 48, 64, 128, 256, 260, 512, 768, 1024])
@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("hot", [0.0, 0.6])
def test_fused_equals_separate_calls_bitwise(H, dim, mode, hot):
    import torch
    rng = np.random.default_rng(dim + 7 * mode + int(hot * 10))
    R, Bn = 5000, 4001
    lens = rng.integers(0, 12, size=Bn)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    keys = rng.integers(0, R, size=int(off[-1])).astype(np.int64)
    if hot > 0:
        keys[rng.random(keys.shape[0]) < hot] = 11
    table0 = (rng.standard_normal((R, dim)) * 0.01).astype(np.float32)
    state0 = (rng.random(R) * 0.1).astype(np.float32)
    dY = H.dev(rng.standard_normal((Bn, dim)).astype(np.float32))
    t1, s1, t2, s2, d, U, g = _run_both(H, table0, state0, keys, off, dY, mode, 1, 13)
    assert torch.equal(t1, t2) and torch.equal(s1, s2)
    assert not torch.equal(t1, H.dev(table0))
    # and the oracle, from the GPU's own gradient rows
    tr, sr = table0.copy(), state0.copy()
    unique = H.host(d["unique"])[:U]
    H.O.sparse_adagrad(tr, sr, unique, H.host(g)[:U], 0.01, 1e-8)
    delta = np.abs(tr[unique].astype(np.float64) - table0[unique])
    H.assert_close(H.host(t2)[unique], tr[unique], np.abs(table0[unique]) + delta, H.RTOL_F32, "fused update")
    rest = np.setdiff1d(np.arange(R), unique)
    assert H.host(t2)[rest].tobytes() == table0[rest].tobytes() and H.host(s2)[rest].tobytes() == state0[rest].tobytes()


@pytest.mark.parametrize("kind", ["bf16", "f16"])
@pytest.mark.parametrize("dim,mode", [(8, 0), (64, 1), (256, 0), (512, 1), (1024, 0)])
def test_fused_on_16bit_tables_equals_separate_calls_bitwise(H, kind, dim, mode):
    """np_lookup_bwd_adagrad_t on a bf16 / fp16 table against np_lookup_bwd + np_sparse_adagrad_t: same bits."""
    import torch
    B = H.B
    tdt = torch.bfloat16 if kind == "bf16" else torch.float16
    rng = np.random.default_rng(dim * 3 + mode + (kind == "f16"))
    R, Bn = 5000, 3001
    lens = rng.integers(0, 12, size=Bn)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    keys = rng.integers(0, R, size=int(off[-1])).astype(np.int64)
    keys[rng.random(keys.shape[0]) < 0.4] = 11
    n = keys.shape[0]
    table0 = torch.from_numpy((rng.standard_normal((R, dim)) * 0.01).astype(np.float32)).to(tdt).cuda()
    state0 = H.dev((rng.random(R) * 0.1).astype(np.float32))
    dY = H.dev(rng.standard_normal((Bn, dim)).astype(np.float32))
    od = H.dev(off)
    d = B.np_dedup(H.dev(keys), 13)
    torch.cuda.synchronize()
    U = int(d["num_unique"].item())
    t1, s1 = table0.clone(), state0.clone()
    g = B.np_lookup_bwd(dY, dim, mode, 1, od, n, d["occ_offsets"], d["occ"], d["num_unique"], U)
    B.np_sparse_adagrad_t(t1, s1, d["unique"], g, d["num_unique"], U, 0.01, 1e-8)
    t2, s2 = table0.clone(), state0.clone()
    B.np_lookup_bwd_adagrad_t(dY, mode, 1, od, n, d["occ_offsets"], d["occ"], d["unique"], d["num_unique"], U, t2, s2, 0.01, 1e-8)
    torch.cuda.synchronize()
    assert torch.equal(t1.view(torch.int16), t2.view(torch.int16)) and torch.equal(s1, s2)
    assert not torch.equal(t1.view(torch.int16), table0.view(torch.int16))


def test_fused_with_an_upstream_gradient_larger_than_the_last_level_cache(H):
    """The locality-ordered tile schedule (dY above 256 MB) with the fused sink: still the bits of the separate calls."""
    import torch
    rng = np.random.default_rng(9)
    R, Bn, dim = 200_000, 1_100_000, 64
    lens = rng.integers(0, 6, size=Bn)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    keys = rng.integers(0, R, size=int(off[-1])).astype(np.int64)
    keys[rng.random(keys.shape[0]) < 0.3] = 5
    table0 = (rng.standard_normal((R, dim)) * 0.01).astype(np.float32)
    state0 = np.zeros(R, np.float32)
    dY = H.dev(rng.standard_normal((Bn, dim)).astype(np.float32))
    assert dY.numel() * 4 > 256 << 20
    t1, s1, t2, s2, *_ = _run_both(H, table0, state0, keys, off, dY, 0, 1, 18)
    assert torch.equal(t1, t2) and torch.equal(s1, s2)
    assert not torch.equal(t1, H.dev(table0))


def test_fused_sequence_mode_bf16(H):
    import torch
    rng = np.random.default_rng(5)
    R, Bn, dim = 800, 61, 128
    lens = rng.integers(0, 200, size=Bn)
    max_len = int(lens.max())
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    keys = rng.integers(0, R, size=int(off[-1])).astype(np.int64)
    table0 = (rng.standard_normal((R, dim)) * 0.01).astype(np.float32)
    state0 = np.zeros(R, np.float32)
    dY = H.bf16_dev(H.wl.round_to_bf16(rng.standard_normal((Bn, max_len, dim)).astype(np.float32)))
    t1, s1, t2, s2, *_ = _run_both(H, table0, state0, keys, off, dY, 2, max_len, 10)
    assert torch.equal(t1, t2) and torch.equal(s1, s2)


def test_fused_scaled_large_config(H):
    import torch
    cfg = H.wl.scaled(H.wl.config("large"), 2000, 64)
    batch = H.wl.make_batch(cfg, 0)
    table0 = H.wl.table_init_rows(np.arange(cfg.num_rows), cfg.dim, cfg.table_seed)
    state0 = np.zeros(cfg.num_rows, np.float32)
    t1, s1, t2, s2, *_ = _run_both(H, table0, state0, batch.keys, batch.bag_offsets, H.dev(batch.dY), cfg.mode, 1, cfg.key_bits)
    assert torch.equal(t1, t2) and torch.equal(s1, s2)


def test_fused_rejects_rows_wider_than_the_library_takes(H):
    import torch
    t = torch.zeros((10, 2048), device="cuda")
    s = torch.zeros(10, device="cuda")
    z = torch.zeros(4, dtype=torch.int32, device="cuda")
    with pytest.raises(H.B.NestPipeError) as e:
        H.B.np_lookup_bwd_adagrad(torch.zeros((1, 2048), device="cuda"), 0, 1, z[:2], 1, z, z, torch.zeros(4, dtype=torch.int64, device="cuda"),
                                  z[:1], 1, t, s, 0.01, 1e-8)
    assert e.value.status == -3
