"""GPU parity of the 16-bit-table variants, bf16 and fp16 (np_lookup_fwd_t, np_sparse_adagrad_t, the dtype-generic
harness calls) against the CPU oracle.  Reading a 16-bit row is exact, so forward results carry the fp32 bar (1e-5
against the sum of absolute terms; copies bit exact).  An updated row is a value rounded to the storage format: the bar
is 1e-2 for bf16 (the stated one) and 2e-3 for fp16 (two of its 2^-10 spacings), and on top of it all but a tiny
fraction of the elements must carry the oracle's bit pattern, the others the pattern next to it (the two sides round
values that agree to fp32 precision, so they part only where such a value sits on a rounding boundary)."""
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


class _Kind:
    """One 16-bit storage format: conversions through library routines (torch / numpy), the oracle's entry points."""

    def __init__(self, name):
        import torch
        self.name = name
        self.torch_dtype = torch.bfloat16 if name == "bf16" else torch.float16
        self.rtol = 1e-2 if name == "bf16" else 2e-3

    def to_bits(self, a):
        import torch
        a = np.ascontiguousarray(a, np.float32)
        if self.name == "bf16":
            return torch.from_numpy(a).bfloat16().view(torch.int16).numpy().view(np.uint16).copy()
        return a.astype(np.float16).view(np.uint16).copy()

    def widen(self, bits):
        if self.name == "bf16":
            return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)
        return bits.view(np.float16).astype(np.float32)

    def dev(self, bits):
        import torch
        return torch.from_numpy(bits.view(np.int16)).cuda().view(self.torch_dtype)

    def oracle_table(self, bits):
        return bits if self.name == "bf16" else bits.view(np.float16)

    def oracle_adagrad(self, O):
        return O.sparse_adagrad_bf16 if self.name == "bf16" else O.sparse_adagrad_f16


@pytest.fixture(params=["bf16", "f16"])
def K(request):
    return _Kind(request.param)


def _host_bits(t):
    import torch
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def _assert_rows(H, K, got_bits, ref_bits, scale, what):
    got, ref = K.widen(got_bits), K.widen(ref_bits)
    H.assert_close(got, ref, scale, K.rtol, what)
    diff = got_bits != ref_bits
    frac = float(diff.mean()) if diff.size else 0.0
    assert frac < 2e-3, f"{what}: {frac:.2e} of the elements differ from the oracle's bit pattern"
    # away from cancellation (result not much smaller than its terms) a differing element is the neighbouring pattern
    big = diff & (np.abs(ref) > 0.05 * scale)
    if big.any():
        step = np.abs(got_bits[big].astype(np.int32) - ref_bits[big].astype(np.int32))
        assert step.max() == 1, f"{what}: a differing element is {step.max()} patterns away"


def _bags(rng, B, max_l, R):
    lens = rng.integers(0, max_l + 1, size=B)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    keys = rng.integers(0, R, size=int(off[-1])).astype(np.int64)
    return off, keys


def test_table_init_is_the_rounded_generator(H, K):
    import torch
    for R, D in ((1000, 16), (777, 64), (50, 128), (3, 4)):
        t = torch.empty((R, D), dtype=K.torch_dtype, device="cuda")
        H.B.np_util_table_init_t(t, 7)
        ref = K.to_bits(H.wl.table_init_rows(np.arange(R), D, 7))
        assert np.array_equal(_host_bits(t), ref)
        assert H.B.np_util_table_count_changed_t(t, 7) == 0
        t[R // 2, D - 1] = 1.0
        t[0, 0] = 1.0
        assert H.B.np_util_table_count_changed_t(t, 7) == (2 if R // 2 != 0 else 1)
    t32 = torch.empty((100, 8), dtype=torch.float32, device="cuda")
    H.B.np_util_table_init_t(t32, 9)
    assert H.host(t32).tobytes() == H.wl.table_init_rows(np.arange(100), 8, 9).tobytes()


@pytest.mark.parametrize("dim", [4, 8, 16, 48, 64, 128, 256, 512, 1024])
@pytest.mark.parametrize("mode", [0, 1])
def test_fwd_pooled_16bit_table(H, K, dim, mode):
    import torch
    rng = np.random.default_rng(dim * 5 + mode)
    R, Bn = 3000, 1237
    tbits = K.to_bits(rng.standard_normal((R, dim)))
    off, keys = _bags(rng, Bn, 70 if dim <= 128 else 9, R)
    unique, inverse, *_ = H.O.dedup(keys)
    ref, _, ab = H.O.lookup_fwd(K.oracle_table(tbits), unique, inverse, off, mode, want_abs=True)
    tab = K.dev(tbits)
    out, _ = H.B.np_lookup_fwd_t(tab, H.dev(unique), H.dev(inverse), H.dev(off), keys.shape[0], mode)
    torch.cuda.synchronize()
    H.assert_close(H.host(out), ref, ab, H.RTOL_F32, f"fwd pooled {K.name} table dim={dim} mode={mode}")
    assert not H.host(out)[np.diff(off) == 0].any()
    out2, _ = H.B.np_lookup_fwd_t(tab, H.dev(keys), None, H.dev(off), keys.shape[0], mode)
    torch.cuda.synchronize()
    assert H.host(out2).tobytes() == H.host(out).tobytes()
    # the same table widened to fp32 goes through the fp32 kernels to the same bits: only the row read differs
    out3, _ = H.B.np_lookup_fwd(tab.float(), H.dev(unique), H.dev(inverse), H.dev(off), keys.shape[0], mode)
    torch.cuda.synchronize()
    assert H.host(out3).tobytes() == H.host(out).tobytes()


@pytest.mark.parametrize("dim", [16, 128, 512])
def test_fwd_seq_and_rows_out_16bit_table_bit_exact(H, K, dim):
    import torch
    rng = np.random.default_rng(dim + 11)
    R, Bn = 5000, 211
    tbits = K.to_bits(rng.standard_normal((R, dim)))
    off, keys = _bags(rng, Bn, 37, R)
    max_len = int(np.diff(off).max())
    unique, inverse, *_ = H.O.dedup(keys)
    U = unique.shape[0]
    tab = K.dev(tbits)
    for dt in (H.B.BF16, H.B.F32):
        ref, rows, _ = H.O.lookup_fwd(K.oracle_table(tbits), unique, inverse, off, 2, max_len, dt, want_rows=True)
        out = torch.full((Bn, max_len, dim), 7.0, dtype=torch.bfloat16 if dt == H.B.BF16 else torch.float32, device="cuda")
        out, rows_g = H.B.np_lookup_fwd_t(tab, H.dev(unique), H.dev(inverse), H.dev(off), keys.shape[0], 2, max_len, dt,
                                          num_list=H.dev(np.array([U], np.int32)), cap=U + 5, want_rows=True, out=out)
        torch.cuda.synchronize()
        assert H.host(out).tobytes() == ref.tobytes()
        assert rows_g.dtype == K.torch_dtype
        assert np.array_equal(K.widen(_host_bits(rows_g)[:U]), rows)


@pytest.mark.parametrize("dim", [4, 16, 64, 128, 512, 1024])
def test_adagrad_16bit_table(H, K, dim):
    import torch
    rng = np.random.default_rng(dim + 3)
    R, U = 20000, 6000
    t0 = K.to_bits(rng.standard_normal((R, dim)) * 0.01)
    s0 = (rng.random(R) * 0.1).astype(np.float32)
    s0[::3] = 0
    keys = rng.permutation(np.sort(rng.choice(R, size=U, replace=False))).astype(np.int64)
    grads = rng.standard_normal((U, dim)).astype(np.float32)
    grads[5] = 0.0
    s0[keys[5]] = 0.0
    tr, sr = t0.copy(), s0.copy()
    K.oracle_adagrad(H.O)(tr, sr, keys, grads, 0.01, 1e-8)
    tg, sg = K.dev(t0), H.dev(s0)
    gbuf = np.zeros((U + 50, dim), np.float32)
    gbuf[:U] = grads
    kbuf = np.zeros(U + 50, np.int64)
    kbuf[:U] = keys
    H.B.np_sparse_adagrad_t(tg, sg, H.dev(kbuf), H.dev(gbuf), H.dev(np.array([U], np.int32)), U + 50, 0.01, 1e-8)
    torch.cuda.synchronize()
    tgot, sgot = _host_bits(tg), H.host(sg)
    w0 = K.widen(t0).astype(np.float64)
    delta = np.abs(K.widen(tr).astype(np.float64) - w0)
    _assert_rows(H, K, tgot[keys], tr[keys], np.abs(w0[keys]) + delta[keys], f"updated {K.name} rows dim={dim}")
    H.assert_close(sgot[keys], sr[keys], np.abs(sr[keys]), H.RTOL_F32, "updated state")
    rest = np.setdiff1d(np.arange(R), keys)
    assert np.array_equal(tgot[rest], t0[rest]) and sgot[rest].tobytes() == s0[rest].tobytes()
    assert np.array_equal(tgot[keys[5]], t0[keys[5]]) and sgot[keys[5]] == 0.0


@pytest.mark.parametrize("dim", [8, 64, 512])
def test_fused_bwd_adagrad_16bit_table_against_the_oracle(H, K, dim):
    """np_lookup_bwd_adagrad_t on a 16-bit table held against the oracle directly (not through the separate HIP calls):
    oracle gradient sums, then the oracle's 16-bit update.  The upstream gradients are small integers, so the fp32 sums
    are exact and the update on both sides starts from the same gradient rows; what remains is the update's own rounding."""
    import torch
    rng = np.random.default_rng(dim + 5)
    R, Bn = 4000, 2501
    off, keys = _bags(rng, Bn, 9, R)
    keys[rng.random(keys.shape[0]) < 0.35] = 17                       # one key with a long occurrence list
    n = keys.shape[0]
    t0 = K.to_bits(rng.standard_normal((R, dim)) * 0.01)
    s0 = (rng.random(R) * 0.1).astype(np.float32)
    dY = rng.integers(-6, 7, size=(Bn, dim)).astype(np.float32)
    unique, inverse, *_ = H.O.dedup(keys)
    U = unique.size
    grads, _ = H.O.lookup_bwd(dY, H.O.F32, dim, 0, 1, off, inverse, U)
    tr, sr = t0.copy(), s0.copy()
    K.oracle_adagrad(H.O)(tr, sr, unique, grads, 0.01, 1e-8)
    tg, sg = K.dev(t0), H.dev(s0)
    d = H.B.np_dedup(H.dev(keys), 12)
    H.B.np_lookup_bwd_adagrad_t(H.dev(dY), 0, 1, H.dev(off), n, d["occ_offsets"], d["occ"], d["unique"], d["num_unique"], n, tg, sg,
                                0.01, 1e-8)
    torch.cuda.synchronize()
    assert int(d["num_unique"].item()) == U
    tgot, sgot = _host_bits(tg), H.host(sg)
    w0 = K.widen(t0).astype(np.float64)
    delta = np.abs(K.widen(tr).astype(np.float64) - w0)
    _assert_rows(H, K, tgot[unique], tr[unique], np.abs(w0[unique]) + delta[unique], f"fused update of {K.name} rows dim={dim}")
    H.assert_close(sgot[unique], sr[unique], np.abs(sr[unique]), H.RTOL_F32, "updated state")
    rest = np.setdiff1d(np.arange(R), unique)
    assert np.array_equal(tgot[rest], t0[rest]) and sgot[rest].tobytes() == s0[rest].tobytes()


def test_bad_table_dtype_and_alignment_are_refused(H):
    import torch
    t = torch.zeros((16, 8), dtype=torch.bfloat16, device="cuda")
    s = torch.zeros(16, dtype=torch.float32, device="cuda")
    k = torch.zeros(4, dtype=torch.int64, device="cuda")
    off = torch.tensor([0, 2, 4], dtype=torch.int32, device="cuda")
    g = torch.zeros((4, 8), dtype=torch.float32, device="cuda")
    one = torch.ones(1, dtype=torch.int32, device="cuda")
    L = H.B.lib
    st = torch.cuda.current_stream().cuda_stream
    out = torch.zeros((2, 8), dtype=torch.float32, device="cuda")
    args = (16, 8, k.data_ptr(), 0, 0, 0, off.data_ptr(), 2, 4, 0, 1, 0, out.data_ptr(), 0, 0, 0, st)
    assert L.np_lookup_fwd_t(t.data_ptr(), 7, *args) == -1
    assert L.np_lookup_fwd_t(t.data_ptr() + 2, 1, *args) == -1
    assert L.np_lookup_fwd_t(t.data_ptr() + 4, 2, *args) == -1
    assert L.np_lookup_fwd_t(t.data_ptr(), 1, *args) == 0
    assert L.np_lookup_fwd_t(t.data_ptr(), 2, *args) == 0
    assert L.np_sparse_adagrad_t(t.data_ptr(), 5, s.data_ptr(), 16, 8, k.data_ptr(), g.data_ptr(), one.data_ptr(), 1, 0.01, 1e-8,
                                 st) == -1
    assert L.np_sparse_adagrad_t(t.data_ptr() + 4, 1, s.data_ptr(), 16, 8, k.data_ptr(), g.data_ptr(), one.data_ptr(), 1, 0.01,
                                 1e-8, st) == -1
    assert L.np_util_table_init_t(t.data_ptr(), 3, 16, 8, 1, st) == -1
    torch.cuda.synchronize()
    assert not H.host(out).any() and not H.host(t).any()


def _step_16bit(H, K, cfg, steps):
    """`steps` consecutive batches through dedup -> route -> np_lookup_fwd_t -> np_lookup_bwd -> np_sparse_adagrad_t on a
    16-bit table.  Each call is held against the oracle on the inputs the GPU call had (the rows the GPU holds before the
    step), so rounding differences do not leak from one step into the next."""
    import torch
    wl, O, B = H.wl, H.O, H.B
    R, D, S = cfg.num_rows, cfg.dim, cfg.num_shards
    seq = cfg.mode == wl.SEQ
    dt = O.BF16 if seq else O.F32
    table = torch.empty((R, D), dtype=K.torch_dtype, device="cuda")
    B.np_util_table_init_t(table, cfg.table_seed)
    state = torch.zeros(R, dtype=torch.float32, device="cuda")
    prev = None
    touched = np.empty(0, np.int64)
    for t in range(steps):
        batch = wl.make_batch(cfg, t, prev=prev)
        prev = batch
        n, max_len = batch.n, batch.max_len
        keys_d, off_d = H.dev(batch.keys), H.dev(batch.bag_offsets)
        dY = H.bf16_dev(batch.dY) if seq else H.dev(batch.dY)
        unique, inverse, *_ = O.dedup(batch.keys)
        U = unique.shape[0]
        send_keys, _, _, sfu, uts = O.route(unique, S, cfg.shard_fn)
        l2s = O.compose(inverse, uts)
        rows_before = _host_bits(table[H.dev(unique)])       # [U, D] bit patterns as the GPU holds them, compact
        state_before = H.host(state[H.dev(unique)])
        d = B.np_dedup(keys_d, cfg.key_bits)
        r = B.np_route(d["unique"], d["num_unique"], n, S, cfg.shard_fn, inverse=d["inverse"], n=n)
        out, _ = B.np_lookup_fwd_t(table, r["send_keys"], r["lookup_to_send"], off_d, n, cfg.mode, max_len,
                                   B.BF16 if seq else B.F32, num_list=d["num_unique"], cap=n)
        grads = B.np_lookup_bwd(dY, D, cfg.mode, max_len, off_d, n, d["occ_offsets"], d["occ"], d["num_unique"], n,
                                unique_to_send=r["unique_to_send"])
        B.np_sparse_adagrad_t(table, state, r["send_keys"], grads, d["num_unique"], n, cfg.lr, cfg.eps)
        torch.cuda.synchronize()
        assert int(d["num_unique"].item()) == U and np.array_equal(H.host(r["send_keys"])[:U], send_keys)
        list_c = sfu.astype(np.int64)                         # send slot -> row of the compact table
        out_ref, _, ab = O.lookup_fwd(K.oracle_table(rows_before), list_c, l2s, batch.bag_offsets, cfg.mode, max_len, dt, want_abs=not seq)
        if seq:
            assert H.host(out).tobytes() == out_ref.tobytes()
        else:
            H.assert_close(H.host(out), out_ref, ab, H.RTOL_F32, f"{cfg.name} step {t} forward ({K.name} table)")
        g_gpu = H.host(grads)[:U]
        rows_ref, state_ref = rows_before.copy(), state_before.copy()
        K.oracle_adagrad(O)(rows_ref, state_ref, list_c, g_gpu, cfg.lr, cfg.eps)
        rows_after = _host_bits(table[H.dev(unique)])
        w0 = K.widen(rows_before).astype(np.float64)
        delta = np.abs(K.widen(rows_ref).astype(np.float64) - w0)
        _assert_rows(H, K, rows_after, rows_ref, np.abs(w0) + delta, f"{cfg.name} step {t} updated {K.name} rows")
        H.assert_close(H.host(state[H.dev(unique)]), state_ref, np.abs(state_ref), H.RTOL_F32, f"{cfg.name} step {t} state")
        # rows outside the batches keep their bits, everywhere in the table
        touched = np.union1d(touched, unique)
        rows_all = _host_bits(table[H.dev(touched)])
        init_all = K.to_bits(wl.table_init_rows(touched, D, cfg.table_seed))
        changed = int(np.any(rows_all != init_all, axis=1).sum())
        assert B.np_util_table_count_changed_t(table, cfg.table_seed) == changed
        assert changed > 0.5 * touched.size
        H.progress(f"[{cfg.name} {K.name} table] step {t}: U={U} ok")


def test_step_tiny_16bit_table(H, K):
    _step_16bit(H, K, H.wl.config("tiny"), steps=2)


@pytest.mark.parametrize("name,row_div,batch_div", [("dlrm", 64, 16), ("seq", 256, 64), ("skew", 128, 16), ("large", 2048, 64)])
def test_step_scaled_configs_16bit_table(H, K, name, row_div, batch_div):
    _step_16bit(H, K, H.wl.scaled(H.wl.config(name), row_div, batch_div), steps=2)


@pytest.mark.timeout(900)
@pytest.mark.parametrize("kind", ["bf16", "f16"])
def test_full_large_16bit_table_one_batch(H, kind):
    """Configuration 5 at full size with the table in 16 bits (102 GB)."""
    _step_16bit(H, _Kind(kind), H.wl.config("large"), steps=1)
