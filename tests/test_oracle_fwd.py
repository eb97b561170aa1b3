"""Pins for the oracle's forward lookup (Section IV-A: the vectors indexed by the deduplicated keys
are read from the table, and each requester ends up with the vector of every lookup of its batch)."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F


def _case(seed, R=200, D=8, B=37, maxL=9, allow_empty=True):
    rng = np.random.default_rng(seed)
    table = rng.standard_normal((R, D)).astype(np.float32)
    lens = rng.integers(0 if allow_empty else 1, maxL + 1, size=B)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    keys = rng.integers(0, R, size=int(off[-1])).astype(np.int64)
    return table, off, keys


def _brute(table, list_keys, idx, off, mode, max_len):
    B = len(off) - 1
    D = table.shape[1]
    out = [[[0.0] * D for _ in range(max_len)] for _ in range(B)] if mode == 2 else [[0.0] * D for _ in range(B)]
    for b in range(B):
        L = off[b + 1] - off[b]
        for p in range(L):
            j = off[b] + p
            row = list_keys[idx[j] if idx is not None else j]
            for d in range(D):
                v = float(table[row][d])
                if mode == 2:
                    out[b][p][d] = v
                else:
                    out[b][d] += v
        if mode == 1 and L > 0:
            for d in range(D):
                out[b][d] /= L
    return np.array(out, dtype=np.float64)


@pytest.mark.parametrize("mode", [0, 1])
def test_pooled_brute_force_and_embedding_bag(oracle, mode):
    table, off, keys = _case(1 + mode)
    out, _, ab = oracle.lookup_fwd(table, keys, None, off, mode, want_abs=True)
    ref = _brute(table, keys, None, off, mode, 1)
    assert np.allclose(out, ref.astype(np.float32), rtol=0, atol=1e-6)
    # library routine: CPU embedding_bag with offsets
    tb = F.embedding_bag(torch.from_numpy(keys), torch.from_numpy(table).double(),
                         torch.from_numpy(off[:-1].astype(np.int64)), mode="sum" if mode == 0 else "mean")
    assert np.allclose(out, tb.numpy(), rtol=1e-6, atol=1e-7)
    # abs_out is the pooled |value|
    ta = F.embedding_bag(torch.from_numpy(keys), torch.from_numpy(np.abs(table)).double(),
                         torch.from_numpy(off[:-1].astype(np.int64)), mode="sum" if mode == 0 else "mean")
    assert np.allclose(ab, ta.numpy(), rtol=1e-12, atol=0)
    # empty bags give zeros
    empty = np.diff(off) == 0
    assert empty.any() and not out[empty].any()


def test_dedup_path_equals_direct_path_bitwise(oracle):
    table, off, keys = _case(5)
    unique, inverse, *_ = oracle.dedup(keys)
    send_keys, _, _, _, uts = oracle.route(unique, 8, oracle.SHARD_HASH)
    l2s = oracle.compose(inverse, uts)
    for mode in (0, 1):
        a, _, _ = oracle.lookup_fwd(table, keys, None, off, mode)
        b, _, _ = oracle.lookup_fwd(table, unique, inverse, off, mode)
        c, _, _ = oracle.lookup_fwd(table, send_keys, l2s, off, mode)
        assert a.tobytes() == b.tobytes() == c.tobytes()


def test_closed_forms(oracle):
    _, off, keys = _case(7, R=50)
    ones = np.ones((50, 4), np.float32)
    lens = np.diff(off)
    s, _, _ = oracle.lookup_fwd(ones, keys, None, off, 0)
    assert np.array_equal(s, np.repeat(lens[:, None], 4, 1).astype(np.float32))
    m, _, _ = oracle.lookup_fwd(ones, keys, None, off, 1)
    assert np.array_equal(m, np.repeat((lens > 0)[:, None], 4, 1).astype(np.float32))
    ramp = np.repeat(np.arange(50, dtype=np.float32)[:, None], 4, 1)        # table[r, d] = r
    s, _, _ = oracle.lookup_fwd(ramp, keys, None, off, 0)
    expect = np.array([keys[off[b]:off[b + 1]].sum() for b in range(len(lens))], dtype=np.float32)
    assert np.array_equal(s[:, 0], expect) and np.array_equal(s[:, 3], expect)
    # a key repeated inside one bag counts every time
    out, _, _ = oracle.lookup_fwd(ramp, np.array([4, 4, 4], np.int64), None, np.array([0, 3], np.int32), 0)
    assert out[0, 0] == 12.0


def test_seq_mode_bit_exact_bf16_and_padding(oracle):
    table, off, keys = _case(9, R=300, D=16, B=11, maxL=7, allow_empty=True)
    max_len = int(np.diff(off).max())
    unique, inverse, *_ = oracle.dedup(keys)
    out, rows, _ = oracle.lookup_fwd(table, unique, inverse, off, 2, max_len, oracle.BF16, want_rows=True)
    assert out.dtype == np.uint16 and out.shape == (11, max_len, 16)
    emb = F.embedding(torch.from_numpy(keys), torch.from_numpy(table)).bfloat16()      # library rounding
    for b in range(11):
        L = off[b + 1] - off[b]
        got = torch.from_numpy(out[b, :L].astype(np.int16)).view(torch.bfloat16)
        assert torch.equal(got, emb[off[b]:off[b + 1]])
        assert not out[b, L:].any()                                                 # padding is exactly zero
    assert rows.tobytes() == table[unique].tobytes()                                # rows_out is a bit copy
    # fp32 sequence output is a bit copy of the rows
    out32, _, _ = oracle.lookup_fwd(table, unique, inverse, off, 2, max_len, oracle.F32)
    ref = _brute(table, unique, inverse, off, 2, max_len).astype(np.float32)
    assert out32.tobytes() == ref.tobytes()


def test_bf16_rounding_cases(oracle):
    # ties to even, carry into the exponent, subnormals, infinities, signed zero
    cases = {0x3F800000: 0x3F80, 0x3F808000: 0x3F80, 0x3F818000: 0x3F82, 0x3F808001: 0x3F81,
             0x3FFFFFFF: 0x4000, 0x7F7FFFFF: 0x7F80, 0x00000001: 0x0000, 0x00008000: 0x0000,
             0x00018000: 0x0002, 0x80000000: 0x8000, 0x7F800000: 0x7F80, 0xFF800000: 0xFF80}
    for bits, want in cases.items():
        x = np.array([bits], np.uint32).view(np.float32)[0]
        assert oracle.f32_to_bf16(float(x)) == want, hex(bits)
        t = torch.tensor([x], dtype=torch.float32).bfloat16().view(torch.int16).item() & 0xFFFF
        assert t == want
    rng = np.random.default_rng(0)
    xs = rng.standard_normal(2000).astype(np.float32) * np.float32(10.0) ** rng.integers(-30, 30, 2000).astype(np.float32)
    got = oracle.f32_to_bf16_bits(xs)
    ref = torch.from_numpy(xs).bfloat16().view(torch.int16).numpy().astype(np.uint16)
    assert np.array_equal(got, ref)
    assert oracle.bf16_to_f32(0x3F80) == 1.0 and oracle.bf16_to_f32(0xC000) == -2.0


def test_bad_inputs_are_rejected(oracle):
    table, off, keys = _case(3)
    bad = keys.copy()
    bad[0] = table.shape[0]
    with pytest.raises(RuntimeError):
        oracle.lookup_fwd(table, bad, None, off, 0)
    with pytest.raises(RuntimeError):
        oracle.lookup_fwd(table, keys, None, off, 2, 1, oracle.F32)      # a bag longer than max_len
