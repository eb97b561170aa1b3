"""Pins for the oracle's bf16-table variant: one-step rounding from fp64 to bf16, the exact read of a bf16 row in the
forward pass, and the row-wise Adagrad step that stores bf16 (Section IV-B applies gradients to the stored vectors;
the storage precision is a variant of this build, not of the paper)."""
from fractions import Fraction

import numpy as np
import torch


def _bf16_value(bits: int) -> Fraction:
    """Exact value of a finite bf16 bit pattern, from the format's definition (1 sign, 8 exponent, 7 fraction bits)."""
    sign = -1 if bits & 0x8000 else 1
    e = (bits >> 7) & 0xFF
    f = bits & 0x7F
    if e == 0:
        return sign * Fraction(f, 128) * Fraction(2) ** -126
    return sign * (1 + Fraction(f, 128)) * Fraction(2) ** (e - 127)


def _nearest_bf16_brute(x: float) -> int:
    """Nearest finite bf16 to x, ties to the even pattern: exact rational comparison of the five patterns around the
    truncated fp32 pattern (independent of the oracle's arithmetic)."""
    fx = Fraction(x)
    start = int(np.array([x], np.float32).view(np.uint32)[0] >> 16) & 0xFFFF
    best, best_err = None, None
    for cand in range(max(0, (start & 0x7FFF) - 2), min(0x7F7F, (start & 0x7FFF) + 2) + 1):
        bits = cand | (start & 0x8000)
        err = abs(_bf16_value(bits) - fx)
        if best is None or err < best_err or (err == best_err and bits % 2 == 0 and best % 2 == 1):
            best, best_err = bits, err
    return best


def test_f64_to_bf16_matches_brute_force_and_torch(oracle):
    rng = np.random.default_rng(5)
    xs = np.concatenate([rng.standard_normal(300), rng.standard_normal(100) * 1e-3, rng.standard_normal(100) * 1e5,
                         np.array([0.0, 1.0, -1.0, 0.5, 3.0, 1e-40, -1e-40, 2.0 ** -133, 2.0 ** -134, 1.5 * 2.0 ** -133])])
    for x in xs:
        assert oracle.f64_to_bf16(float(x)) == _nearest_bf16_brute(float(x)), x
    # on values that are already fp32 the one-step rounding is the library's fp32 -> bf16 conversion
    f = xs.astype(np.float32)
    want = torch.from_numpy(f).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([oracle.f64_to_bf16(float(v)) for v in f], np.uint16)
    nz = f != 0
    assert np.array_equal(got[nz], want[nz])


def test_f64_to_bf16_rounds_once_and_handles_ties_and_specials(oracle):
    one = 0x3F80
    assert oracle.f64_to_bf16(1.0 + 2.0 ** -8) == one              # exact tie: to the even pattern
    assert oracle.f64_to_bf16(1.0 + 2.0 ** -8 + 2.0 ** -40) == one + 1   # just above the tie: up (fp32 first would give 1.0)
    assert oracle.f64_to_bf16(1.0 + 3 * 2.0 ** -8) == one + 2      # tie between odd and even: to even
    assert oracle.f64_to_bf16(-(1.0 + 2.0 ** -8 + 2.0 ** -40)) == (one + 1) | 0x8000
    assert oracle.f64_to_bf16(float("inf")) == 0x7F80 and oracle.f64_to_bf16(float("-inf")) == 0xFF80
    assert oracle.f64_to_bf16(3.4e38) == 0x7F80                    # above the largest finite bf16 after rounding
    assert oracle.f64_to_bf16(float("nan")) & 0x7FC0 == 0x7FC0
    assert oracle.f64_to_bf16(0.0) == 0 and oracle.f64_to_bf16(-0.0) == 0x8000
    assert oracle.f64_to_bf16(2.0 ** -133) == 1 and oracle.f64_to_bf16(2.0 ** -135) == 0


def _bits(a32: np.ndarray) -> np.ndarray:
    return torch.from_numpy(np.ascontiguousarray(a32, np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16).copy()


def test_forward_reads_bf16_rows_exactly(oracle):
    """Pooled sums over a bf16 table equal the library's embedding_bag over the widened table (all values exact in
    fp32, few terms: the fp64 sum rounded once equals torch's fp64 result rounded once)."""
    rng = np.random.default_rng(6)
    R, D, B = 40, 8, 12
    tbits = _bits(rng.standard_normal((R, D)).astype(np.float32))
    wide = oracle.bf16_bits_to_f32(tbits)
    lens = rng.integers(0, 6, B)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    keys = rng.integers(0, R, int(off[-1])).astype(np.int64)
    out, rows, _ = oracle.lookup_fwd(tbits, keys, None, off, oracle.POOL_SUM, want_rows=True)
    ref = torch.nn.functional.embedding_bag(torch.from_numpy(keys), torch.from_numpy(wide).double(),
                                            torch.from_numpy(off[:-1].astype(np.int64)), mode="sum")
    assert np.array_equal(out, ref.float().numpy())
    assert np.array_equal(rows, wide[keys])


def test_adagrad_bf16_closed_form_first_step(oracle):
    R, D, c, lr, eps = 6, 8, 0.5, 0.01, 1e-8
    w0 = 2.0
    tbits = _bits(np.full((R, D), w0, np.float32))
    state = np.zeros(R, np.float32)
    oracle.sparse_adagrad_bf16(tbits, state, np.array([2], np.int64), np.full((1, D), c, np.float32), lr, eps)
    assert state[2] == np.float32(c * c)
    want = _nearest_bf16_brute(w0 - float(np.float32(lr)) * c / (c + float(np.float32(eps))))
    assert np.all(tbits[2] == want)
    others = np.delete(np.arange(R), 2)
    assert np.all(tbits[others] == _bits(np.array([w0], np.float32))[0]) and np.all(state[others] == 0)


def test_adagrad_bf16_zero_gradient_keeps_bits_and_matches_fp32_rule(oracle):
    rng = np.random.default_rng(7)
    R, D = 50, 16
    tbits0 = _bits(rng.standard_normal((R, D)).astype(np.float32))
    s0 = rng.random(R).astype(np.float32)
    keys = np.array([1, 7, 20, 44], np.int64)
    g = rng.standard_normal((4, D)).astype(np.float32)
    g[1] = 0.0
    tbits, state = tbits0.copy(), s0.copy()
    oracle.sparse_adagrad_bf16(tbits, state, keys, g, 0.05, 1e-6)
    assert np.array_equal(tbits[7], tbits0[7]) and state[7] == s0[7]
    rest = np.setdiff1d(np.arange(R), keys)
    assert np.array_equal(tbits[rest], tbits0[rest]) and np.array_equal(state[rest], s0[rest])
    # the fp32-table rule on the widened rows gives the same fp64 result rounded to fp32: the bf16 result is the
    # nearest bf16 to it up to the fp32 rounding, i.e. within half a bf16 spacing (at most 2^-8 relative) plus an fp32 ulp
    t32, s32 = oracle.bf16_bits_to_f32(tbits0).copy(), s0.copy()
    oracle.sparse_adagrad(t32, s32, keys, g, 0.05, 1e-6)
    assert np.array_equal(state, s32)
    got = oracle.bf16_bits_to_f32(tbits)
    assert np.all(np.abs(got[keys] - t32[keys]) <= np.abs(t32[keys]) * (2.0 ** -8 + 2.0 ** -23) + 1e-38)
    # and rounding the fp32 result again lands on the same pattern except where the fp32 value sits on a bf16 tie
    again = _bits(t32[keys])
    assert np.mean(again == tbits[keys]) > 0.99


def test_adagrad_bf16_rounds_the_fp64_step_once(oracle):
    """A step whose exact result lies just above the midpoint of two bf16 neighbours: rounding it to fp32 first lands on
    the midpoint and the tie then goes to the even neighbour below; rounding once goes up.  old = 1, g = -1, state 0,
    eps = 0, lr = 2^-8 + 2^-30 (exact in fp32) -> G = 1, new = 1 + 2^-8 + 2^-30 -> bf16 1 + 2^-7."""
    table = np.array([[0x3F80]], dtype=np.uint16)                     # 1.0
    state = np.zeros(1, np.float32)
    lr = float(np.float32(2.0 ** -8 + 2.0 ** -30))
    assert lr == 2.0 ** -8 + 2.0 ** -30
    oracle.sparse_adagrad_bf16(table, state, [0], np.array([[-1.0]], np.float32), lr, 0.0)
    assert state[0] == 1.0
    assert table[0, 0] == 0x3F81                                       # 1 + 2^-7; the two-step rounding would give 0x3F80
