"""Pins for the oracle's fp16-table variant (IEEE binary16 storage): the decoder, the one-step rounding from fp64 and
the row-wise Adagrad step that stores fp16.  The storage precision is a variant of this build, not of the paper."""
from fractions import Fraction

import numpy as np
import torch


def _f16_value(bits: int) -> Fraction:
    """Exact value of a finite binary16 pattern from the format's definition (1 sign, 5 exponent, 10 fraction bits)."""
    sign = -1 if bits & 0x8000 else 1
    e = (bits >> 10) & 0x1F
    f = bits & 0x3FF
    if e == 0:
        return sign * Fraction(f, 1024) * Fraction(2) ** -14
    return sign * (1 + Fraction(f, 1024)) * Fraction(2) ** (e - 15)


def _nearest_f16_brute(x: float) -> int:
    """Nearest finite binary16 to x (|x| < 65520), ties to the even pattern: exact rational comparison with every
    pattern of the same sign in a window around numpy's answer (independent of the oracle's arithmetic)."""
    fx = Fraction(x)
    start = int(np.array([x], np.float64).astype(np.float16).view(np.uint16)[0])
    mag = start & 0x7FFF
    best, best_err = None, None
    for cand in range(max(0, mag - 2), min(0x7BFF, mag + 2) + 1):
        bits = cand | (0x8000 if x < 0 or (x == 0 and np.signbit(x)) else 0)
        err = abs(_f16_value(bits) - fx)
        if best is None or err < best_err or (err == best_err and bits % 2 == 0 and best % 2 == 1):
            best, best_err = bits, err
    return best


def test_decoder_matches_numpy_on_every_pattern(oracle):
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float32)
    got = np.array([oracle.f16_to_f32(int(b)) for b in bits], np.float32)
    fin = np.isfinite(want)
    assert np.array_equal(got[fin].view(np.uint32), want[fin].view(np.uint32))
    assert np.array_equal(np.isnan(got), np.isnan(want)) and np.array_equal(np.isinf(got), np.isinf(want))
    for b in (0x0001, 0x03FF, 0x0400, 0x3C00, 0x7BFF, 0xC000):
        assert Fraction(oracle.f16_to_f32(b)) == _f16_value(b)


def test_f64_to_f16_matches_brute_force_and_numpy(oracle):
    rng = np.random.default_rng(8)
    xs = np.concatenate([rng.standard_normal(300), rng.standard_normal(100) * 1e-3, rng.standard_normal(100) * 1e3,
                         rng.standard_normal(100) * 1e-6,
                         np.array([0.0, 1.0, -1.0, 0.5, 3.0, 65504.0, 65519.9, 2.0 ** -24, 2.0 ** -25, 1.5 * 2.0 ** -24, 6.1e-5,
                                   2.0 ** -14, 2.0 ** -14 - 2.0 ** -26])])
    for x in xs:
        assert oracle.f64_to_f16(float(x)) == _nearest_f16_brute(float(x)), x
    want = xs.astype(np.float16).view(np.uint16)                 # numpy rounds fp64 -> fp16 in one step
    got = np.array([oracle.f64_to_f16(float(v)) for v in xs], np.uint16)
    assert np.array_equal(got, want)


def test_f64_to_f16_rounds_once_and_handles_ties_and_specials(oracle):
    one = 0x3C00
    assert oracle.f64_to_f16(1.0 + 2.0 ** -11) == one                       # exact tie: to the even pattern
    assert oracle.f64_to_f16(1.0 + 2.0 ** -11 + 2.0 ** -40) == one + 1      # just above the tie (fp32 first would give 1.0)
    assert oracle.f64_to_f16(1.0 + 3 * 2.0 ** -11) == one + 2
    assert oracle.f64_to_f16(-(1.0 + 2.0 ** -11 + 2.0 ** -40)) == (one + 1) | 0x8000
    assert oracle.f64_to_f16(65520.0) == 0x7C00 and oracle.f64_to_f16(-1e9) == 0xFC00   # rounds to infinity
    assert oracle.f64_to_f16(65519.99) == 0x7BFF
    assert oracle.f64_to_f16(float("inf")) == 0x7C00 and oracle.f64_to_f16(float("nan")) & 0x7E00 == 0x7E00
    assert oracle.f64_to_f16(0.0) == 0 and oracle.f64_to_f16(-0.0) == 0x8000
    assert oracle.f64_to_f16(2.0 ** -24) == 1 and oracle.f64_to_f16(2.0 ** -26) == 0 and oracle.f64_to_f16(2.0 ** -25) == 0
    assert oracle.f64_to_f16(2.0 ** -14 - 2.0 ** -25) == 0x0400            # largest subnormal + half a step: up into the normals


def _bits(a) -> np.ndarray:
    return np.ascontiguousarray(a, np.float64).astype(np.float16).view(np.uint16).copy()


def test_forward_reads_fp16_rows_exactly(oracle):
    rng = np.random.default_rng(9)
    R, D, B = 40, 8, 12
    tab = rng.standard_normal((R, D)).astype(np.float16)
    wide = tab.astype(np.float32)
    lens = rng.integers(0, 6, B)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    keys = rng.integers(0, R, int(off[-1])).astype(np.int64)
    out, rows, _ = oracle.lookup_fwd(tab, keys, None, off, oracle.POOL_SUM, want_rows=True)
    ref = torch.nn.functional.embedding_bag(torch.from_numpy(keys), torch.from_numpy(wide).double(),
                                            torch.from_numpy(off[:-1].astype(np.int64)), mode="sum")
    assert np.array_equal(out, ref.float().numpy())
    assert np.array_equal(rows, wide[keys])
    assert np.array_equal(oracle.f16_bits_to_f32(tab.view(np.uint16)), wide)


def test_adagrad_f16_closed_form_zero_gradient_and_fp32_rule(oracle):
    R, D, c, lr, eps = 6, 8, 0.5, 0.01, 1e-8
    tbits = _bits(np.full((R, D), 2.0))
    state = np.zeros(R, np.float32)
    oracle.sparse_adagrad_f16(tbits, state, np.array([2], np.int64), np.full((1, D), c, np.float32), lr, eps)
    assert state[2] == np.float32(c * c)
    want = _nearest_f16_brute(2.0 - float(np.float32(lr)) * c / (c + float(np.float32(eps))))
    assert np.all(tbits[2] == want)
    assert np.all(np.delete(tbits, 2, axis=0) == _bits([2.0])[0]) and np.all(np.delete(state, 2) == 0)

    rng = np.random.default_rng(10)
    R, D = 50, 16
    t0 = _bits(rng.standard_normal((R, D)))
    s0 = rng.random(R).astype(np.float32)
    keys = np.array([1, 7, 20, 44], np.int64)
    g = rng.standard_normal((4, D)).astype(np.float32)
    g[1] = 0.0
    tb, st = t0.copy(), s0.copy()
    oracle.sparse_adagrad_f16(tb, st, keys, g, 0.05, 1e-6)
    assert np.array_equal(tb[7], t0[7]) and st[7] == s0[7]
    rest = np.setdiff1d(np.arange(R), keys)
    assert np.array_equal(tb[rest], t0[rest]) and np.array_equal(st[rest], s0[rest])
    t32, s32 = t0.view(np.float16).astype(np.float32), s0.copy()
    oracle.sparse_adagrad(t32, s32, keys, g, 0.05, 1e-6)
    assert np.array_equal(st, s32)
    got = tb.view(np.float16).astype(np.float32)
    assert np.all(np.abs(got[keys] - t32[keys]) <= np.abs(t32[keys]) * (2.0 ** -11 + 2.0 ** -23) + 2.0 ** -25)
    assert np.mean(_bits(t32[keys]) == tb[keys]) > 0.99


def test_adagrad_f16_rounds_the_fp64_step_once(oracle):
    """old = 1, g = -1, state 0, eps = 0, lr = 2^-11 + 2^-30: the exact new value 1 + 2^-11 + 2^-30 lies just above the
    midpoint of 1 and 1 + 2^-10; through fp32 it would become the midpoint and then the even neighbour 1."""
    table = np.array([[0x3C00]], dtype=np.uint16)                     # 1.0
    state = np.zeros(1, np.float32)
    lr = float(np.float32(2.0 ** -11 + 2.0 ** -30))
    assert lr == 2.0 ** -11 + 2.0 ** -30
    oracle.sparse_adagrad_f16(table, state, [0], np.array([[-1.0]], np.float32), lr, 0.0)
    assert state[0] == 1.0
    assert table[0, 0] == 0x3C01                                       # 1 + 2^-10
