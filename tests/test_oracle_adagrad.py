"""Pins for the oracle's row-wise sparse Adagrad (Section IV-B: gradients are applied directly to the
vectors of the active buffer; Eq. (2): keys outside the batch keep their vectors)."""
import numpy as np
import torch


def test_dim1_equals_torch_adagrad(oracle):
    """With one column the row-wise rule is element-wise Adagrad: pins eps outside the square root,
    the accumulator semantics and the sign, over three consecutive steps."""
    rng = np.random.default_rng(0)
    R = 50
    w0 = rng.standard_normal((R, 1)).astype(np.float32)
    table, state = w0.copy(), np.zeros(R, np.float32)
    p = torch.nn.Parameter(torch.from_numpy(w0.copy()).double())
    opt = torch.optim.Adagrad([p], lr=0.01, eps=1e-8, initial_accumulator_value=0.0, lr_decay=0.0, weight_decay=0.0)
    for step in range(3):
        keys = np.sort(rng.choice(R, size=20, replace=False)).astype(np.int64)
        g = rng.standard_normal((20, 1)).astype(np.float32)
        oracle.sparse_adagrad(table, state, keys, g, 0.01, 1e-8)
        dense = torch.zeros(R, 1, dtype=torch.float64)
        dense[torch.from_numpy(keys)] = torch.from_numpy(g).double()
        p.grad = dense
        opt.step()
        assert np.allclose(table, p.detach().numpy(), rtol=1e-6, atol=1e-8)
        assert np.allclose(state, opt.state[p]["sum"].numpy()[:, 0], rtol=1e-6)


def test_closed_form_first_step_constant_gradient(oracle):
    R, D, c = 10, 8, np.float32(0.5)
    table = np.full((R, D), 2.0, np.float32)
    state = np.zeros(R, np.float32)
    oracle.sparse_adagrad(table, state, np.array([3], np.int64), np.full((1, D), c, np.float32), 0.01, 1e-8)
    assert state[3] == c * c                                       # mean of squares, not their sum
    assert np.allclose(table[3], 2.0 - 0.01 * 0.5 / (0.5 + 1e-8), rtol=1e-7)
    # negative gradient moves the other way by the same amount
    table2 = np.full((R, D), 2.0, np.float32)
    state2 = np.zeros(R, np.float32)
    oracle.sparse_adagrad(table2, state2, np.array([3], np.int64), np.full((1, D), -c, np.float32), 0.01, 1e-8)
    assert np.allclose(table2[3] - 2.0, 2.0 - table[3])


def test_zero_gradient_and_untouched_rows_are_bit_unchanged(oracle):
    rng = np.random.default_rng(1)
    R, D = 64, 16
    t0 = rng.standard_normal((R, D)).astype(np.float32)
    s0 = rng.random(R).astype(np.float32)
    s0[5] = 0.0
    table, state = t0.copy(), s0.copy()
    keys = np.array([5, 9, 33], np.int64)
    g = rng.standard_normal((3, D)).astype(np.float32)
    g[0] = 0.0                       # zero gradient on a row whose state is zero: 0 / (0 + eps) = 0, no NaN
    oracle.sparse_adagrad(table, state, keys, g, 0.01, 1e-8)
    assert table[5].tobytes() == t0[5].tobytes() and state[5] == 0.0
    rest = np.setdiff1d(np.arange(R), keys)
    assert table[rest].tobytes() == t0[rest].tobytes() and state[rest].tobytes() == s0[rest].tobytes()
    assert not np.array_equal(table[9], t0[9]) and state[9] > s0[9]


def test_brute_force_dim_gt_1(oracle):
    rng = np.random.default_rng(2)
    R, D = 30, 12
    t0 = rng.standard_normal((R, D)).astype(np.float32)
    s0 = rng.random(R).astype(np.float32)
    keys = np.array([2, 7, 29], np.int64)
    g = rng.standard_normal((3, D)).astype(np.float32)
    table, state = t0.copy(), s0.copy()
    oracle.sparse_adagrad(table, state, keys, g, 0.05, 1e-6)
    for p, k in enumerate(keys):
        G = float(s0[k]) + sum(float(x) ** 2 for x in g[p]) / D
        assert state[k] == np.float32(G)
        for d in range(D):
            want = float(t0[k, d]) - float(np.float32(0.05)) * float(g[p, d]) / (G ** 0.5 + float(np.float32(1e-6)))
            assert table[k, d] == np.float32(want)
