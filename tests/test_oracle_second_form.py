"""A second, independent form of the whole step, built from library routines only (numpy set / sort routines, torch
autograd through embedding_bag / embedding in fp64, the Adagrad rule written out on dense fp64 arrays), against the C
oracle on small inputs: integer outputs bit for bit, values to fp32 rounding.  A dropped term, a swapped operand or a
wrong index in either form shows up as a disagreement."""
import numpy as np
import pytest
import torch

M64 = (1 << 64) - 1


def _mix_py(k: int) -> int:
    c = 0x9E3779B97F4A7C15
    a = (k * c) & M64
    a ^= a >> 32
    a = (a * c) & M64
    a ^= a >> 29
    return a


def _second_form(table, state, keys, off, dY, mode, max_len, S, shard_fn, lr, eps):
    unique, inverse, counts = np.unique(keys, return_inverse=True, return_counts=True)
    occ = np.argsort(keys, kind="stable")
    shard = unique % S if shard_fn == 0 else np.array([_mix_py(int(k)) % S for k in unique], np.int64)
    sfu = np.argsort(shard, kind="stable")
    uts = np.empty_like(sfu)
    uts[sfu] = np.arange(sfu.size)
    splits = np.bincount(shard, minlength=S)
    W = torch.tensor(table, dtype=torch.float64, requires_grad=True)
    kt = torch.from_numpy(keys)
    B = off.size - 1
    if mode in (0, 1):
        lens = np.diff(off)
        out = torch.nn.functional.embedding_bag(kt, W, torch.from_numpy(off[:-1].astype(np.int64)),
                                                mode="sum" if mode == 0 else "mean")
        out = out * torch.from_numpy((lens > 0).astype(np.float64))[:, None]      # an empty bag pools to zeros
        loss = (out * torch.from_numpy(dY.astype(np.float64))).sum()
    else:
        rows = torch.nn.functional.embedding(kt, W)                                # [n, D]
        bag = np.repeat(np.arange(B), np.diff(off))
        pos = np.arange(keys.size) - off[bag]
        out = torch.zeros((B, max_len, table.shape[1]), dtype=torch.float64)
        out[bag, pos] = rows.detach()
        loss = (rows * torch.from_numpy(dY.astype(np.float64))[bag, pos]).sum()
    loss.backward()
    G = W.grad.numpy()[unique]                                                     # [U, D] in distinct-key order
    G32 = G.astype(np.float32).astype(np.float64)                                  # the step hands fp32 gradient rows on
    st = state[unique].astype(np.float64) + (G32 ** 2).mean(axis=1)
    newW = table[unique].astype(np.float64) - lr * G32 / (np.sqrt(st) + eps)[:, None]
    return dict(unique=unique, inverse=inverse.astype(np.int32), counts=counts.astype(np.int32), occ=occ.astype(np.int32),
                occ_offsets=np.concatenate([[0], np.cumsum(counts)]).astype(np.int32), send_keys=unique[sfu], splits=splits,
                send_from_unique=sfu.astype(np.int32), unique_to_send=uts.astype(np.int32),
                lookup_to_send=uts[inverse].astype(np.int32), out=out.detach().numpy(), grads_send=G[sfu], new_rows=newW,
                new_state=st)


@pytest.mark.parametrize("mode", [0, 1, 2])
@pytest.mark.parametrize("S,shard_fn", [(1, 0), (7, 0), (16, 1)])
def test_c_oracle_agrees_with_the_library_form(oracle, mode, S, shard_fn):
    rng = np.random.default_rng(100 * mode + S)
    R, D, B = 300, 8, 40
    table = (rng.standard_normal((R, D)) * 0.01).astype(np.float32)
    state = (rng.random(R) * 0.01).astype(np.float32)
    lens = rng.integers(0, 7, size=B)
    lens[3] = 0
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    keys = (rng.zipf(1.3, size=int(off[-1])) % R).astype(np.int64)
    max_len = int(max(1, lens.max()))
    lr, eps = 0.01, 1e-8
    if mode == 2:
        from paper_2604_06956_amd import workloads as wl
        dY = wl.round_to_bf16(rng.standard_normal((B, max_len, D)).astype(np.float32))
        dy_arg, dy_dt, out_dt = (dY.view(np.uint32) >> 16).astype(np.uint16), oracle.BF16, oracle.F32   # exact: dY is bf16-valued
    else:
        dY = rng.standard_normal((B, D)).astype(np.float32)
        dy_arg, dy_dt, out_dt = dY, oracle.F32, oracle.F32
    ref = _second_form(table, state, keys, off, dY, mode, max_len, S, shard_fn, np.float32(lr).item(), np.float32(eps).item())
    t, s = table.copy(), state.copy()
    got = oracle.step(t, s, keys, off, dy_arg, dy_dt, mode, max_len, S, shard_fn, lr, eps, out_dt)
    for name in ("unique", "inverse", "counts", "occ", "occ_offsets", "send_keys", "splits", "send_from_unique",
                 "unique_to_send", "lookup_to_send"):
        assert np.array_equal(got[name], ref[name]), name
    assert np.allclose(got["out"], ref["out"], rtol=1e-6, atol=1e-9)
    assert np.allclose(got["grads"], ref["grads_send"], rtol=1e-6, atol=1e-8)
    u = ref["unique"]
    assert np.allclose(t[u], ref["new_rows"], rtol=1e-6, atol=1e-9)
    assert np.allclose(s[u], ref["new_state"], rtol=1e-6, atol=1e-12)
    rest = np.setdiff1d(np.arange(R), u)
    assert np.array_equal(t[rest], table[rest]) and np.array_equal(s[rest], state[rest])
