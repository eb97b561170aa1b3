"""Shared plumbing of the GPU parity tests: device transfer, the five-call step through the C-ABI
binding, and the comparison rules (bit-exact for integer outputs, scaled tolerance for values)."""
from __future__ import annotations

import numpy as np
import torch

from oracle import np_oracle as O
from paper_2604_06956_amd import binding as B
from paper_2604_06956_amd import workloads as wl

RTOL_F32 = 1e-5
RTOL_BF16 = 1e-2


def progress(msg: str) -> None:
    """A flushed line on stdout (shown with pytest -s, kept in the captured output otherwise): names the case before a
    long GPU step starts, so that the tail of a run that dies still says where it was."""
    print(msg, flush=True)


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def bf16_dev(bits_or_f32: np.ndarray) -> torch.Tensor:
    """fp32 array holding bf16-exact values -> bf16 device tensor."""
    return torch.from_numpy(np.ascontiguousarray(bits_or_f32, dtype=np.float32)).bfloat16().cuda()


def assert_close(got: np.ndarray, ref: np.ndarray, scale: np.ndarray, rtol: float, what: str) -> float:
    """|got - ref| <= rtol * |ref| + rtol * scale, where scale = sum of |terms| of that element (the bound of
    a backward-stable sum).  Returns the worst ratio err / bound."""
    got = got.astype(np.float64)
    ref = ref.astype(np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    bound = rtol * np.abs(ref) + rtol * scale + 1e-300
    ratio = np.abs(got - ref) / bound
    worst = float(ratio.max()) if ratio.size else 0.0
    assert np.isfinite(got).all(), f"{what}: non-finite values"
    assert worst <= 1.0, f"{what}: error {worst:.3g}x the tolerance at {np.unravel_index(ratio.argmax(), ratio.shape)}"
    return worst


def gpu_dedup(keys: np.ndarray, key_bits: int):
    d = B.np_dedup(dev(keys.astype(np.int64)), key_bits)
    torch.cuda.synchronize()
    U = int(d["num_unique"].item())
    n = keys.shape[0]
    return dict(unique=host(d["unique"])[:U], inverse=host(d["inverse"])[:n], counts=host(d["counts"])[:U],
                occ_offsets=host(d["occ_offsets"])[:U + 1], occ=host(d["occ"])[:n], U=U), d


def assert_dedup_equal(g: dict, keys: np.ndarray):
    unique, inverse, counts, occ_offsets, occ = O.dedup(keys)
    assert g["U"] == unique.shape[0]
    for name, ref in (("unique", unique), ("inverse", inverse), ("counts", counts), ("occ_offsets", occ_offsets),
                      ("occ", occ)):
        assert np.array_equal(g[name], ref), f"dedup output {name} differs"
    return unique, inverse, counts, occ_offsets, occ


def gpu_step(cfg: wl.Config, batch: wl.Batch, table: torch.Tensor, state: torch.Tensor, out_dtype=None):
    """dedup -> route -> forward -> backward -> update through the binding; returns device tensors."""
    n = batch.n
    keys = dev(batch.keys)
    off = dev(batch.bag_offsets)
    seq = cfg.mode == wl.SEQ
    if out_dtype is None:
        out_dtype = B.BF16 if seq else B.F32
    dY = bf16_dev(batch.dY) if seq else dev(batch.dY)
    d = B.np_dedup(keys, cfg.key_bits)
    r = B.np_route(d["unique"], d["num_unique"], n, cfg.num_shards, cfg.shard_fn, inverse=d["inverse"], n=n)
    out, _ = B.np_lookup_fwd(table, r["send_keys"], r["lookup_to_send"], off, n, cfg.mode, batch.max_len, out_dtype,
                             num_list=d["num_unique"], cap=n)
    grads = B.np_lookup_bwd(dY, cfg.dim, cfg.mode, batch.max_len, off, n, d["occ_offsets"], d["occ"], d["num_unique"], n,
                            unique_to_send=r["unique_to_send"])
    B.np_sparse_adagrad(table, state, r["send_keys"], grads, d["num_unique"], n, cfg.lr, cfg.eps)
    torch.cuda.synchronize()
    return dict(dedup=d, route=r, out=out, grads=grads, dY=dY)


def assert_int_outputs_equal(g: dict, ref: dict, n: int, S: int):
    U = int(g["dedup"]["num_unique"].item())
    assert U == ref["unique"].shape[0]
    d, r = g["dedup"], g["route"]
    pairs = [(d["unique"], "unique", U), (d["inverse"], "inverse", n), (d["counts"], "counts", U),
             (d["occ_offsets"], "occ_offsets", U + 1), (d["occ"], "occ", n), (r["send_keys"], "send_keys", U),
             (r["splits"], "splits", S), (r["send_offsets"], "send_offsets", S + 1),
             (r["send_from_unique"], "send_from_unique", U), (r["unique_to_send"], "unique_to_send", U),
             (r["lookup_to_send"], "lookup_to_send", n)]
    for t, name, k in pairs:
        assert np.array_equal(host(t)[:k], ref[name]), f"{name} differs from the oracle"
    return U
