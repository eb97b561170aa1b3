"""numpy front end of the CPU oracle (``np_oracle.c``).  TEST INFRASTRUCTURE ONLY.

Imported by the tests, by the smoke check and by the benchmark's CPU-baseline leg.  The
product package never imports this module, and this module never imports the product.

``build()`` compiles ``np_oracle.c`` with gcc into ``libnp_oracle.so`` next to it; the
wrappers below only marshal numpy arrays into the C calls and allocate the outputs.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "np_oracle.c")
_LIB = os.path.join(_HERE, "libnp_oracle.so")

POOL_SUM, POOL_MEAN, SEQ = 0, 1, 2
F32, BF16, F16 = 0, 1, 2
SHARD_MOD, SHARD_HASH = 0, 1

_lib = None


def build(force: bool = False, sanitize: bool = False) -> str:
    """Compile the oracle.  ``sanitize`` builds an ASan/UBSan variant under another name."""
    out = _LIB if not sanitize else os.path.join(_HERE, "libnp_oracle_asan.so")
    if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(_SRC):
        return out
    cmd = ["gcc", "-std=c11", "-O2", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", out, _SRC, "-lm"]
    if sanitize:
        cmd[3:3] = ["-g", "-fsanitize=address,undefined", "-fno-omit-frame-pointer"]
    subprocess.run(cmd, check=True)
    return out


def build_selftest(out: Optional[str] = None) -> str:
    """Compile the stand-alone self-check (oracle/selftest.c + np_oracle.c); the tests build it with sanitizers."""
    out = out or os.path.join(_HERE, "selftest.bin")
    subprocess.run(["gcc", "-std=c11", "-O1", "-Wall", "-o", out, _SRC, os.path.join(_HERE, "selftest.c"), "-lm"], check=True)
    return out


def _load():
    global _lib
    if _lib is None:
        # NP_ORACLE_LIB: load another build of np_oracle.c instead (the tests point it at deliberately broken copies
        # to show that the pins notice them)
        _lib = ctypes.CDLL(os.environ.get("NP_ORACLE_LIB") or build())
        _lib.np_ref_mix.restype = ctypes.c_uint64
        _lib.np_ref_mix.argtypes = [ctypes.c_uint64]
        _lib.np_ref_shard.restype = ctypes.c_int32
        _lib.np_ref_shard.argtypes = [ctypes.c_int64, ctypes.c_int32, ctypes.c_int32]
        _lib.np_ref_f32_to_bf16.restype = ctypes.c_uint16
        _lib.np_ref_f32_to_bf16.argtypes = [ctypes.c_float]
        _lib.np_ref_bf16_to_f32.restype = ctypes.c_float
        _lib.np_ref_bf16_to_f32.argtypes = [ctypes.c_uint16]
        _lib.np_ref_f64_to_bf16.restype = ctypes.c_uint16
        _lib.np_ref_f64_to_bf16.argtypes = [ctypes.c_double]
        _lib.np_ref_f64_to_f16.restype = ctypes.c_uint16
        _lib.np_ref_f64_to_f16.argtypes = [ctypes.c_double]
        _lib.np_ref_f16_to_f32.restype = ctypes.c_float
        _lib.np_ref_f16_to_f32.argtypes = [ctypes.c_uint16]
        for name in ("np_ref_dedup", "np_ref_route", "np_ref_compose", "np_ref_lookup_fwd", "np_ref_lookup_bwd",
                     "np_ref_sparse_adagrad", "np_ref_sparse_adagrad_bf16", "np_ref_sparse_adagrad_16", "np_ref_intersect", "np_ref_sync_rows"):
            getattr(_lib, name).restype = ctypes.c_int
    return _lib


def _p(a: Optional[np.ndarray]):
    if a is None:
        return ctypes.c_void_p(0)
    assert a.flags["C_CONTIGUOUS"]
    return ctypes.c_void_p(a.ctypes.data)


def _chk(rc: int, what: str) -> None:
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


def _as(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


def mix(k: int) -> int:
    return int(_load().np_ref_mix(ctypes.c_uint64(k & 0xFFFFFFFFFFFFFFFF)))


def shard(key: int, num_shards: int, shard_fn: int) -> int:
    return int(_load().np_ref_shard(int(key), int(num_shards), int(shard_fn)))


def f64_to_bf16(x: float) -> int:
    return int(_load().np_ref_f64_to_bf16(ctypes.c_double(x)))


def f64_to_f16(x: float) -> int:
    return int(_load().np_ref_f64_to_f16(ctypes.c_double(x)))


def f16_to_f32(bits: int) -> float:
    return float(_load().np_ref_f16_to_f32(ctypes.c_uint16(bits)))


def f32_to_bf16(x: float) -> int:
    return int(_load().np_ref_f32_to_bf16(ctypes.c_float(x)))


def bf16_to_f32(h: int) -> float:
    return float(_load().np_ref_bf16_to_f32(ctypes.c_uint16(h)))


def dedup(keys) -> Tuple[np.ndarray, np.ndarray, np.ndarray, np.ndarray, np.ndarray]:
    """-> unique[U] i64, inverse[n] i32, counts[U] i32, occ_offsets[U+1] i32, occ[n] i32."""
    keys = _as(keys, np.int64)
    n = keys.shape[0]
    unique = np.empty(max(n, 1), np.int64)
    inverse = np.empty(max(n, 1), np.int32)
    counts = np.empty(max(n, 1), np.int32)
    occ_offsets = np.empty(n + 1, np.int32)
    occ = np.empty(max(n, 1), np.int32)
    nu = ctypes.c_int32(-1)
    rc = _load().np_ref_dedup(_p(keys), ctypes.c_int32(n), _p(unique), _p(inverse), _p(counts), _p(occ_offsets),
                              _p(occ), ctypes.byref(nu))
    _chk(rc, "dedup")
    U = nu.value
    return unique[:U].copy(), inverse[:n].copy(), counts[:U].copy(), occ_offsets[:U + 1].copy(), occ[:n].copy()


def route(unique, num_shards: int, shard_fn: int):
    """-> send_keys[U] i64, splits[S] i32, send_offsets[S+1] i32, send_from_unique[U] i32, unique_to_send[U] i32."""
    unique = _as(unique, np.int64)
    U = unique.shape[0]
    S = int(num_shards)
    send_keys = np.empty(max(U, 1), np.int64)
    splits = np.empty(max(S, 1), np.int32)
    send_offsets = np.empty(max(S, 1) + 1, np.int32)
    sfu = np.empty(max(U, 1), np.int32)
    uts = np.empty(max(U, 1), np.int32)
    rc = _load().np_ref_route(_p(unique), ctypes.c_int32(U), ctypes.c_int32(S), ctypes.c_int32(shard_fn),
                              _p(send_keys), _p(splits), _p(send_offsets), _p(sfu), _p(uts))
    _chk(rc, "route")
    return send_keys[:U].copy(), splits[:S].copy(), send_offsets[:S + 1].copy(), sfu[:U].copy(), uts[:U].copy()


def compose(inverse, unique_to_send) -> np.ndarray:
    inverse = _as(inverse, np.int32)
    uts = _as(unique_to_send, np.int32)
    out = np.empty(inverse.shape[0], np.int32)
    _chk(_load().np_ref_compose(_p(inverse), ctypes.c_int32(inverse.shape[0]), _p(uts), _p(out)), "compose")
    return out


def lookup_fwd(table, list_keys, idx, bag_offsets, mode: int, max_len: int = 1, out_dtype: int = F32,
               want_rows: bool = False, want_abs: bool = False):
    """-> out (fp32 array, or uint16 array of bf16 bit patterns), rows_out or None, abs_out or None.

    ``table`` is fp32, uint16 bf16 bit patterns, or a numpy float16 array (both widened exactly before use; rows_out
    then holds the widened rows).
    """
    if isinstance(table, np.ndarray) and table.dtype == np.uint16:
        table = bf16_bits_to_f32(table)
    elif isinstance(table, np.ndarray) and table.dtype == np.float16:
        table = f16_bits_to_f32(table.view(np.uint16))
    table = _as(table, np.float32)
    R, D = table.shape
    list_keys = _as(list_keys, np.int64)
    L = list_keys.shape[0]
    bag_offsets = _as(bag_offsets, np.int32)
    B = bag_offsets.shape[0] - 1
    n = int(bag_offsets[-1]) if B >= 0 and bag_offsets.size else 0
    idx_a = None if idx is None else _as(idx, np.int32)
    shape = (B, max_len, D) if mode == SEQ else (B, D)
    out = np.zeros(shape, np.uint16 if out_dtype == BF16 else np.float32)
    rows = np.zeros((L, D), np.float32) if want_rows else None
    ab = np.zeros(shape, np.float64) if want_abs else None
    rc = _load().np_ref_lookup_fwd(_p(table), ctypes.c_int64(R), ctypes.c_int32(D), _p(list_keys), ctypes.c_int32(L),
                                   _p(idx_a), _p(bag_offsets), ctypes.c_int32(B), ctypes.c_int32(n),
                                   ctypes.c_int32(mode), ctypes.c_int32(max_len), ctypes.c_int32(out_dtype),
                                   _p(out), _p(rows), _p(ab))
    _chk(rc, "lookup_fwd")
    return out, rows, ab


def lookup_bwd(dY, dy_dtype: int, dim: int, mode: int, max_len: int, bag_offsets, inverse, num_unique: int,
               unique_to_send=None, want_abs: bool = False):
    """-> grads[U, dim] fp32, abs_out or None.  ``dY`` is fp32, or uint16 bf16 bit patterns."""
    dY = _as(dY, np.uint16 if dy_dtype == BF16 else np.float32)
    bag_offsets = _as(bag_offsets, np.int32)
    B = bag_offsets.shape[0] - 1
    n = int(bag_offsets[-1]) if bag_offsets.size else 0
    inverse = _as(inverse, np.int32)
    uts = None if unique_to_send is None else _as(unique_to_send, np.int32)
    grads = np.zeros((num_unique, dim), np.float32)
    ab = np.zeros((num_unique, dim), np.float64) if want_abs else None
    rc = _load().np_ref_lookup_bwd(_p(dY), ctypes.c_int32(dy_dtype), ctypes.c_int32(dim), ctypes.c_int32(mode),
                                   ctypes.c_int32(max_len), _p(bag_offsets), ctypes.c_int32(B), ctypes.c_int32(n),
                                   _p(inverse), ctypes.c_int32(num_unique), _p(uts), _p(grads), _p(ab))
    _chk(rc, "lookup_bwd")
    return grads, ab


def sparse_adagrad(table: np.ndarray, state: np.ndarray, list_keys, grads, lr: float, eps: float) -> None:
    """In place on ``table`` [R, D] fp32 and ``state`` [R] fp32 (both must be C-contiguous fp32 arrays)."""
    assert table.dtype == np.float32 and state.dtype == np.float32
    assert table.flags["C_CONTIGUOUS"] and state.flags["C_CONTIGUOUS"]
    R, D = table.shape
    list_keys = _as(list_keys, np.int64)
    grads = _as(grads, np.float32)
    rc = _load().np_ref_sparse_adagrad(_p(table), _p(state), ctypes.c_int64(R), ctypes.c_int32(D), _p(list_keys),
                                       _p(grads), ctypes.c_int32(list_keys.shape[0]), ctypes.c_float(lr),
                                       ctypes.c_float(eps))
    _chk(rc, "sparse_adagrad")


def sparse_adagrad_bf16(table_bits: np.ndarray, state: np.ndarray, list_keys, grads, lr: float, eps: float) -> None:
    """In place on ``table_bits`` [R, D] uint16 (bf16 bit patterns) and ``state`` [R] fp32."""
    assert table_bits.dtype == np.uint16 and state.dtype == np.float32
    assert table_bits.flags["C_CONTIGUOUS"] and state.flags["C_CONTIGUOUS"]
    R, D = table_bits.shape
    list_keys = _as(list_keys, np.int64)
    grads = _as(grads, np.float32)
    rc = _load().np_ref_sparse_adagrad_bf16(_p(table_bits), _p(state), ctypes.c_int64(R), ctypes.c_int32(D), _p(list_keys),
                                            _p(grads), ctypes.c_int32(list_keys.shape[0]), ctypes.c_float(lr),
                                            ctypes.c_float(eps))
    _chk(rc, "sparse_adagrad_bf16")


def sparse_adagrad_f16(table_bits: np.ndarray, state: np.ndarray, list_keys, grads, lr: float, eps: float) -> None:
    """In place on ``table_bits`` [R, D] uint16 (IEEE binary16 bit patterns) and ``state`` [R] fp32."""
    assert table_bits.dtype == np.uint16 and state.dtype == np.float32
    assert table_bits.flags["C_CONTIGUOUS"] and state.flags["C_CONTIGUOUS"]
    R, D = table_bits.shape
    list_keys = _as(list_keys, np.int64)
    grads = _as(grads, np.float32)
    rc = _load().np_ref_sparse_adagrad_16(_p(table_bits), ctypes.c_int32(F16), _p(state), ctypes.c_int64(R), ctypes.c_int32(D),
                                          _p(list_keys), _p(grads), ctypes.c_int32(list_keys.shape[0]), ctypes.c_float(lr),
                                          ctypes.c_float(eps))
    _chk(rc, "sparse_adagrad_f16")


def intersect(keys_a, keys_b) -> Tuple[np.ndarray, np.ndarray]:
    """-> idx_a, idx_b (int32): positions of the common keys of two ascending distinct key lists, ascending."""
    a = _as(keys_a, np.int64)
    b = _as(keys_b, np.int64)
    m = max(1, min(a.shape[0], b.shape[0]))
    ia = np.empty(m, np.int32)
    ib = np.empty(m, np.int32)
    c = ctypes.c_int32(-1)
    rc = _load().np_ref_intersect(_p(a), ctypes.c_int32(a.shape[0]), _p(b), ctypes.c_int32(b.shape[0]), _p(ia), _p(ib),
                                  ctypes.byref(c))
    _chk(rc, "intersect")
    return ia[:c.value].copy(), ib[:c.value].copy()


def sync_rows(src: np.ndarray, src_idx, dst: np.ndarray, dst_idx) -> None:
    """dst[dst_idx[i]] = src[src_idx[i]] in place on ``dst`` (both [*, D] fp32, C-contiguous)."""
    assert src.dtype == np.float32 and dst.dtype == np.float32 and src.shape[1] == dst.shape[1]
    assert src.flags["C_CONTIGUOUS"] and dst.flags["C_CONTIGUOUS"]
    si = _as(src_idx, np.int32)
    di = _as(dst_idx, np.int32)
    rc = _load().np_ref_sync_rows(_p(src), _p(si), _p(dst), _p(di), ctypes.c_int32(si.shape[0]), ctypes.c_int32(src.shape[1]))
    _chk(rc, "sync_rows")


def f16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact widening of IEEE binary16 bit patterns (uint16) to fp32 values, element by element through the oracle's
    decoder (array helper for comparisons; small and medium arrays only)."""
    flat = np.ascontiguousarray(bits, np.uint16).ravel()
    lut = np.array([f16_to_f32(b) for b in range(65536)], np.float32) if flat.size > 65536 else None
    if lut is not None:
        return lut[flat].reshape(bits.shape)
    return np.array([f16_to_f32(int(b)) for b in flat], np.float32).reshape(bits.shape)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns (uint16) to fp32 values (array helper for comparisons)."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Elementwise ``np_ref_f32_to_bf16`` over an array (slow path through the C scalar for small arrays)."""
    x = _as(x, np.float32)
    lib = _load()
    flat = x.ravel()
    out = np.empty(flat.shape[0], np.uint16)
    for i in range(flat.shape[0]):
        out[i] = lib.np_ref_f32_to_bf16(ctypes.c_float(float(flat[i])))
    return out.reshape(x.shape)


def step(table: np.ndarray, state: np.ndarray, keys, bag_offsets, dY, dy_dtype: int, mode: int, max_len: int,
         num_shards: int, shard_fn: int, lr: float, eps: float, out_dtype: int = F32):
    """One sequential step dedup -> route -> forward -> backward -> update on (table, state) in place.

    The forward reads the send-ordered key list through lookup_to_send; gradients are produced in send order
    and applied with the send-ordered keys, exactly the single-worker flow of Section IV-A with the three
    All2All exchanges elided.  Returns a dict of every intermediate.
    """
    unique, inverse, counts, occ_offsets, occ = dedup(keys)
    send_keys, splits, send_offsets, sfu, uts = route(unique, num_shards, shard_fn)
    l2s = compose(inverse, uts)
    out, _, _ = lookup_fwd(table, send_keys, l2s, bag_offsets, mode, max_len, out_dtype)
    grads, _ = lookup_bwd(dY, dy_dtype, table.shape[1], mode, max_len, bag_offsets, inverse, unique.shape[0], uts)
    sparse_adagrad(table, state, send_keys, grads, lr, eps)
    return dict(unique=unique, inverse=inverse, counts=counts, occ_offsets=occ_offsets, occ=occ, send_keys=send_keys,
                splits=splits, send_offsets=send_offsets, send_from_unique=sfu, unique_to_send=uts,
                lookup_to_send=l2s, out=out, grads=grads)
