"""Thin Python layer over the C-ABI HIP library (``include/nestpipe.h``).

Argument marshalling only: every step of the path runs in the library's kernels.  torch supplies device
memory and the stream; no torch op takes part in the computation.  The functions carry the names of the
C entry points.  Output and workspace tensors are allocated here unless the caller passes them in
(``out=...`` dictionaries / ``ws=`` tensors), which the benchmark does to keep allocation out of the loop.

The library must have been built (``python -m paper_2604_06956_amd.build``); if it is missing the import
fails: there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional, Tuple

import torch  # imported before the library so that the library binds to torch's HIP runtime

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("NESTPIPE_LIB") or os.path.join(_PKG, "libnestpipe_hip.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2604_06956_amd.build`")


NP_OK = 0
SHARD_MOD, SHARD_HASH = 0, 1
POOL_SUM, POOL_MEAN, SEQ = 0, 1, 2
F32, BF16, F16 = 0, 1, 2
MAX_SHARDS = 4096
ROUTE_STATIC_MAX_SHARDS = 2048

_vp, _i32, _i64, _sz, _f32, _u64 = (ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t, ctypes.c_float,
                                    ctypes.c_uint64)



def _configure(L: ctypes.CDLL) -> ctypes.CDLL:
    """Declare the prototypes of include/nestpipe.h on a loaded library handle."""
    L.np_version.restype = ctypes.c_int
    L.np_status_string.restype = ctypes.c_char_p
    L.np_status_string.argtypes = [ctypes.c_int]
    L.np_dedup.restype = ctypes.c_int
    L.np_dedup.argtypes = [_vp, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]
    L.np_dedup_workspace_bytes.restype = _sz
    L.np_dedup_workspace_bytes.argtypes = [_i32, _i32]
    L.np_route.restype = ctypes.c_int
    L.np_route.argtypes = [_vp, _vp, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _vp, _vp, _sz, _vp]
    L.np_route_static.restype = ctypes.c_int
    L.np_route_static.argtypes = [_vp, _vp, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _vp, _vp]
    L.np_route_workspace_bytes.restype = _sz
    L.np_route_workspace_bytes.argtypes = [_i32, _i32]
    L.np_lookup_fwd.restype = ctypes.c_int
    L.np_lookup_fwd.argtypes = [_vp, _i64, _i32, _vp, _vp, _i32, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _sz,
                                  _vp]
    L.np_lookup_fwd_workspace_bytes.restype = _sz
    L.np_lookup_fwd_workspace_bytes.argtypes = [_i32, _i32, _i32, _i32]
    L.np_lookup_bwd.restype = ctypes.c_int
    L.np_lookup_bwd.argtypes = [_vp, _i32, _i32, _i32, _i32, _vp, _i32, _i32, _vp, _vp, _vp, _i32, _vp, _vp, _vp, _sz, _vp]
    L.np_lookup_bwd_prepared.restype = ctypes.c_int
    L.np_lookup_bwd_prepared.argtypes = L.np_lookup_bwd.argtypes
    L.np_lookup_bwd_prepare.restype = ctypes.c_int
    L.np_lookup_bwd_prepare.argtypes = [_i32, _i32, _i32, _i32, _vp, _i32, _i32, _vp, _vp, _vp, _vp, _sz, _vp]
    L.np_lookup_bwd_workspace_bytes.restype = _sz
    L.np_lookup_bwd_workspace_bytes.argtypes = [_i32, _i32, _i32, _i32]
    L.np_lookup_bwd_adagrad.restype = ctypes.c_int
    L.np_lookup_bwd_adagrad.argtypes = [_vp, _i32, _i32, _i32, _i32, _vp, _i32, _i32, _vp, _vp, _vp, _vp, _i32, _vp, _vp, _i64,
                                        _f32, _f32, _vp, _sz, _vp]
    L.np_lookup_bwd_adagrad_t.restype = ctypes.c_int
    L.np_lookup_bwd_adagrad_t.argtypes = [_vp, _i32, _i32, _i32, _i32, _vp, _i32, _i32, _vp, _vp, _vp, _vp, _i32, _vp, _i32, _vp,
                                          _i64, _f32, _f32, _vp, _sz, _vp]
    L.np_sparse_adagrad.restype = ctypes.c_int
    L.np_sparse_adagrad.argtypes = [_vp, _vp, _i64, _i32, _vp, _vp, _vp, _i32, _f32, _f32, _vp]
    L.np_lookup_fwd_t.restype = ctypes.c_int
    L.np_lookup_fwd_t.argtypes = [_vp, _i32, _i64, _i32, _vp, _vp, _i32, _vp, _vp, _i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp,
                                  _sz, _vp]
    L.np_sparse_adagrad_t.restype = ctypes.c_int
    L.np_sparse_adagrad_t.argtypes = [_vp, _i32, _vp, _i64, _i32, _vp, _vp, _vp, _i32, _f32, _f32, _vp]
    L.np_util_table_init_t.restype = ctypes.c_int
    L.np_util_table_init_t.argtypes = [_vp, _i32, _i64, _i32, _u64, _vp]
    L.np_util_table_count_changed_t.restype = ctypes.c_int
    L.np_util_table_count_changed_t.argtypes = [_vp, _i32, _i64, _i32, _u64, _vp, _vp]
    L.np_intersect.restype = ctypes.c_int
    L.np_intersect.argtypes = [_vp, _vp, _i32, _vp, _vp, _i32, _vp, _vp, _vp, _vp, _sz, _vp]
    L.np_intersect_workspace_bytes.restype = _sz
    L.np_intersect_workspace_bytes.argtypes = [_i32]
    L.np_sync_rows.restype = ctypes.c_int
    L.np_sync_rows.argtypes = [_vp, _vp, _vp, _vp, _vp, _i32, _i32, _vp]
    L.np_util_table_init.restype = ctypes.c_int
    L.np_util_table_init.argtypes = [_vp, _i64, _i32, _u64, _vp]
    L.np_util_table_count_changed.restype = ctypes.c_int
    L.np_util_table_count_changed.argtypes = [_vp, _i64, _i32, _u64, _vp, _vp]
    L.np_util_check_batch.restype = ctypes.c_int
    L.np_util_check_batch.argtypes = [_vp, _i32, _i64, _vp, _i32, _vp, _vp]
    L.np_util_gather_rate.restype = ctypes.c_int
    L.np_util_gather_rate.argtypes = [_vp, _i64, _i64, ctypes.c_uint32, _vp, _vp]
    L.np_util_stream_copy.restype = ctypes.c_int
    L.np_util_stream_copy.argtypes = [_vp, _vp, _sz, _vp]
    L.np_tune_set.restype = ctypes.c_int
    L.np_tune_set.argtypes = [ctypes.c_char_p, _i64]
    L.np_tune_get.restype = _i64
    L.np_tune_get.argtypes = [ctypes.c_char_p]
    L.np_prof_enable.restype = ctypes.c_int
    L.np_prof_enable.argtypes = [ctypes.c_int]
    L.np_prof_only.restype = ctypes.c_int
    L.np_prof_only.argtypes = [ctypes.c_char_p]
    L.np_prof_collect.restype = ctypes.c_int
    L.np_prof_collect.argtypes = [ctypes.POINTER(ctypes.c_char_p), ctypes.POINTER(ctypes.c_float), ctypes.c_int]
    return L


lib = _configure(ctypes.CDLL(LIB_PATH))


class NestPipeError(RuntimeError):
    def __init__(self, call: str, status: int):
        self.status = status
        super().__init__(f"{call} failed: {status} ({lib.np_status_string(status).decode()})")


def _chk(call: str, rc: int) -> None:
    if rc != NP_OK:
        raise NestPipeError(call, rc)


def _ptr(t: Optional[torch.Tensor], dtype: Optional[torch.dtype] = None) -> int:
    """Device address of ``t`` (0 for None) after checking what the C side cannot: residency, contiguity and, when
    ``dtype`` is given, the element type the entry point reads the buffer as."""
    if t is None:
        return 0
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("tensors handed to the library must be contiguous device tensors")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"expected a {dtype} tensor, got {t.dtype}")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ws(nbytes: int, ws: Optional[torch.Tensor], device) -> Tuple[Optional[torch.Tensor], int]:
    if nbytes == 0 and ws is None:
        return None, 0
    if ws is None:
        ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)
    return ws, ws.numel() * ws.element_size()


def _dt(dtype: int):
    return torch.bfloat16 if dtype == BF16 else torch.float32


def version() -> int:
    return int(lib.np_version())


def np_dedup_workspace_bytes(n: int, key_bits: int) -> int:
    return int(lib.np_dedup_workspace_bytes(n, key_bits))


def np_dedup(keys: torch.Tensor, key_bits: int, out: Optional[Dict[str, torch.Tensor]] = None,
             ws: Optional[torch.Tensor] = None, want_inverse: bool = True) -> Dict[str, torch.Tensor]:
    """-> dict(unique[n] i64, inverse[n] i32, counts[n] i32, occ_offsets[n+1] i32, occ[n] i32, num_unique[1] i32).
    Only the first U = num_unique entries of unique / counts / occ_offsets(+1) are meaningful.  ``want_inverse=False``
    (or ``out["inverse"] is None``) passes NULL for the optional inverse map."""
    n = keys.numel()
    dev = keys.device
    if out is None:
        out = dict(unique=torch.empty(max(n, 1), dtype=torch.int64, device=dev),
                   inverse=torch.empty(max(n, 1), dtype=torch.int32, device=dev) if want_inverse else None,
                   counts=torch.empty(max(n, 1), dtype=torch.int32, device=dev),
                   occ_offsets=torch.empty(n + 1, dtype=torch.int32, device=dev),
                   occ=torch.empty(max(n, 1), dtype=torch.int32, device=dev),
                   num_unique=torch.empty(1, dtype=torch.int32, device=dev))
    ws, ws_bytes = _ws(np_dedup_workspace_bytes(n, key_bits), ws, dev)
    rc = lib.np_dedup(_ptr(keys, torch.int64), n, key_bits, _ptr(out["unique"], torch.int64), _ptr(out.get("inverse") if want_inverse else None, torch.int32),
                      _ptr(out["counts"], torch.int32),
                      _ptr(out["occ_offsets"], torch.int32), _ptr(out["occ"], torch.int32), _ptr(out["num_unique"], torch.int32), _ptr(ws), ws_bytes, _stream())
    _chk("np_dedup", rc)
    return out


def np_route_workspace_bytes(cap: int, num_shards: int) -> int:
    return int(lib.np_route_workspace_bytes(cap, num_shards))


def np_route(unique: torch.Tensor, num_unique: torch.Tensor, cap: int, num_shards: int, shard_fn: int,
             inverse: Optional[torch.Tensor] = None, n: int = 0, out: Optional[Dict[str, torch.Tensor]] = None,
             ws: Optional[torch.Tensor] = None) -> Dict[str, torch.Tensor]:
    """-> dict(send_keys[cap] i64, splits[S] i32, send_offsets[S+1] i32, send_from_unique[cap] i32,
    unique_to_send[cap] i32, lookup_to_send[n] i32 when ``inverse`` is given)."""
    dev = unique.device
    if out is None:
        out = dict(send_keys=torch.empty(max(cap, 1), dtype=torch.int64, device=dev),
                   splits=torch.empty(max(num_shards, 1), dtype=torch.int32, device=dev),
                   send_offsets=torch.empty(max(num_shards, 1) + 1, dtype=torch.int32, device=dev),
                   send_from_unique=torch.empty(max(cap, 1), dtype=torch.int32, device=dev),
                   unique_to_send=torch.empty(max(cap, 1), dtype=torch.int32, device=dev))
        if inverse is not None:
            out["lookup_to_send"] = torch.empty(max(n, 1), dtype=torch.int32, device=dev)
    ws, ws_bytes = _ws(np_route_workspace_bytes(cap, num_shards), ws, dev)
    rc = lib.np_route(_ptr(unique, torch.int64), _ptr(num_unique, torch.int32), cap, num_shards, shard_fn, _ptr(out["send_keys"], torch.int64),
                      _ptr(out["splits"], torch.int32), _ptr(out["send_offsets"], torch.int32), _ptr(out["send_from_unique"], torch.int32),
                      _ptr(out["unique_to_send"], torch.int32), _ptr(inverse, torch.int32), n if inverse is not None else 0,
                      _ptr(out.get("lookup_to_send"), torch.int32) if inverse is not None else 0, _ptr(ws), ws_bytes, _stream())
    _chk("np_route", rc)
    return out


def np_route_static(unique: torch.Tensor, num_unique: torch.Tensor, cap: int, num_shards: int, shard_fn: int,
                    out: Dict[str, torch.Tensor], inverse: Optional[torch.Tensor] = None, n: int = 0) -> Dict[str, torch.Tensor]:
    """np_route on the library's built-in scratch.  Nothing is allocated on the way, here or in the library: the caller
    brings every output tensor in ``out`` (the keys np_route returns; ``lookup_to_send`` too when ``inverse`` is given)."""
    rc = lib.np_route_static(_ptr(unique, torch.int64), _ptr(num_unique, torch.int32), cap, num_shards, shard_fn,
                             _ptr(out["send_keys"], torch.int64), _ptr(out["splits"], torch.int32), _ptr(out["send_offsets"], torch.int32),
                             _ptr(out["send_from_unique"], torch.int32), _ptr(out["unique_to_send"], torch.int32), _ptr(inverse, torch.int32),
                             n if inverse is not None else 0, _ptr(out["lookup_to_send"], torch.int32) if inverse is not None else 0,
                             _stream())
    _chk("np_route_static", rc)
    return out


def np_lookup_fwd(table: torch.Tensor, list_keys: torch.Tensor, idx: Optional[torch.Tensor], bag_offsets: torch.Tensor,
                  n: int, mode: int, max_len: int = 1, out_dtype: int = F32, num_list: Optional[torch.Tensor] = None,
                  cap: int = 0, want_rows: bool = False, out: Optional[torch.Tensor] = None,
                  rows_out: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, Optional[torch.Tensor]]:
    """-> (out [B, D] or [B, max_len, D], rows_out [cap, D] or None)."""
    num_rows, dim = table.shape
    num_bags = bag_offsets.numel() - 1
    dev = table.device
    if out is None:
        shape = (num_bags, max_len, dim) if mode == SEQ else (num_bags, dim)
        out = torch.empty(shape, dtype=_dt(out_dtype), device=dev)
    if want_rows and rows_out is None:
        rows_out = torch.empty((max(cap, 1), dim), dtype=torch.float32, device=dev)
    rc = lib.np_lookup_fwd(_ptr(table, torch.float32), num_rows, dim, _ptr(list_keys, torch.int64), _ptr(num_list, torch.int32), cap,
                           _ptr(idx, torch.int32), _ptr(bag_offsets, torch.int32), num_bags, n, mode, max_len, out_dtype,
                           _ptr(out, _dt(out_dtype)), _ptr(rows_out, torch.float32), 0, 0, _stream())
    _chk("np_lookup_fwd", rc)
    return out, rows_out


def _table_dtype(table: torch.Tensor) -> int:
    if table.dtype == torch.float32:
        return F32
    if table.dtype == torch.bfloat16:
        return BF16
    if table.dtype == torch.float16:
        return F16
    raise TypeError(f"table dtype {table.dtype} is not supported (float32, bfloat16 or float16)")


def np_lookup_fwd_t(table: torch.Tensor, list_keys: torch.Tensor, idx: Optional[torch.Tensor], bag_offsets: torch.Tensor,
                    n: int, mode: int, max_len: int = 1, out_dtype: int = F32, num_list: Optional[torch.Tensor] = None,
                    cap: int = 0, want_rows: bool = False, out: Optional[torch.Tensor] = None,
                    rows_out: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, Optional[torch.Tensor]]:
    """np_lookup_fwd for a float32 or bfloat16 table (the dtype of ``table`` is passed on); rows_out has the table's dtype."""
    num_rows, dim = table.shape
    num_bags = bag_offsets.numel() - 1
    dev = table.device
    if out is None:
        shape = (num_bags, max_len, dim) if mode == SEQ else (num_bags, dim)
        out = torch.empty(shape, dtype=_dt(out_dtype), device=dev)
    if want_rows and rows_out is None:
        rows_out = torch.empty((max(cap, 1), dim), dtype=table.dtype, device=dev)
    rc = lib.np_lookup_fwd_t(_ptr(table), _table_dtype(table), num_rows, dim, _ptr(list_keys, torch.int64), _ptr(num_list, torch.int32), cap, _ptr(idx, torch.int32),
                             _ptr(bag_offsets, torch.int32), num_bags, n, mode, max_len, out_dtype, _ptr(out), _ptr(rows_out), 0, 0, _stream())
    _chk("np_lookup_fwd_t", rc)
    return out, rows_out


def np_lookup_bwd_workspace_bytes(num_bags: int, n: int, dim: int, mode: int) -> int:
    return int(lib.np_lookup_bwd_workspace_bytes(num_bags, n, dim, mode))


def np_lookup_bwd(dY: torch.Tensor, dim: int, mode: int, max_len: int, bag_offsets: torch.Tensor, n: int,
                  occ_offsets: torch.Tensor, occ: torch.Tensor, num_unique: torch.Tensor, cap: int,
                  unique_to_send: Optional[torch.Tensor] = None, grads: Optional[torch.Tensor] = None,
                  ws: Optional[torch.Tensor] = None) -> torch.Tensor:
    """-> grads [cap, D] fp32 (rows >= U untouched)."""
    dev = dY.device
    num_bags = bag_offsets.numel() - 1
    dy_dtype = BF16 if dY.dtype == torch.bfloat16 else F32
    if dY.dtype not in (torch.bfloat16, torch.float32):
        raise ValueError("dY must be fp32 or bf16")
    if grads is None:
        grads = torch.empty((max(cap, 1), dim), dtype=torch.float32, device=dev)
    ws, ws_bytes = _ws(np_lookup_bwd_workspace_bytes(num_bags, n, dim, mode), ws, dev)
    rc = lib.np_lookup_bwd(_ptr(dY), dy_dtype, dim, mode, max_len, _ptr(bag_offsets, torch.int32), num_bags, n, _ptr(occ_offsets, torch.int32),
                           _ptr(occ, torch.int32), _ptr(num_unique, torch.int32), cap, _ptr(unique_to_send, torch.int32), _ptr(grads, torch.float32), _ptr(ws), ws_bytes,
                           _stream())
    _chk("np_lookup_bwd", rc)
    return grads


def np_lookup_bwd_prepare(dy_dtype: int, dim: int, mode: int, max_len: int, bag_offsets: torch.Tensor, n: int,
                          occ_offsets: torch.Tensor, occ: torch.Tensor, num_unique: torch.Tensor, ws: torch.Tensor) -> None:
    """The part of np_lookup_bwd that needs no dY, written into ``ws`` (hand the same ``ws`` to np_lookup_bwd_prepared)."""
    num_bags = bag_offsets.numel() - 1
    rc = lib.np_lookup_bwd_prepare(dy_dtype, dim, mode, max_len, _ptr(bag_offsets, torch.int32), num_bags, n,
                                   _ptr(occ_offsets, torch.int32), _ptr(occ, torch.int32), _ptr(num_unique, torch.int32), _ptr(ws),
                                   ws.numel() * ws.element_size(), _stream())
    _chk("np_lookup_bwd_prepare", rc)


def np_lookup_bwd_prepared(dY: torch.Tensor, dim: int, mode: int, max_len: int, bag_offsets: torch.Tensor, n: int,
                           occ_offsets: torch.Tensor, occ: torch.Tensor, num_unique: torch.Tensor, cap: int, ws: torch.Tensor,
                           unique_to_send: Optional[torch.Tensor] = None, grads: Optional[torch.Tensor] = None) -> torch.Tensor:
    """np_lookup_bwd on a workspace that np_lookup_bwd_prepare has filled for the same batch."""
    if dY.dtype not in (torch.bfloat16, torch.float32):
        raise ValueError("dY must be fp32 or bf16")
    num_bags = bag_offsets.numel() - 1
    dy_dtype = BF16 if dY.dtype == torch.bfloat16 else F32
    if grads is None:
        grads = torch.empty((max(cap, 1), dim), dtype=torch.float32, device=dY.device)
    rc = lib.np_lookup_bwd_prepared(_ptr(dY), dy_dtype, dim, mode, max_len, _ptr(bag_offsets, torch.int32), num_bags, n,
                                    _ptr(occ_offsets, torch.int32), _ptr(occ, torch.int32), _ptr(num_unique, torch.int32), cap,
                                    _ptr(unique_to_send, torch.int32), _ptr(grads, torch.float32), _ptr(ws),
                                    ws.numel() * ws.element_size(), _stream())
    _chk("np_lookup_bwd_prepared", rc)
    return grads


def np_lookup_bwd_adagrad(dY: torch.Tensor, mode: int, max_len: int, bag_offsets: torch.Tensor, n: int, occ_offsets: torch.Tensor,
                          occ: torch.Tensor, unique: torch.Tensor, num_unique: torch.Tensor, cap: int, table: torch.Tensor,
                          state: torch.Tensor, lr: float, eps: float, ws: Optional[torch.Tensor] = None) -> None:
    """Backward reduction fused with the row-wise Adagrad update of ``table`` / ``state`` (no gradient buffer)."""
    num_rows, dim = table.shape
    num_bags = bag_offsets.numel() - 1
    if dY.dtype not in (torch.bfloat16, torch.float32):
        raise ValueError("dY must be fp32 or bf16")
    dy_dtype = BF16 if dY.dtype == torch.bfloat16 else F32
    ws, ws_bytes = _ws(np_lookup_bwd_workspace_bytes(num_bags, n, dim, mode), ws, dY.device)
    rc = lib.np_lookup_bwd_adagrad(_ptr(dY), dy_dtype, dim, mode, max_len, _ptr(bag_offsets, torch.int32), num_bags, n, _ptr(occ_offsets, torch.int32),
                                   _ptr(occ, torch.int32), _ptr(unique, torch.int64), _ptr(num_unique, torch.int32), cap, _ptr(table, torch.float32), _ptr(state, torch.float32), num_rows, lr, eps,
                                   _ptr(ws), ws_bytes, _stream())
    _chk("np_lookup_bwd_adagrad", rc)


def np_lookup_bwd_adagrad_t(dY: torch.Tensor, mode: int, max_len: int, bag_offsets: torch.Tensor, n: int,
                            occ_offsets: torch.Tensor, occ: torch.Tensor, unique: torch.Tensor, num_unique: torch.Tensor, cap: int,
                            table: torch.Tensor, state: torch.Tensor, lr: float, eps: float,
                            ws: Optional[torch.Tensor] = None) -> None:
    """np_lookup_bwd_adagrad for a float32, bfloat16 or float16 table."""
    num_rows, dim = table.shape
    num_bags = bag_offsets.numel() - 1
    if dY.dtype not in (torch.bfloat16, torch.float32):
        raise ValueError("dY must be fp32 or bf16")
    dy_dtype = BF16 if dY.dtype == torch.bfloat16 else F32
    ws, ws_bytes = _ws(np_lookup_bwd_workspace_bytes(num_bags, n, dim, mode), ws, dY.device)
    rc = lib.np_lookup_bwd_adagrad_t(_ptr(dY), dy_dtype, dim, mode, max_len, _ptr(bag_offsets, torch.int32), num_bags, n, _ptr(occ_offsets, torch.int32),
                                     _ptr(occ, torch.int32), _ptr(unique, torch.int64), _ptr(num_unique, torch.int32), cap, _ptr(table), _table_dtype(table), _ptr(state, torch.float32),
                                     num_rows, lr, eps, _ptr(ws), ws_bytes, _stream())
    _chk("np_lookup_bwd_adagrad_t", rc)


def np_sparse_adagrad(table: torch.Tensor, state: torch.Tensor, list_keys: torch.Tensor, grads: torch.Tensor,
                      num_list: torch.Tensor, cap: int, lr: float, eps: float) -> None:
    num_rows, dim = table.shape
    rc = lib.np_sparse_adagrad(_ptr(table, torch.float32), _ptr(state, torch.float32), num_rows, dim, _ptr(list_keys, torch.int64), _ptr(grads, torch.float32), _ptr(num_list, torch.int32), cap,
                               lr, eps, _stream())
    _chk("np_sparse_adagrad", rc)


def np_sparse_adagrad_t(table: torch.Tensor, state: torch.Tensor, list_keys: torch.Tensor, grads: torch.Tensor,
                        num_list: torch.Tensor, cap: int, lr: float, eps: float) -> None:
    num_rows, dim = table.shape
    rc = lib.np_sparse_adagrad_t(_ptr(table), _table_dtype(table), _ptr(state, torch.float32), num_rows, dim, _ptr(list_keys, torch.int64), _ptr(grads, torch.float32),
                                 _ptr(num_list, torch.int32), cap, lr, eps, _stream())
    _chk("np_sparse_adagrad_t", rc)


def np_intersect(keys_a: torch.Tensor, num_a: torch.Tensor, cap_a: int, keys_b: torch.Tensor, num_b: torch.Tensor, cap_b: int,
                 out: Optional[Dict[str, torch.Tensor]] = None, ws: Optional[torch.Tensor] = None) -> Dict[str, torch.Tensor]:
    """-> dict(idx_a, idx_b [min(cap_a, cap_b)] i32, num_common[1] i32)."""
    dev = keys_a.device
    if out is None:
        m = max(1, min(cap_a, cap_b))
        out = dict(idx_a=torch.empty(m, dtype=torch.int32, device=dev), idx_b=torch.empty(m, dtype=torch.int32, device=dev),
                   num_common=torch.empty(1, dtype=torch.int32, device=dev))
    ws, ws_bytes = _ws(int(lib.np_intersect_workspace_bytes(cap_b)), ws, dev)
    rc = lib.np_intersect(_ptr(keys_a, torch.int64), _ptr(num_a, torch.int32), cap_a, _ptr(keys_b, torch.int64), _ptr(num_b, torch.int32), cap_b, _ptr(out["idx_a"], torch.int32),
                          _ptr(out["idx_b"], torch.int32), _ptr(out["num_common"], torch.int32), _ptr(ws), ws_bytes, _stream())
    _chk("np_intersect", rc)
    return out


def np_sync_rows(src_rows: torch.Tensor, src_idx: torch.Tensor, dst_rows: torch.Tensor, dst_idx: torch.Tensor,
                 count: torch.Tensor, cap: int) -> None:
    dim = src_rows.shape[1]
    rc = lib.np_sync_rows(_ptr(src_rows), _ptr(src_idx, torch.int32), _ptr(dst_rows), _ptr(dst_idx, torch.int32), _ptr(count, torch.int32), cap, dim, _stream())
    _chk("np_sync_rows", rc)


def np_util_table_init(table: torch.Tensor, seed: int) -> None:
    num_rows, dim = table.shape
    _chk("np_util_table_init", lib.np_util_table_init(_ptr(table, torch.float32), num_rows, dim, seed, _stream()))


def np_util_table_count_changed(table: torch.Tensor, seed: int) -> int:
    """Rows of ``table`` that differ from the initialiser (synchronises)."""
    num_rows, dim = table.shape
    cnt = torch.zeros(1, dtype=torch.int64, device=table.device)
    _chk("np_util_table_count_changed", lib.np_util_table_count_changed(_ptr(table, torch.float32), num_rows, dim, seed, _ptr(cnt), _stream()))
    return int(cnt.item())


def np_util_table_init_t(table: torch.Tensor, seed: int) -> None:
    num_rows, dim = table.shape
    _chk("np_util_table_init_t", lib.np_util_table_init_t(_ptr(table), _table_dtype(table), num_rows, dim, seed, _stream()))


def np_util_table_count_changed_t(table: torch.Tensor, seed: int) -> int:
    """Rows of ``table`` (float32 or bfloat16) that differ from the initialiser (synchronises)."""
    num_rows, dim = table.shape
    cnt = torch.zeros(1, dtype=torch.int64, device=table.device)
    _chk("np_util_table_count_changed_t",
         lib.np_util_table_count_changed_t(_ptr(table), _table_dtype(table), num_rows, dim, seed, _ptr(cnt), _stream()))
    return int(cnt.item())


def np_util_check_batch(keys: Optional[torch.Tensor], num_rows: int, bag_offsets: Optional[torch.Tensor]) -> Tuple[int, int, int, int]:
    """Precondition check (synchronises): (keys out of range, decreasing offsets, offsets[0] != 0, offsets[-1] != n)."""
    n = keys.numel() if keys is not None else 0
    num_bags = bag_offsets.numel() - 1 if bag_offsets is not None else 0
    dev = keys.device if keys is not None else bag_offsets.device
    err = torch.empty(4, dtype=torch.int64, device=dev)
    _chk("np_util_check_batch", lib.np_util_check_batch(_ptr(keys, torch.int64), n, num_rows, _ptr(bag_offsets, torch.int32), num_bags,
                                                        _ptr(err), _stream()))
    return tuple(int(v) for v in err.tolist())


def np_util_stream_copy(dst: torch.Tensor, src: torch.Tensor) -> None:
    nbytes = src.numel() * src.element_size()
    _chk("np_util_stream_copy", lib.np_util_stream_copy(_ptr(dst), _ptr(src), nbytes, _stream()))


def np_tune_set(name: str, value: int) -> None:
    _chk("np_tune_set", lib.np_tune_set(name.encode(), int(value)))


def np_tune_get(name: str) -> int:
    return int(lib.np_tune_get(name.encode()))


def np_util_gather_rate(src: torch.Tensor, num_rows: int, n: int, seed: int, out: torch.Tensor) -> None:
    """n hashed reads of 256-byte rows from the first num_rows rows of ``src`` (fp32, row width 64), summed 64 at a time into out."""
    _chk("np_util_gather_rate", lib.np_util_gather_rate(_ptr(src, torch.float32), num_rows, n, seed, _ptr(out, torch.float32), _stream()))


def np_prof_enable(on: bool) -> None:
    lib.np_prof_enable(1 if on else 0)


def np_prof_only(names) -> None:
    """Restrict event timing to launches with these names (an iterable of str); None or empty lifts the restriction."""
    joined = ",".join(names) if names else ""
    lib.np_prof_only(joined.encode() if joined else None)


def np_prof_collect(max_entries: int = 4096):
    """-> list of (kernel name, milliseconds) in launch order since the last collect."""
    names = (ctypes.c_char_p * max_entries)()
    ms = (ctypes.c_float * max_entries)()
    k = lib.np_prof_collect(names, ms, max_entries)
    return [(names[i].decode(), float(ms[i])) for i in range(k)]
