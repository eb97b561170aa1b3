"""np_route_static, the entry point that allocates nothing (for callers that cannot call hipMalloc: graph capture,
serving loops), against np_route: same kernels on the library's built-in scratch, so every output must match bit for
bit.  Two calls in a row on the one scratch array, the second with a smaller input and another shard count, then the
first again: what an earlier call left in the array must not matter."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import gpu_helpers
    return gpu_helpers


NAMES = ("send_keys", "splits", "send_offsets", "send_from_unique", "unique_to_send", "lookup_to_send")


def _case(H, U_target, S, fn, seed):
    import torch
    rng = np.random.default_rng(seed)
    unique = np.unique(rng.integers(0, 1 << 40, size=U_target)).astype(np.int64)
    U = unique.shape[0]
    cap = U + 37
    ubuf = np.zeros(cap, np.int64)
    ubuf[:U] = unique
    inv = rng.integers(0, U, size=3 * U + 5).astype(np.int32)
    d_unique, d_U, d_inv = H.dev(ubuf), H.dev(np.array([U], np.int32)), H.dev(inv)
    n = inv.shape[0]
    ref = H.B.np_route(d_unique, d_U, cap, S, fn, inverse=d_inv, n=n)
    i32, i64 = torch.int32, torch.int64
    # every output buffer exists before the call: the call itself allocates nothing, on either side of the C ABI
    out = dict(send_keys=torch.full((cap,), -1, dtype=i64, device="cuda"), splits=torch.full((S,), -1, dtype=i32, device="cuda"),
               send_offsets=torch.full((S + 1,), -1, dtype=i32, device="cuda"),
               send_from_unique=torch.full((cap,), -1, dtype=i32, device="cuda"),
               unique_to_send=torch.full((cap,), -1, dtype=i32, device="cuda"),
               lookup_to_send=torch.full((n,), -1, dtype=i32, device="cuda"))
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    H.B.np_route_static(d_unique, d_U, cap, S, fn, out, inverse=d_inv, n=n)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    sizes = dict(send_keys=U, splits=S, send_offsets=S + 1, send_from_unique=U, unique_to_send=U, lookup_to_send=n)
    for name in NAMES:
        k = sizes[name]
        assert H.host(out[name])[:k].tobytes() == H.host(ref[name])[:k].tobytes(), (name, U, S, fn)
    # the oracle as well, directly
    send_keys, splits, send_offsets, sfu, uts = H.O.route(unique, S, fn)
    assert np.array_equal(H.host(out["send_keys"])[:U], send_keys)
    assert np.array_equal(H.host(out["splits"]), splits)
    assert np.array_equal(H.host(out["unique_to_send"])[:U], uts)


def test_route_static_matches_route_on_two_calls_in_a_row(H):
    _case(H, 700_000, 1536, 1, seed=11)   # several chunks, hashed shards
    _case(H, 5_000, 7, 0, seed=12)        # smaller input, fewer (and an odd number of) shards, on the same scratch
    _case(H, 700_000, 2048, 1, seed=13)   # the largest shard count the built-in scratch covers


def test_route_static_limits(H):
    import torch
    U, S = 100, H.B.ROUTE_STATIC_MAX_SHARDS + 1
    i32, i64 = torch.int32, torch.int64
    out = dict(send_keys=torch.zeros(U, dtype=i64, device="cuda"), splits=torch.full((S,), -1, dtype=i32, device="cuda"),
               send_offsets=torch.zeros(S + 1, dtype=i32, device="cuda"), send_from_unique=torch.zeros(U, dtype=i32, device="cuda"),
               unique_to_send=torch.zeros(U, dtype=i32, device="cuda"))
    with pytest.raises(H.B.NestPipeError) as e:
        H.B.np_route_static(torch.arange(U, dtype=i64, device="cuda"), H.dev(np.array([U], np.int32)), U, S, 0, out)
    assert e.value.status == -3                       # NP_ERR_UNSUPPORTED, decided on the host
    torch.cuda.synchronize()
    assert (H.host(out["splits"]) == -1).all()        # nothing was enqueued
