"""The C-ABI library loads and exports every symbol that include/nestpipe.h declares; host-only entry
points (version, status text, workspace sizes, argument validation) behave without a GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "nestpipe.h")
LIB = os.path.join(ROOT, "paper_2604_06956_amd", "libnestpipe_hip.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2604_06956_amd import build
        build.build(verbose=False)
    import torch  # noqa: F401  (the library binds to the HIP runtime torch ships)
    return ctypes.CDLL(LIB)


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(np_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_five_calls():
    names = declared_symbols()
    for n in ("np_dedup", "np_route", "np_lookup_fwd", "np_lookup_bwd", "np_sparse_adagrad"):
        assert n in names


def test_every_declared_symbol_is_exported(lib):
    for name in declared_symbols():
        assert hasattr(lib, name), f"{name} declared in nestpipe.h but not exported"


def test_status_strings_and_version(lib):
    lib.np_status_string.restype = ctypes.c_char_p
    assert lib.np_status_string(0) == b"ok"
    for code in (-1, -2, -3, -4):
        assert len(lib.np_status_string(code)) > 3
    assert lib.np_version() >= 100


def test_tunables_are_host_only(lib):
    lib.np_tune_get.restype = ctypes.c_int64
    lib.np_tune_get.argtypes = [ctypes.c_char_p]
    lib.np_tune_set.restype = ctypes.c_int
    lib.np_tune_set.argtypes = [ctypes.c_char_p, ctypes.c_int64]
    assert lib.np_tune_get(b"emit_order_min_n") == 1 << 22
    assert lib.np_tune_get(b"nope") == -1 and lib.np_tune_get(None) == -1
    assert lib.np_tune_set(b"nope", 1) == -1 and lib.np_tune_set(b"emit_order_min_n", -1) == -1
    assert lib.np_tune_set(b"emit_order_min_n", 77) == 0 and lib.np_tune_get(b"emit_order_min_n") == 77
    assert lib.np_tune_set(b"emit_order_min_n", 1 << 22) == 0


def test_workspace_sizes_are_monotone_and_aligned(lib):
    f = lib.np_dedup_workspace_bytes
    f.restype = ctypes.c_size_t
    f.argtypes = [ctypes.c_int32, ctypes.c_int32]
    assert f(0, 30) == 0
    a, b, c = f(1000, 30), f(100000, 30), f(100000, 40)
    assert 0 < a < b < c and a % 256 == 0 and c % 256 == 0
    assert f(41_900_000, 30) < 700 * 2 ** 20           # ~12 bytes per key plus the histogram matrix
    g = lib.np_lookup_bwd_workspace_bytes
    g.restype = ctypes.c_size_t
    g.argtypes = [ctypes.c_int32] * 4
    assert g(10, 1000, 64, 0) > 4 * 1000 and g(10, 0, 64, 0) == 0
    r = lib.np_route_workspace_bytes
    r.restype = ctypes.c_size_t
    r.argtypes = [ctypes.c_int32, ctypes.c_int32]
    assert r(1000, 1536) >= 1536 * 4 and r(1000, 5000) == 0


def test_bad_arguments_are_rejected_before_any_launch(lib):
    """Validation happens on the host: these calls return an error code without touching a device."""
    vp = ctypes.c_void_p
    lib.np_dedup.restype = ctypes.c_int
    lib.np_dedup.argtypes = [vp, ctypes.c_int32, ctypes.c_int32, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    assert lib.np_dedup(None, 10, 30, None, None, None, None, None, None, None, 0, None) == -1
    assert lib.np_dedup(None, -1, 30, None, None, None, 8, None, 8, None, 0, None) == -1
    assert lib.np_dedup(8, 10, 0, 8, 8, 8, 8, 8, 8, None, 0, None) == -1          # key_bits out of range
    assert lib.np_dedup(8, 10, 30, 8, 8, 8, 8, 8, 8, None, 0, None) == -2         # no workspace
    assert lib.np_dedup(8, 10, 30, 8, 8, 8, 8, 8, 8, 256, 16, None) == -2         # workspace too small
    lib.np_sparse_adagrad.restype = ctypes.c_int
    lib.np_sparse_adagrad.argtypes = [vp, vp, ctypes.c_int64, ctypes.c_int32, vp, vp, vp, ctypes.c_int32, ctypes.c_float,
                                      ctypes.c_float, vp]
    assert lib.np_sparse_adagrad(16, 16, 100, 6, 16, 16, 16, 10, 0.01, 1e-8, None) == -3      # dim not a multiple of 4
    assert lib.np_sparse_adagrad(16, 16, 100, 2048, 16, 16, 16, 10, 0.01, 1e-8, None) == -3   # dim too large
    assert lib.np_sparse_adagrad(None, 16, 100, 64, 16, 16, 16, 10, 0.01, 1e-8, None) == -1
    lib.np_route.restype = ctypes.c_int
    lib.np_route.argtypes = [vp, vp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, vp, vp, vp, vp, vp, vp, ctypes.c_int32, vp,
                             vp, ctypes.c_size_t, vp]
    assert lib.np_route(8, 8, 10, 0, 0, 8, 8, 8, 8, 8, None, 0, None, 256, 1 << 20, None) == -1      # no shards
    assert lib.np_route(8, 8, 10, 8, 7, 8, 8, 8, 8, 8, None, 0, None, 256, 1 << 20, None) == -1      # bad rule
    assert lib.np_route(8, 8, 10, 5000, 0, 8, 8, 8, 8, 8, None, 0, None, 256, 1 << 20, None) == -3   # too many shards
    assert lib.np_route(8, 8, 10, 8, 0, 8, 8, 8, 8, 8, 8, 5, None, 256, 1 << 20, None) == -1         # inverse without output
    lib.np_route_static.restype = ctypes.c_int
    lib.np_route_static.argtypes = [vp, vp, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, vp, vp, vp, vp, vp, vp, ctypes.c_int32, vp, vp]
    assert lib.np_route_static(8, 8, 10, 2049, 0, 8, 8, 8, 8, 8, None, 0, None, None) == -3   # beyond the built-in scratch
    assert lib.np_route_static(8, 8, 10, 0, 0, 8, 8, 8, 8, 8, None, 0, None, None) == -1      # no shards
    lib.np_lookup_fwd.restype = ctypes.c_int
    lib.np_lookup_fwd.argtypes = [vp, ctypes.c_int64, ctypes.c_int32, vp, vp, ctypes.c_int32, vp, vp, ctypes.c_int32,
                                  ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, vp, vp, vp, ctypes.c_size_t, vp]
    assert lib.np_lookup_fwd(16, 100, 64, 16, None, 0, None, 16, 4, 10, 2, 0, 0, 16, None, None, 0, None) == -1  # SEQ, max_len 0
    assert lib.np_lookup_fwd(16, 100, 64, 16, None, 0, None, 16, 4, 10, 5, 1, 0, 16, None, None, 0, None) == -1  # bad mode
    assert lib.np_lookup_fwd(16, 100, 6, 16, None, 0, None, 16, 4, 10, 0, 1, 0, 16, None, None, 0, None) == -3   # dim
    assert lib.np_lookup_fwd(20, 100, 64, 16, None, 0, None, 16, 4, 10, 0, 1, 0, 16, None, None, 0, None) == -1  # misaligned table
    assert lib.np_lookup_fwd(16, 100, 64, None, None, 0, None, 16, 4, 10, 0, 1, 0, 16, None, None, 0, None) == -1  # neither list nor idx


def test_header_is_plain_c(tmp_path):
    """include/nestpipe.h is a C header: a C99 translation unit that includes it and takes the address of every
    declared function compiles with gcc (no C++-only constructs, no missing includes)."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    names = declared_symbols()
    src = tmp_path / "use_header.c"
    refs = "\n".join(f"    p[{i}] = (void (*)(void))&{n};" for i, n in enumerate(names))
    src.write_text('#include "nestpipe.h"\n'
                   f"void (*p[{len(names)}])(void);\n"
                   "void take_addresses(void) {\n" + refs + "\n}\n"
                   "int status_is_int[sizeof(np_status) >= 1 ? 1 : -1];\n")
    r = subprocess.run([gcc, "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), "-c", str(src), "-o",
                        str(tmp_path / "use_header.o")], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
