"""Do the oracle's pins have teeth?  Each case below plants one plausible mistake in a copy of oracle/np_oracle.c (a
dropped term, a wrong sign, an index off by one, a transposed operand, a convention read the other way), builds it, and
runs the oracle's own CPU tests against that build: they must fail.  The untouched source, built the same way, must
pass.  Every planted mistake stays inside the arrays the function owns (no out-of-bounds access), runs on the CPU only
and never reaches the GPU path."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "np_oracle.c")

# (name, text in np_oracle.c, replacement, test files whose pins must notice)
MUTANTS = [
    ("dedup: positions descend inside a key", "if (x->pos != y->pos) return x->pos < y->pos ? -1 : 1;",
     "if (x->pos != y->pos) return x->pos < y->pos ? 1 : -1;", ["test_oracle_dedup.py"]),
    ("dedup: keys descend", "if (x->key != y->key) return x->key < y->key ? -1 : 1;",
     "if (x->key != y->key) return x->key < y->key ? 1 : -1;", ["test_oracle_dedup.py"]),
    ("dedup: inverse off by one", "inverse[p[i].pos] = U - 1;", "inverse[p[i].pos] = U > 1 ? U - 2 : 0;", ["test_oracle_dedup.py"]),
    ("dedup: segment starts off by one", "occ_offsets[U] = i;\n", "occ_offsets[U] = i > 0 ? i - 1 : 0;\n", ["test_oracle_dedup.py"]),
    ("dedup: multiplicity not counted", "counts[U - 1] += 1;", "counts[U - 1] = 1;", ["test_oracle_dedup.py"]),
    ("mix: second shift 28 instead of 29", "a ^= a >> 29;", "a ^= a >> 28;", ["test_oracle_route.py"]),
    ("mix: first xor-shift dropped", "a ^= a >> 32;", "a ^= 0;", ["test_oracle_route.py"]),
    ("mix: multiplier with one bit changed", "0x9E3779B97F4A7C15ull", "0x9E3779B97F4A7C17ull", ["test_oracle_route.py"]),
    ("shard: hash applied under the modulo rule", "if (shard_fn == REF_SHARD_HASH) k = np_ref_mix(k);",
     "if (shard_fn == REF_SHARD_MOD) k = np_ref_mix(k);", ["test_oracle_route.py"]),
    ("route: the two permutations exchanged", "send_from_unique[p] = u;\n        unique_to_send[u] = p;",
     "send_from_unique[u] = p;\n        unique_to_send[p] = u;", ["test_oracle_route.py"]),
    ("route: keys descend inside a bucket", "for (int32_t u = 0; u < U; ++u) {\n        int32_t s = np_ref_shard(",
     "for (int32_t u = U - 1; u >= 0; --u) {\n        int32_t s = np_ref_shard(", ["test_oracle_route.py"]),
    ("route: send buffer filled in unique order", "send_keys[p] = unique[u];", "send_keys[p] = unique[p];", ["test_oracle_route.py"]),
    ("fwd: mean pooling does not divide", "v /= (double)len;", "v /= 1.0;", ["test_oracle_fwd.py"]),
    ("fwd: the slot indirection is ignored", "int32_t slot = idx ? idx[j] : j;", "int32_t slot = idx ? idx[lo] : j;",
     ["test_oracle_fwd.py"]),
    ("fwd: sequence output transposed inside a bag", "size_t o = (size_t)b * per_bag + (size_t)p * (size_t)dim + (size_t)d;",
     "size_t o = (size_t)b * per_bag + (size_t)d * (size_t)max_len + (size_t)p;", ["test_oracle_fwd.py"]),
    ("fwd: absolute values summed into the result", "acc[d] += v;", "acc[d] += fabs(v);", ["test_oracle_fwd.py"]),
    ("bf16: ties away from zero", "b += 0x7FFFu + lsb;", "b += 0x8000u;", ["test_oracle_fwd.py"]),
    ("bwd: mean weight dropped", "double w = (mode == REF_POOL_MEAN && len > 0) ? 1.0 / (double)len : 1.0;", "double w = 1.0;",
     ["test_oracle_bwd.py"]),
    ("bwd: sequence position ignored", "((size_t)b * (size_t)max_len + (size_t)(j - lo)) * (size_t)dim", "((size_t)b * (size_t)max_len) * (size_t)dim",
     ["test_oracle_bwd.py"]),
    ("bwd: send-order placement ignored", "(size_t)(unique_to_send ? unique_to_send[u] : u) * (size_t)dim", "(size_t)u * (size_t)dim",
     ["test_oracle_bwd.py"]),
    ("bwd: sign", "acc[dst + d] += w * y;", "acc[dst + d] -= w * y;", ["test_oracle_bwd.py"]),
    ("bwd: bf16 gradient read with the halves exchanged", "(double)np_ref_bf16_to_f32(((const uint16_t*)dY)[src + d])",
     "(double)np_ref_bf16_to_f32(((const uint16_t*)dY)[src + (d ^ 1)])", ["test_oracle_bwd.py"]),
    ("adagrad: sum of squares instead of their mean", "double G = (double)state[k] + ss / (double)dim;\n        state[k] = (float)G;\n        double denom = sqrt(G) + (double)eps;\n        float* w",
     "double G = (double)state[k] + ss;\n        state[k] = (float)G;\n        double denom = sqrt(G) + (double)eps;\n        float* w",
     ["test_oracle_adagrad.py"]),
    ("adagrad: eps inside the square root", "double denom = sqrt(G) + (double)eps;\n        float* w", "double denom = sqrt(G + (double)eps);\n        float* w",
     ["test_oracle_adagrad.py"]),
    ("adagrad: step added", "w[d] = (float)((double)w[d] - (double)lr * (double)g[d] / denom);", "w[d] = (float)((double)w[d] + (double)lr * (double)g[d] / denom);",
     ["test_oracle_adagrad.py"]),
    ("adagrad: state overwritten instead of accumulated", "state[k] = (float)G;\n        double denom = sqrt(G) + (double)eps;\n        float* w",
     "state[k] = (float)(ss / (double)dim);\n        double denom = sqrt(G) + (double)eps;\n        float* w", ["test_oracle_adagrad.py", "test_oracle_step.py"]),
    ("16-bit tables: rounded through fp32 first (two roundings)", "w[d] = table_dtype == REF_BF16 ? np_ref_f64_to_bf16(upd) : np_ref_f64_to_f16(upd);",
     "w[d] = table_dtype == REF_BF16 ? np_ref_f32_to_bf16((float)upd) : np_ref_f64_to_f16((double)(float)upd);",
     ["test_oracle_bf16_table.py", "test_oracle_f16_table.py"]),
    ("fp16: one significant bit too few", "double r = ref_round_sig(a, 11, -24);", "double r = ref_round_sig(a, 10, -24);", ["test_oracle_f16_table.py"]),
    ("bwd: tolerance scale inflated", "if (abs_out) abs_out[dst + d] += fabs(w * y);", "if (abs_out) abs_out[dst + d] += 16.0 * fabs(w * y);",
     ["test_oracle_bwd.py"]),
    ("fwd: tolerance scale inflated", "aab[d] += fabs(v);", "aab[d] += 16.0 * fabs(v);", ["test_oracle_fwd.py"]),
    ("compose: the send permutation is not applied", "lookup_to_send[j] = unique_to_send[inverse[j]];", "lookup_to_send[j] = inverse[j];",
     ["test_oracle_route.py"]),
    ("fwd: rows_out copied by slot instead of by key", "memcpy(rows_out + (size_t)p * (size_t)dim, table + (size_t)row * (size_t)dim,",
     "memcpy(rows_out + (size_t)p * (size_t)dim, table + (size_t)p * (size_t)dim,", ["test_oracle_fwd.py"]),
    ("fp16 decoder: exponent bias off by one", "else v = ldexp(1.0 + (double)f / 1024.0, e - 15);", "else v = ldexp(1.0 + (double)f / 1024.0, e - 14);",
     ["test_oracle_f16_table.py"]),
    ("bf16 from fp64: subnormal spacing of the wrong format", "double r = ref_round_sig(a, 8, -133);", "double r = ref_round_sig(a, 8, -126);",
     ["test_oracle_bf16_table.py"]),
    ("dedup: empty batch leaves the count unset", "*num_unique = 0;\n        occ_offsets[0] = 0;", "occ_offsets[0] = 0;", ["test_oracle_dedup.py"]),
    ("intersect: indices of the second list off by one", "idx_b[c] = j;", "idx_b[c] = j > 0 ? j - 1 : 0;", ["test_oracle_dbsync.py"]),
    ("sync_rows: source and destination rows exchanged", "memcpy(dst + (size_t)dst_idx[i] * (size_t)dim, src + (size_t)src_idx[i] * (size_t)dim,",
     "memcpy(dst + (size_t)dst_idx[i] * (size_t)dim, src + (size_t)src_idx[count - 1 - i] * (size_t)dim,", ["test_oracle_dbsync.py"]),
]


def _build(text: str, path: str) -> None:
    src = path + ".c"
    with open(src, "w") as f:
        f.write(text)
    subprocess.run(["gcc", "-std=c11", "-O1", "-fPIC", "-shared", "-o", path, src, "-lm"], check=True, capture_output=True)


def _run_pins(lib: str, files) -> subprocess.CompletedProcess:
    env = dict(os.environ, NP_ORACLE_LIB=lib)
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider"] + [os.path.join(ROOT, "tests", f) for f in files]
    return subprocess.run(cmd, env=env, cwd=ROOT, capture_output=True, text=True, timeout=900)


ALL_PIN_FILES = ["test_oracle_dedup.py", "test_oracle_route.py", "test_oracle_fwd.py", "test_oracle_bwd.py", "test_oracle_adagrad.py",
                 "test_oracle_step.py", "test_oracle_dbsync.py", "test_oracle_bf16_table.py", "test_oracle_f16_table.py",
                 "test_oracle_second_form.py"]


def test_the_untouched_source_passes_when_built_this_way(tmp_path):
    lib = str(tmp_path / "libnp_oracle_plain.so")
    _build(open(SRC).read(), lib)
    r = _run_pins(lib, ALL_PIN_FILES)
    assert r.returncode == 0, r.stdout[-3000:]


def test_every_planted_mistake_is_noticed(tmp_path):
    text = open(SRC).read()
    jobs = []
    for i, (name, old, new, files) in enumerate(MUTANTS):
        assert text.count(old) >= 1, f"mutation site not found: {name}"
        lib = str(tmp_path / f"mutant{i}.so")
        _build(text.replace(old, new), lib)
        jobs.append((name, lib, files))
    with ThreadPoolExecutor(max_workers=4) as pool:
        results = list(pool.map(lambda j: _run_pins(j[1], j[2]), jobs))
    survivors = [name for (name, _, _), r in zip(jobs, results) if r.returncode == 0]
    assert not survivors, "no pin notices: " + "; ".join(survivors)
    # the failures are test failures, not crashes of the harness (pytest exit code 1)
    odd = [(name, r.returncode) for (name, _, _), r in zip(jobs, results) if r.returncode not in (1,)]
    assert not odd, odd
