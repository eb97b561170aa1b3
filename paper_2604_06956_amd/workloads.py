"""Seeded synthetic workloads for the sparse-embedding hot path.

This module only *generates inputs*: key batches with a bounded-Zipf popularity law, bag
lengths, upstream gradients and the stateless table initialiser.  It holds none of the
method's arithmetic (no dedup, routing hash, pooling, reduction or optimizer step) and
imports neither the HIP binding nor the CPU oracle, so both sides can be fed from it.

The paper states only that embedding accesses are highly skewed (Section IV-A) and
measures on a public and a proprietary click log; the batches built here stand in for
those logs with the shapes, popularity exponents and length mixes of the five benchmark
configurations.

Everything is numpy with ``np.random.Generator(PCG64(seed))``.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional, Tuple

import numpy as np

BASE_SEED = 20260406

# ----------------------------------------------------------------------------------------
# Stateless table initialiser (a counter-based generator).
#
# value(row, col) depends only on (row * dim + col, seed): the GPU fills a 205 GB table
# with a kernel that evaluates the same integer recipe, and the tests evaluate it here for
# just the rows a batch touches.  The result is an integer in [-2^23, 2^23) times one
# constant, so it is exactly representable and identical on every platform.
# ----------------------------------------------------------------------------------------
_INIT_M1 = np.uint64(0xD6E8FEB86659FD93)
_INIT_M2 = np.uint64(0xA3B195354A39B70D)
_INIT_S0 = np.uint64(0x2545F4914F6CDD1D)
TABLE_INIT_SCALE = np.float32(0.01) / np.float32(8388608.0)


def table_init_hash(counter: np.ndarray, seed: int) -> np.ndarray:
    """64-bit scramble of ``counter`` (uint64 array) under ``seed``; wraps mod 2^64."""
    with np.errstate(over="ignore"):
        h = counter.astype(np.uint64) + np.uint64(seed & 0xFFFFFFFFFFFFFFFF) * _INIT_S0
        h ^= h >> np.uint64(31)
        h *= _INIT_M1
        h ^= h >> np.uint64(27)
        h *= _INIT_M2
        h ^= h >> np.uint64(33)
    return h


def table_init_rows(rows: np.ndarray, dim: int, seed: int) -> np.ndarray:
    """fp32 ``[len(rows), dim]`` initial values of the given table rows, uniform on [-0.01, 0.01)."""
    rows = np.asarray(rows, dtype=np.int64).astype(np.uint64)
    cols = np.arange(dim, dtype=np.uint64)
    out = np.empty((rows.shape[0], dim), dtype=np.float32)
    step = max(1, (1 << 24) // max(dim, 1))          # bound the uint64 temporaries to ~128 MB each
    for a in range(0, rows.shape[0], step):
        with np.errstate(over="ignore"):
            counter = rows[a:a + step, None] * np.uint64(dim) + cols[None, :]
        h = table_init_hash(counter, seed)
        q = (h >> np.uint64(40)).astype(np.int64) - 8388608  # 24 bits -> [-2^23, 2^23)
        out[a:a + step] = q.astype(np.float32) * TABLE_INIT_SCALE
    return out


# ----------------------------------------------------------------------------------------
# Bounded Zipf sampler
# ----------------------------------------------------------------------------------------
_HEAD_MAX = 1 << 22


class BoundedZipf:
    """Ranks 1..R with p(r) proportional to r^-alpha.

    Head (ranks <= M = min(R, 2^22)): exact discrete CDF in fp64, inverted by search.
    Tail (ranks > M): mass of rank r approximated by the integral of x^-alpha over
    [r - 1/2, r + 1/2]; that integral is inverted analytically and rounded to a rank.
    """

    def __init__(self, num_ranks: int, alpha: float):
        if num_ranks < 1:
            raise ValueError("num_ranks must be >= 1")
        self.R = int(num_ranks)
        self.alpha = float(alpha)
        self.M = min(self.R, _HEAD_MAX)
        w = np.arange(1, self.M + 1, dtype=np.float64) ** (-self.alpha)
        self.head_cdf = np.cumsum(w)
        self.head_mass = float(self.head_cdf[-1])
        self.tail_mass = 0.0
        if self.R > self.M:
            self._lo = self.M + 0.5
            self._hi = self.R + 0.5
            self.tail_mass = self._integral(self._lo, self._hi)
        self.total_mass = self.head_mass + self.tail_mass

    def _integral(self, a: float, b: float) -> float:
        al = self.alpha
        if abs(al - 1.0) < 1e-12:
            return float(np.log(b) - np.log(a))
        return float((a ** (1.0 - al) - b ** (1.0 - al)) / (al - 1.0))

    def pmf_head(self) -> np.ndarray:
        """Probabilities of ranks 1..M."""
        return np.diff(self.head_cdf, prepend=0.0) / self.total_mass

    def sample(self, rng: np.random.Generator, size: int) -> np.ndarray:
        u = rng.random(size) * self.total_mass
        ranks = np.empty(size, dtype=np.int64)
        in_head = u < self.head_mass
        uh = u[in_head]
        r = np.searchsorted(self.head_cdf, uh, side="right") + 1
        ranks[in_head] = np.minimum(r, self.M)
        if self.R > self.M:
            v = u[~in_head] - self.head_mass
            al = self.alpha
            if abs(al - 1.0) < 1e-12:
                x = self._lo * np.exp(v)
            else:
                x = (self._lo ** (1.0 - al) - v * (al - 1.0)) ** (1.0 / (1.0 - al))
            rt = np.rint(x).astype(np.int64)
            ranks[~in_head] = np.clip(rt, self.M + 1, self.R)
        else:
            ranks[~in_head] = self.M
        return ranks


RANK_STRIDE = 4294967291  # prime just below 2^32: coprime with any table size below it


def ranks_to_ids(ranks: np.ndarray, num_rows: int, offset: int) -> np.ndarray:
    """Bijection ranks 1..R -> row ids 0..R-1 that scatters popular ranks over the table."""
    if num_rows >= RANK_STRIDE or num_rows > (1 << 30):
        raise ValueError("num_rows too large for the rank permutation")
    r = (ranks.astype(np.uint64) - np.uint64(1)) * np.uint64(RANK_STRIDE) + np.uint64(offset % num_rows)
    return (r % np.uint64(num_rows)).astype(np.int64)


# ----------------------------------------------------------------------------------------
# Configurations
# ----------------------------------------------------------------------------------------
POOL_SUM, POOL_MEAN, SEQ = 0, 1, 2
SHARD_MOD, SHARD_HASH = 0, 1


@dataclass(frozen=True)
class Config:
    name: str
    index: int                       # 1..5, enters the seed
    table_rows: Tuple[int, ...]      # rows per table (fused in this order)
    dim: int
    batch: int                       # samples
    features: int                    # bags per sample; feature f reads table f % len(table_rows)
    length_law: str                  # "uniform", "poisson_clip", "poisson", "fixed", "seq_uniform"
    length_args: Tuple[int, ...]
    alpha: float
    num_shards: int
    shard_fn: int
    mode: int
    lr: float = 0.01
    eps: float = 1e-8
    overlap: Optional[float] = None  # target |K1 & K2| / |K2| for the second batch
    table_seed: int = 7

    @property
    def num_rows(self) -> int:
        return int(sum(self.table_rows))

    @property
    def num_bags(self) -> int:
        return self.batch * self.features

    @property
    def key_bits(self) -> int:
        return max(1, int(self.num_rows - 1).bit_length())

    @property
    def table_base(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum(self.table_rows)[:-1]]).astype(np.int64)


def _dlrm_rows(seed: int = BASE_SEED + 2000 + 999) -> Tuple[int, ...]:
    rng = np.random.Generator(np.random.PCG64(seed))
    return tuple(int(x) for x in np.rint(10.0 ** rng.uniform(4.0, 7.0, size=26)))


def config(name: str) -> Config:
    """The five benchmark configurations at full size."""
    if name == "tiny":
        return Config("tiny", 1, (100_000,), 16, 256, 8, "uniform", (1, 20), 1.05, 8, SHARD_MOD, POOL_SUM)
    if name == "dlrm":
        return Config("dlrm", 2, _dlrm_rows(), 64, 16_384, 26, "poisson_clip", (4, 1, 64), 1.1, 64,
                      SHARD_HASH, POOL_MEAN)
    if name == "seq":
        return Config("seq", 3, (50_000_000,) * 4, 128, 4_096, 4, "seq_uniform", (200, 1000), 1.2, 1536,
                      SHARD_HASH, SEQ)
    if name == "skew":
        return Config("skew", 4, (200_000_000,), 64, 65_536, 1, "fixed", (32,), 1.5, 1536, SHARD_HASH, POOL_SUM)
    if name == "large":
        return Config("large", 5, (800_000_000,), 64, 131_072, 40, "poisson", (8,), 1.05, 1536, SHARD_HASH,
                      POOL_SUM, overlap=0.30)
    raise KeyError(name)


CONFIG_NAMES = ("tiny", "dlrm", "seq", "skew", "large")


def scaled(cfg: Config, row_div: int, batch_div: int) -> Config:
    """Same structure with fewer rows and samples (for cases the CPU oracle finishes in seconds)."""
    rows = tuple(max(64, r // row_div) for r in cfg.table_rows)
    return replace(cfg, name=f"{cfg.name}/r{row_div}b{batch_div}", table_rows=rows,
                   batch=max(1, cfg.batch // batch_div))


@dataclass
class Batch:
    keys: np.ndarray          # int64 [n], global (fused-table) row ids, bag-contiguous
    bag_offsets: np.ndarray   # int32 [B+1]
    max_len: int              # longest bag (>= 1)
    dY: np.ndarray            # fp32 [B, D] (pooled) or fp32 [B, max_len, D] holding bf16-exact values (SEQ)
    meta: Dict[str, float] = field(default_factory=dict)

    @property
    def n(self) -> int:
        return int(self.keys.shape[0])

    @property
    def num_bags(self) -> int:
        return int(self.bag_offsets.shape[0] - 1)


def _lengths(cfg: Config, rng: np.random.Generator) -> np.ndarray:
    B = cfg.num_bags
    law, a = cfg.length_law, cfg.length_args
    if law == "uniform":
        return rng.integers(a[0], a[1] + 1, size=B).astype(np.int64)
    if law == "poisson_clip":
        return np.clip(rng.poisson(a[0], size=B), a[1], a[2]).astype(np.int64)
    if law == "poisson":
        return rng.poisson(a[0], size=B).astype(np.int64)
    if law == "fixed":
        return np.full(B, a[0], dtype=np.int64)
    if law == "seq_uniform":
        per_sample = rng.integers(a[0], a[1] + 1, size=cfg.batch).astype(np.int64)
        return np.tile(per_sample, cfg.features)  # bag b = feature * batch + sample
    raise ValueError(law)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 values rounded to the nearest bf16 (ties to even), returned as fp32.  Input-prep only."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((b >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((b + r) & np.uint32(0xFFFF0000)).view(np.float32)


def _draw_keys(cfg: Config, rng: np.random.Generator, lengths: np.ndarray) -> np.ndarray:
    n = int(lengths.sum())
    keys = np.empty(n, dtype=np.int64)
    offs = np.concatenate([[0], np.cumsum(lengths)])
    T = len(cfg.table_rows)
    base = cfg.table_base
    samplers: Dict[int, BoundedZipf] = {}
    for f in range(cfg.features):
        t = f % T
        lo, hi = int(offs[f * cfg.batch]), int(offs[(f + 1) * cfg.batch])
        if hi == lo:
            continue
        R = cfg.table_rows[t]
        if R not in samplers:
            samplers[R] = BoundedZipf(R, cfg.alpha)
        ranks = samplers[R].sample(rng, hi - lo)
        keys[lo:hi] = ranks_to_ids(ranks, R, 12345 + 7919 * t) + base[t]
    return keys


def _force_overlap(keys2: np.ndarray, keys1: np.ndarray, target: float, num_rows: int,
                   rng: np.random.Generator) -> np.ndarray:
    """Substitute whole keys of batch 2 so that |K1 & K2| / |K2| hits ``target`` (multiplicities kept)."""
    K1 = np.unique(keys1)
    K2 = np.unique(keys2)
    both = np.intersect1d(K1, K2, assume_unique=True)
    want = int(round(target * K2.size))
    src = dst = None
    if both.size < want:
        m = want - both.size
        only2 = np.setdiff1d(K2, K1, assume_unique=True)
        only1 = np.setdiff1d(K1, K2, assume_unique=True)
        m = min(m, only2.size, only1.size)
        src = rng.choice(only2, size=m, replace=False)
        dst = rng.choice(only1, size=m, replace=False)
    elif both.size > want:
        m = both.size - want
        src = rng.choice(both, size=m, replace=False)
        union = np.union1d(K1, K2)
        fresh = np.empty(0, dtype=np.int64)
        while fresh.size < m:
            cand = np.unique(rng.integers(0, num_rows, size=2 * (m - fresh.size) + 16))
            cand = np.setdiff1d(cand, union, assume_unique=True)
            cand = np.setdiff1d(cand, fresh, assume_unique=True)
            fresh = np.concatenate([fresh, cand])
        dst = rng.permutation(fresh)[:m]
    if src is None or src.size == 0:
        return keys2
    order = np.argsort(src)
    src_s, dst_s = src[order], dst[order]
    pos = np.searchsorted(src_s, keys2)
    pos = np.minimum(pos, src_s.size - 1)
    hit = src_s[pos] == keys2
    out = keys2.copy()
    out[hit] = dst_s[pos[hit]]
    return out


def make_batch(cfg: Config, batch_index: int = 0, prev: Optional[Batch] = None,
               with_dy: bool = True) -> Batch:
    """Batch ``batch_index`` of ``cfg``.  With ``cfg.overlap`` set and ``prev`` given, keys are
    substituted so the distinct-key overlap with ``prev`` meets the target."""
    rng = np.random.Generator(np.random.PCG64(BASE_SEED + 1000 * cfg.index + batch_index))
    lengths = _lengths(cfg, rng)
    keys = _draw_keys(cfg, rng, lengths)
    meta: Dict[str, float] = {}
    if cfg.overlap is not None and prev is not None:
        keys = _force_overlap(keys, prev.keys, cfg.overlap, cfg.num_rows, rng)
    bag_offsets = np.concatenate([[0], np.cumsum(lengths)]).astype(np.int64)
    if bag_offsets[-1] >= 2 ** 31:
        raise ValueError("batch too large for int32 offsets")
    max_len = int(max(1, lengths.max() if lengths.size else 1))
    B, D = cfg.num_bags, cfg.dim
    if not with_dy:
        dY = np.empty((0, D), dtype=np.float32)
    elif cfg.mode == SEQ:
        dY = round_to_bf16(rng.standard_normal((B, max_len, D), dtype=np.float32))
    else:
        dY = rng.standard_normal((B, D), dtype=np.float32)
    return Batch(keys=keys, bag_offsets=bag_offsets.astype(np.int32), max_len=max_len, dY=dY, meta=meta)


def batch_stats(keys: np.ndarray) -> Dict[str, float]:
    """Realised n, U, U/n and hottest-key multiplicity of a key batch (a generator sanity record)."""
    if keys.size == 0:
        return {"n": 0, "U": 0, "U_over_n": 0.0, "hottest": 0}
    _, c = np.unique(keys, return_counts=True)
    return {"n": int(keys.size), "U": int(c.size), "U_over_n": float(c.size / keys.size), "hottest": int(c.max())}


def expected_unique(cfg_rows: int, alpha: float, n: int) -> float:
    """E[U] = sum_k 1 - exp(-n p_k) for one table (head exact, tail by the same integral split)."""
    z = BoundedZipf(cfg_rows, alpha)
    p = np.diff(z.head_cdf, prepend=0.0) / z.total_mass
    e = float(np.sum(-np.expm1(-n * p)))
    if z.R > z.M:
        # tail probabilities are tiny: 1 - exp(-n p) ~ n p - (n p)^2 / 2 ; integrate n p only when small
        r = np.unique(np.rint(np.geomspace(z.M + 1, z.R, 20000)).astype(np.int64))
        pr = r.astype(np.float64) ** (-alpha) / z.total_mass
        f = -np.expm1(-n * pr)
        e += float(np.trapezoid(f, r.astype(np.float64)))
    return e
