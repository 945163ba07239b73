"""Seeded synthetic workloads shaped like click-log ranking batches.

A batch has F multi-hot categorical fields (hashed ids with a heavy-tailed,
bounded-Zipf frequency and a uniform bag length), a few dense N(0,1) features
and Bernoulli labels.  Parameters are drawn procedurally from a counter-based
mixer so that a single row of a table that is far too large for host memory
can still be evaluated on its own.

Nothing here is part of the training step's arithmetic.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace
from functools import lru_cache
from typing import List, Optional, Sequence, Tuple

import numpy as np

SEED0 = 20240409
TABLE_SCALE = 0.05  # embeddings ~ U(-0.05, 0.05)


# --------------------------------------------------------------------------
# configurations
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class RankingConfig:
    name: str
    num_fields: int
    rows_per_field: int
    dim: int
    table_dtype: str          # "f32" | "bf16"
    adagrad_state: str        # "elementwise" | "rowwise"
    num_dense: int
    layer_sizes: Tuple[int, ...]   # (input, hidden..., 1)
    gemm_dtype: str           # "f32" | "bf16"
    max_bag: int              # bag length ~ U{min_bag..max_bag}
    zipf_s: float
    shard_sizes: Tuple[int, ...]
    seed: int
    min_bag: int = 1
    lr: float = 0.01
    eps: float = 1e-8
    pooling: str = "sum"      # "sum" | "mean"

    @property
    def batch(self) -> int:
        return int(sum(self.shard_sizes))

    @property
    def num_shards(self) -> int:
        return len(self.shard_sizes)

    @property
    def input_width(self) -> int:
        return self.num_fields * self.dim + self.num_dense

    @property
    def num_params(self) -> int:
        s = self.layer_sizes
        return sum(s[i] * s[i + 1] + s[i + 1] for i in range(len(s) - 1))


@dataclass(frozen=True)
class DenseConfig:
    name: str
    n: int
    num_buffers: int
    grad_std: float
    param_std: float
    lr: float
    beta1: float
    beta2: float
    eps: float
    seed: int


CONFIGS = {
    1: RankingConfig("cfg1-tiny-ctr", 8, 10_000, 16, "f32", "elementwise", 13,
                     (141, 64, 32, 1), "f32", 4, 1.05, (64,) * 4, SEED0 + 1),
    2: RankingConfig("cfg2-26x1M-d32", 26, 1_000_000, 32, "f32", "elementwise", 13,
                     (845, 1024, 512, 256, 1), "bf16", 20, 1.1, (512,) * 8, SEED0 + 2),
    3: RankingConfig("cfg3-hetero-shards", 26, 1_000_000, 32, "f32", "elementwise", 13,
                     (845, 1024, 512, 256, 1), "bf16", 20, 1.1,
                     (512, 768, 1024, 1536, 2048, 2560, 3072, 4096), SEED0 + 3),
    4: RankingConfig("cfg4-100x10M-d64-bf16", 100, 10_000_000, 64, "bf16", "rowwise", 0,
                     (6400, 1024, 512, 1), "bf16", 50, 1.2, (1024,) * 16, SEED0 + 4),
}
DENSE_CONFIG = DenseConfig("cfg5-dense-adam", 1 << 28, 8, 1e-3, 0.02, 1e-3, 0.9, 0.999,
                           1e-8, SEED0 + 5)


def scaled(cfg: RankingConfig, **kw) -> RankingConfig:
    """A copy of a configuration with some fields replaced (smaller test shapes)."""
    return replace(cfg, **kw)


# --------------------------------------------------------------------------
# counter-based parameter values
# --------------------------------------------------------------------------
def fmix32(x: np.ndarray) -> np.ndarray:
    """The 32-bit finalisation mixer of MurmurHash3 (public domain, A. Appleby)."""
    x = np.asarray(x, dtype=np.uint32).copy()
    x ^= x >> np.uint32(16)
    x *= np.uint32(0x85EBCA6B)
    x ^= x >> np.uint32(13)
    x *= np.uint32(0xC2B2AE35)
    x ^= x >> np.uint32(16)
    return x


def table_values(f: int, rows: np.ndarray, dim: int, scale: float = TABLE_SCALE) -> np.ndarray:
    """Initial embedding rows of field f as float32 [len(rows), dim].

    value(f, r, d) = scale * (u * 2^-23 - 1) with u the top 24 bits of
    fmix32(fmix32(r + 0x9E3779B9*(f+1)) ^ (0x85EBCA6B*(d+1))).  The bracket is
    exact in float32, the product with `scale` is one IEEE rounding, so any
    implementation of the same definition agrees bit for bit.
    """
    rows = np.asarray(rows, dtype=np.int64)
    with np.errstate(over="ignore"):
        r32 = rows.astype(np.uint32) + np.uint32((0x9E3779B9 * (f + 1)) & 0xFFFFFFFF)
        h1 = fmix32(r32)
        dmul = (np.arange(1, dim + 1, dtype=np.uint64) * np.uint64(0x85EBCA6B)).astype(np.uint32)
        h = fmix32(h1[:, None] ^ dmul[None, :])
    u24 = (h >> np.uint32(8)).astype(np.float32)
    t = u24 * np.float32(2.0 ** -23) - np.float32(1.0)
    return (np.float32(scale) * t).astype(np.float32)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round to nearest even."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (b >> np.uint32(16)) & np.uint32(1)
    with np.errstate(over="ignore"):
        r = b + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def make_tables(cfg: RankingConfig) -> np.ndarray:
    """All tables as one [F*R, D] array: float32, or uint16 bf16 bit patterns."""
    F, R, D = cfg.num_fields, cfg.rows_per_field, cfg.dim
    out = np.empty((F * R, D), dtype=np.float32 if cfg.table_dtype == "f32" else np.uint16)
    step = 1 << 18
    for f in range(F):
        for r0 in range(0, R, step):
            r1 = min(R, r0 + step)
            v = table_values(f, np.arange(r0, r1), D)
            out[f * R + r0:f * R + r1] = v if cfg.table_dtype == "f32" else f32_to_bf16_bits(v)
    return out


def table_rows_f32(cfg: RankingConfig, f: int, rows: np.ndarray) -> np.ndarray:
    """Initial rows of field f as the float32 values the stored dtype holds."""
    v = table_values(f, rows, cfg.dim)
    if cfg.table_dtype == "bf16":
        v = bf16_bits_to_f32(f32_to_bf16_bits(v))
    return v


def param_layout(cfg: RankingConfig) -> List[Tuple[int, int, int, int]]:
    """[(w_offset, b_offset, fan_in, fan_out)] of the flat parameter vector.

    Layer l stores W_l as [fan_in, fan_out] row-major followed by b_l.
    """
    out, off = [], 0
    s = cfg.layer_sizes
    for i in range(len(s) - 1):
        out.append((off, off + s[i] * s[i + 1], s[i], s[i + 1]))
        off += s[i] * s[i + 1] + s[i + 1]
    return out


def make_mlp_params(cfg: RankingConfig) -> np.ndarray:
    """Flat float32 parameters: W_l ~ N(0, 2/fan_in), b_l ~ N(0, 0.01^2)."""
    rng = np.random.default_rng(cfg.seed * 7919 + 11)
    flat = np.empty(cfg.num_params, dtype=np.float32)
    for (wo, bo, fi, fo) in param_layout(cfg):
        flat[wo:bo] = rng.standard_normal(fi * fo).astype(np.float32) * np.float32(math.sqrt(2.0 / fi))
        flat[bo:bo + fo] = rng.standard_normal(fo).astype(np.float32) * np.float32(0.01)
    return flat


def split_params(cfg: RankingConfig, flat: np.ndarray):
    """Views [(W [in,out], b [out])] into a flat parameter-shaped vector."""
    return [(flat[wo:bo].reshape(fi, fo), flat[bo:bo + fo]) for (wo, bo, fi, fo) in param_layout(cfg)]


# --------------------------------------------------------------------------
# batches
# --------------------------------------------------------------------------
@dataclass
class Batch:
    ids: np.ndarray        # int32 [sum_f nnz_f], field-major, bags of a field in sample order
    field_ptr: np.ndarray  # int64 [F+1], start of each field's lookups inside ids
    offsets: np.ndarray    # int32 [F, B+1], bag boundaries relative to the field's start
    dense: np.ndarray      # float32 [B, num_dense]
    labels: np.ndarray     # float32 [B]

    @property
    def batch(self) -> int:
        return int(self.labels.shape[0])

    def field_ids(self, f: int) -> np.ndarray:
        return self.ids[self.field_ptr[f]:self.field_ptr[f + 1]]


@lru_cache(maxsize=8)
def _zipf_cdf(rows: int, s: float) -> np.ndarray:
    w = np.arange(1, rows + 1, dtype=np.float64) ** (-s)
    c = np.cumsum(w)
    c /= c[-1]
    return c


def _field_affine(f: int, rows: int) -> Tuple[int, int]:
    """A bijection rank -> row id of field f (scatters the hot ranks as hashing does)."""
    a = int(fmix32(np.array([f + 1], dtype=np.uint32))[0]) | 1
    while math.gcd(a, rows) != 1:
        a += 2
    c = int(fmix32(np.array([f + 0x51ED27], dtype=np.uint32))[0]) % rows
    return a, c


def make_batch(cfg: RankingConfig, index: int = 0, batch: Optional[int] = None) -> Batch:
    """Batch number `index` of a configuration (distinct index -> distinct batch)."""
    B = cfg.batch if batch is None else int(batch)
    F, R = cfg.num_fields, cfg.rows_per_field
    rng = np.random.default_rng([cfg.seed, index])
    cdf = _zipf_cdf(R, cfg.zipf_s)
    lens = rng.integers(cfg.min_bag, cfg.max_bag + 1, size=(F, B), dtype=np.int64)
    offsets = np.zeros((F, B + 1), dtype=np.int64)
    np.cumsum(lens, axis=1, out=offsets[:, 1:])
    field_ptr = np.zeros(F + 1, dtype=np.int64)
    np.cumsum(offsets[:, -1], out=field_ptr[1:])
    ids = np.empty(int(field_ptr[-1]), dtype=np.int32)
    for f in range(F):
        n = int(offsets[f, -1])
        rank = np.searchsorted(cdf, rng.random(n), side="left").astype(np.int64)
        np.minimum(rank, R - 1, out=rank)
        a, c = _field_affine(f, R)
        ids[field_ptr[f]:field_ptr[f + 1]] = ((rank * a + c) % R).astype(np.int32)
    dense = rng.standard_normal((B, cfg.num_dense)).astype(np.float32)
    labels = (rng.random(B) < 0.25).astype(np.float32)
    return Batch(ids, field_ptr, offsets.astype(np.int32), dense, labels)


def batch_from_bags(bags: Sequence[Sequence[Sequence[int]]], dense: np.ndarray,
                    labels: np.ndarray) -> Batch:
    """Build a Batch from explicit bags[f][s] = list of row ids (for hand-made cases)."""
    F, B = len(bags), len(labels)
    offsets = np.zeros((F, B + 1), dtype=np.int32)
    chunks, field_ptr = [], np.zeros(F + 1, dtype=np.int64)
    for f in range(F):
        assert len(bags[f]) == B
        flat = [i for bag in bags[f] for i in bag]
        offsets[f, 1:] = np.cumsum([len(bag) for bag in bags[f]])
        chunks.append(np.asarray(flat, dtype=np.int32))
        field_ptr[f + 1] = field_ptr[f] + len(flat)
    ids = np.concatenate(chunks) if chunks else np.zeros(0, np.int32)
    return Batch(ids.astype(np.int32), field_ptr, offsets,
                 np.asarray(dense, dtype=np.float32).reshape(B, -1),
                 np.asarray(labels, dtype=np.float32))


def shard_slices(sizes: Sequence[int]) -> List[Tuple[int, int]]:
    out, s = [], 0
    for n in sizes:
        out.append((s, int(n)))
        s += int(n)
    return out


# --------------------------------------------------------------------------
# dense (all-reduce style) problem
# --------------------------------------------------------------------------
def make_dense_problem(cfg: DenseConfig, n: Optional[int] = None, weights: Optional[Sequence[float]] = None):
    """(p, m, v, [g_k], w): parameters N(0, param_std), zero moments, K gradient buffers."""
    n = cfg.n if n is None else int(n)
    rng = np.random.default_rng([cfg.seed, n])
    p = (rng.standard_normal(n, dtype=np.float32) * np.float32(cfg.param_std)).astype(np.float32)
    grads = []
    for k in range(cfg.num_buffers):
        rk = np.random.default_rng([cfg.seed + k, n, 1])
        grads.append((rk.standard_normal(n, dtype=np.float32) * np.float32(cfg.grad_std)).astype(np.float32))
    if weights is None:
        w = np.full(cfg.num_buffers, 1.0 / cfg.num_buffers, dtype=np.float64)
    else:
        w = np.asarray(weights, dtype=np.float64)
    return p, np.zeros(n, np.float32), np.zeros(n, np.float32), grads, w
