"""Synthetic stand-ins for production user-interaction-history (UIH) batches.

The paper's workloads are production UIH sequences (Section 2.2, Section 2.3) that are
not public; its own micro-benchmark of prioritized updates also uses synthetic data
(Section 5.2).  The five configurations below reproduce their structure: jagged batches
with heavy-tailed sequence lengths, heavy-tailed (Zipf) row popularity that makes
consecutive iterations share "collision rows", and per-occurrence gradients.

Everything is drawn from ``numpy.random.Generator(PCG64(seed))`` with
``seed = 0xF5CA1E00 + config_index`` consumed in a fixed order: for each iteration t,
for each table: lengths, then IDs, then gradients.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

SEED_BASE = 0xF5CA1E00


# --------------------------------------------------------------------------------------
# configuration records
# --------------------------------------------------------------------------------------
@dataclass(frozen=True)
class TableSpec:
    num_rows: int
    dim: int
    dtype: str          # "f32" | "bf16"   (weights; Adagrad state is always f32)
    zipf_alpha: float
    init: str           # "normal0.01" (host generated) | "hash" (integer-hash rule)


@dataclass(frozen=True)
class WorkloadConfig:
    index: int
    name: str
    tables: Tuple[TableSpec, ...]
    batch: int
    length_rule: str            # "uniform" | "powerlaw" | "skew5pct"
    length_lo: int
    length_hi: int
    length_alpha: float = 1.5
    iterations: int = 2
    drift: bool = False         # rotate the hot 1% of ranks each iteration
    lr: float = 0.01
    eps: float = 1e-8


CONFIGS: Tuple[WorkloadConfig, ...] = (
    WorkloadConfig(0, "tiny",
                   (TableSpec(10_000, 64, "f32", 1.1, "normal0.01"),),
                   batch=32, length_rule="uniform", length_lo=1, length_hi=64),
    WorkloadConfig(1, "shard4M_d128",
                   (TableSpec(4_000_000, 128, "f32", 1.05, "hash"),),
                   batch=1024, length_rule="powerlaw", length_lo=16, length_hi=4096),
    WorkloadConfig(2, "multi8",
                   tuple(TableSpec(r * 1_000_000, d, "f32", a, "hash") for r, d, a in zip(
                       (1, 2, 4, 4, 8, 8, 16, 16),
                       (64, 128, 256, 64, 128, 256, 64, 128),
                       (1.0, 1.05, 1.1, 1.1, 1.15, 1.2, 1.15, 1.2))),
                   batch=2048, length_rule="powerlaw", length_lo=1, length_hi=8192),
    WorkloadConfig(3, "longseq_bf16",
                   (TableSpec(32_000_000, 128, "bf16", 1.2, "hash"),),
                   batch=512, length_rule="skew5pct", length_lo=8, length_hi=256),
    WorkloadConfig(4, "stream64M",
                   (TableSpec(64_000_000, 128, "f32", 1.05, "hash"),),
                   batch=4096, length_rule="powerlaw", length_lo=1, length_hi=4096,
                   iterations=10, drift=True),
)

LONG_UIH = 16_384           # the 5% long users of the skewed configuration


@dataclass
class Iteration:
    """One iteration's inputs for one table."""
    values: np.ndarray      # int64 [N]   row IDs, jagged by ``offsets``
    offsets: np.ndarray     # int64 [B+1]
    grads: Optional[np.ndarray]   # float32 [N, D] per-occurrence gradients (None if skipped)


# --------------------------------------------------------------------------------------
# distributions
# --------------------------------------------------------------------------------------
_cdf_cache: Dict[Tuple[float, int], np.ndarray] = {}


def _zipf_cdf(alpha: float, num_rows: int) -> np.ndarray:
    key = (float(alpha), int(num_rows))
    cdf = _cdf_cache.get(key)
    if cdf is None:
        k = np.arange(1, num_rows + 1, dtype=np.float64)
        w = k ** (-alpha)
        cdf = np.cumsum(w)
        cdf /= cdf[-1]
        _cdf_cache.clear()          # keep at most one big table alive
        _cdf_cache[key] = cdf
    return cdf


def bounded_zipf_ranks(rng: np.random.Generator, n: int, alpha: float, num_rows: int) -> np.ndarray:
    """n ranks k in [1, num_rows] with P(k) proportional to k**-alpha (inverse CDF)."""
    cdf = _zipf_cdf(alpha, num_rows)
    u = rng.random(n)
    k = np.searchsorted(cdf, u, side="left").astype(np.int64) + 1
    return np.minimum(k, num_rows)


def _affine_params(num_rows: int) -> Tuple[int, int]:
    a = int(0.6180339887498949 * num_rows) | 1
    while math.gcd(a, num_rows) != 1:
        a += 2
    b = num_rows // 3
    return a, b


def rank_to_row(ranks: np.ndarray, num_rows: int, iteration: int = 0, drift: bool = False) -> np.ndarray:
    """Scatter popularity ranks over the table through a fixed affine bijection.

    With ``drift`` the hottest 1% of ranks are rotated inside their block by a tenth of
    the block per iteration, so the set of hot rows is fixed while their order drifts.
    """
    pos = ranks.astype(np.int64) - 1
    if drift:
        hot = max(num_rows // 100, 1)
        shift = iteration * ((hot + 9) // 10)
        pos = np.where(pos < hot, (pos + shift) % hot, pos)
    a, b = _affine_params(num_rows)
    # a*pos < 2**63 for every configuration here (64e6 * 40e6 = 2.6e15)
    return (a * pos + b) % num_rows


def powerlaw_lengths(rng: np.random.Generator, n: int, alpha: float, lo: int, hi: int) -> np.ndarray:
    """Integer lengths: density proportional to x**-alpha on [lo, hi+1), floored."""
    u = rng.random(n)
    e = 1.0 - alpha
    a, b = float(lo) ** e, float(hi + 1) ** e
    x = (a + u * (b - a)) ** (1.0 / e)
    return np.clip(np.floor(x).astype(np.int64), lo, hi)


def _lengths(rng: np.random.Generator, cfg: WorkloadConfig, batch: int) -> np.ndarray:
    if cfg.length_rule == "uniform":
        return rng.integers(cfg.length_lo, cfg.length_hi + 1, size=batch, dtype=np.int64)
    if cfg.length_rule == "powerlaw":
        return powerlaw_lengths(rng, batch, cfg.length_alpha, cfg.length_lo, cfg.length_hi)
    if cfg.length_rule == "skew5pct":
        lens = rng.integers(cfg.length_lo, cfg.length_hi + 1, size=batch, dtype=np.int64)
        n_long = int(round(0.05 * batch))
        who = rng.choice(batch, size=n_long, replace=False)
        lens[who] = LONG_UIH
        return lens
    raise ValueError(cfg.length_rule)


def make_iterations(cfg: WorkloadConfig, iterations: Optional[int] = None, batch: Optional[int] = None,
                    with_grads: bool = True, tables: Optional[Sequence[int]] = None,
                    seed_offset: int = 0) -> List[List[Iteration]]:
    """Returns ``out[t][table]`` for t in range(iterations).

    ``batch`` scales the number of users down for parity-sized cases; ``tables`` restricts
    which tables get gradients materialised (random numbers for the others are still drawn
    so the streams stay aligned).
    """
    rng = np.random.Generator(np.random.PCG64(SEED_BASE + cfg.index + seed_offset))
    n_it = cfg.iterations if iterations is None else iterations
    B = cfg.batch if batch is None else batch
    out: List[List[Iteration]] = []
    for t in range(n_it):
        per_table = []
        for ti, tab in enumerate(cfg.tables):
            lens = _lengths(rng, cfg, B)
            offsets = np.zeros(B + 1, dtype=np.int64)
            np.cumsum(lens, out=offsets[1:])
            n = int(offsets[-1])
            ranks = bounded_zipf_ranks(rng, n, tab.zipf_alpha, tab.num_rows)
            values = rank_to_row(ranks, tab.num_rows, iteration=t, drift=cfg.drift)
            want = with_grads and (tables is None or ti in tables)
            if with_grads:
                g = rng.standard_normal((n, tab.dim), dtype=np.float32)
                grads = g if want else None
            else:
                grads = None
            per_table.append(Iteration(values=values, offsets=offsets, grads=grads))
        out.append(per_table)
    return out


# --------------------------------------------------------------------------------------
# table initialisation rule (an input generator: counter-based, reproducible per element)
# --------------------------------------------------------------------------------------
def mix32(x: np.ndarray) -> np.ndarray:
    """A fixed 32-bit integer finaliser (xorshift-multiply)."""
    x = x.astype(np.uint32, copy=True)
    x ^= x >> np.uint32(16)
    x *= np.uint32(0x7FEB352D)
    x ^= x >> np.uint32(15)
    x *= np.uint32(0x846CA68B)
    x ^= x >> np.uint32(16)
    return x


def hash_init_rows(rows: np.ndarray, dim: int, dtype: str) -> np.ndarray:
    """Initial weights of the listed rows under the integer-hash rule.

    element index e = row*dim + col (64 bit); h = mix32(lo32(e) ^ mix32(hi32(e) + 0x9E3779B9))
    f32 : ((h & 0xFFFF) - 32768) * 2**-22        (exact in fp32, |w| < 0.0079)
    bf16: ((h & 0xFF)   - 128)   * 2**-14        (8 significant bits: exact in bf16)
    Returns float32 values (for bf16 tables they are exactly representable in bf16).
    """
    rows = np.asarray(rows, dtype=np.uint64).reshape(-1, 1)
    e = rows * np.uint64(dim) + np.arange(dim, dtype=np.uint64).reshape(1, -1)
    lo = (e & np.uint64(0xFFFFFFFF)).astype(np.uint32)
    hi = (e >> np.uint64(32)).astype(np.uint32)
    with np.errstate(over="ignore"):
        h = mix32(lo ^ mix32(hi + np.uint32(0x9E3779B9)))
    if dtype == "f32":
        return ((h & np.uint32(0xFFFF)).astype(np.int32) - 32768).astype(np.float32) * np.float32(2.0 ** -22)
    if dtype == "bf16":
        return ((h & np.uint32(0xFF)).astype(np.int32) - 128).astype(np.float32) * np.float32(2.0 ** -14)
    raise ValueError(dtype)


def compact_rows(id_arrays: Sequence[np.ndarray]) -> Tuple[np.ndarray, List[np.ndarray]]:
    """Order-preserving renumbering of the rows touched by a set of ID arrays.

    Returns (touched_rows ascending, [ids remapped to their index in touched_rows]).
    Because the map is strictly increasing, ascending ID order is preserved, so results
    computed on the compact table map back to the full table row by row.
    """
    touched = np.unique(np.concatenate([np.asarray(a, dtype=np.int64) for a in id_arrays]))
    remapped = [np.searchsorted(touched, np.asarray(a, dtype=np.int64)) for a in id_arrays]
    return touched, remapped
