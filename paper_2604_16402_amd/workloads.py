"""Seeded synthetic inputs for range-filtered search over a bucketed graph index.

This module only *makes inputs*: base vectors, scalar attributes, query vectors and query
ranges.  It holds none of the method's arithmetic (no distances, no graph, no search) and is
the one module that both the CPU oracle's tests and the HIP library's tests import, so that
both sides see byte-identical inputs.

The shapes stand in for the public vector benchmarks the paper evaluates on (Table 2:
96-, 128-, 960-dimensional descriptors, one million base vectors, Euclidean metric) with
uniformly distributed synthetic scalar attributes (Section 5.1, "Datasets").  None of
those data sets is read here; every value comes from ``numpy.random.Generator(PCG64)``.
"""
from __future__ import annotations

import dataclasses
from typing import Optional, Sequence, Tuple

import numpy as np

EMPTY = np.uint32(0xFFFFFFFF)

L2SQ = 0
IP = 1


@dataclasses.dataclass(frozen=True)
class Config:
    """One workload shape.  ``selectivities`` are fractions of the attribute domain."""
    name: str
    n: int
    dim: int
    components: int
    sigma: float
    domain: int
    buckets: int
    k_local: int
    k_remote: int
    n_queries: int
    selectivities: Tuple[float, ...]
    k: int = 10
    beams: Tuple[int, ...] = (64,)
    metric: int = L2SQ
    attr_dist: str = "uniform"      # "uniform" | "zipf"
    normalise: bool = False
    seed: int = 1000
    log_uniform_width: bool = False  # widths log-uniform in [0.1 %, 100 %] of the domain
    append_rounds: int = 0
    append_batch: int = 0


CONFIGS = {
    # 10k x 128, 16 buckets: the case the oracle finishes in seconds
    "c1": Config("c1", 10_000, 128, 16, 0.3, 10_000, 16, 32, 4, 1_000, (0.1,), seed=1001),
    # 1M x 128, 64 buckets: the headline shape (10 % range)
    "c2": Config("c2", 1_000_000, 128, 256, 0.3, 1_000_000, 64, 32, 8, 10_000,
                 (0.01, 0.1, 0.5), beams=(64, 128), seed=1002),
    # 1M x 960: high-dimensional
    "c3": Config("c3", 1_000_000, 960, 256, 0.5, 1_000_000, 64, 48, 8, 10_000, (0.1,),
                 beams=(128,), seed=1003),
    # 10M x 96, unit vectors, inner product, Zipf attributes, 256 buckets
    "c4": Config("c4", 10_000_000, 96, 256, 0.3, 10_000_000, 256, 32, 8, 100_000, (),
                 beams=(128,), metric=IP, attr_dist="zipf", normalise=True, seed=1004,
                 log_uniform_width=True),
    # dynamic: c2's shape, 10 appends of 100k each followed by a search batch
    "c5": Config("c5", 1_000_000, 128, 256, 0.3, 1_000_000, 64, 32, 8, 10_000, (0.1,),
                 seed=1005, append_rounds=10, append_batch=100_000),
}


def scaled(cfg: Config, n: int, n_queries: Optional[int] = None, buckets: Optional[int] = None,
           components: Optional[int] = None, append_batch: Optional[int] = None) -> Config:
    """Same recipe at a smaller size (attribute domain scales with ``n``)."""
    return dataclasses.replace(
        cfg, name=f"{cfg.name}@{n}", n=n, domain=max(1, cfg.domain * n // cfg.n),
        n_queries=n_queries if n_queries is not None else cfg.n_queries,
        buckets=buckets if buckets is not None else cfg.buckets,
        components=components if components is not None else cfg.components,
        append_batch=append_batch if append_batch is not None else cfg.append_batch)


# --------------------------------------------------------------------------- vectors

def _centres(cfg: Config) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(cfg.seed))
    return rng.standard_normal((cfg.components, cfg.dim), dtype=np.float32)


def _mixture(cfg: Config, count: int, stream: int) -> np.ndarray:
    """``count`` draws from the config's Gaussian mixture; ``stream`` separates base
    vectors, queries and each append round."""
    centres = _centres(cfg)
    rng = np.random.Generator(np.random.PCG64([cfg.seed, stream]))
    comp = rng.integers(0, cfg.components, size=count)
    out = np.empty((count, cfg.dim), dtype=np.float32)
    step = 1 << 18
    for s in range(0, count, step):
        e = min(count, s + step)
        noise = rng.standard_normal((e - s, cfg.dim), dtype=np.float32)
        out[s:e] = centres[comp[s:e]] + np.float32(cfg.sigma) * noise
    if cfg.normalise:
        out /= np.linalg.norm(out, axis=1, keepdims=True).astype(np.float32)
    return out


def base_vectors(cfg: Config) -> np.ndarray:
    return _mixture(cfg, cfg.n, stream=1)


def query_vectors(cfg: Config, count: Optional[int] = None, stream: int = 100) -> np.ndarray:
    return _mixture(cfg, cfg.n_queries if count is None else count, stream=stream)


def append_vectors(cfg: Config, round_idx: int) -> np.ndarray:
    return _mixture(cfg, cfg.append_batch, stream=500 + round_idx)


# ------------------------------------------------------------------------ attributes

def _zipf_table(domain: int, exponent: float = 1.1) -> np.ndarray:
    ranks = np.arange(1, domain + 1, dtype=np.float64)
    cdf = np.cumsum(ranks ** -exponent)
    cdf /= cdf[-1]
    return cdf


def attributes(cfg: Config, count: Optional[int] = None, stream: int = 200) -> np.ndarray:
    """Integer scalar attribute per vector: uniform over ``[0, domain)`` or bounded
    Zipf(1.1) by inverse-CDF lookup (attribute = rank - 1)."""
    count = cfg.n if count is None else count
    rng = np.random.Generator(np.random.PCG64([cfg.seed, stream]))
    if cfg.attr_dist == "uniform":
        return rng.integers(0, cfg.domain, size=count, dtype=np.int64).astype(np.int32)
    if cfg.attr_dist == "zipf":
        cdf = _zipf_table(cfg.domain)
        u = rng.random(count)
        return np.minimum(np.searchsorted(cdf, u, side="left"), cfg.domain - 1).astype(np.int32)
    raise ValueError(cfg.attr_dist)


def append_attributes(cfg: Config, round_idx: int) -> np.ndarray:
    return attributes(cfg, cfg.append_batch, stream=700 + round_idx)


# ---------------------------------------------------------------------------- ranges

def ranges(cfg: Config, selectivity: Optional[float], count: Optional[int] = None,
           stream: int = 300) -> Tuple[np.ndarray, np.ndarray]:
    """Closed ranges ``[lo, hi]``.  Width = selectivity x domain, ``lo`` uniform so that
    the range stays inside the domain.  With ``selectivity=None`` the width is
    log-uniform between 0.1 % and 100 % of the domain."""
    count = cfg.n_queries if count is None else count
    tag = 0 if selectivity is None else int(round(selectivity * 1_000_000))
    rng = np.random.Generator(np.random.PCG64([cfg.seed, stream, tag]))
    if selectivity is None:
        u = rng.uniform(-3.0, 0.0, size=count)
        width = np.floor(cfg.domain * np.power(10.0, u)).astype(np.int64)
    else:
        width = np.full(count, int(round(selectivity * cfg.domain)), dtype=np.int64)
    width = np.clip(width, 1, cfg.domain)
    lo = np.floor(rng.random(count) * (cfg.domain - width + 1)).astype(np.int64)
    hi = lo + width - 1
    return lo.astype(np.int32), hi.astype(np.int32)
