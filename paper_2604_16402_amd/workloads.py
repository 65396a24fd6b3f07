"""Seeded synthetic inputs for range-filtered search over a bucketed graph index.

This module only *makes inputs*: base vectors, scalar attributes, query vectors, query
ranges and a proximity graph to hand to ``load_graph``.  It holds none of the search or
append arithmetic and is the one module that both the CPU oracle's tests and the HIP
library's tests import, so that both sides see byte-identical inputs.

The shapes stand in for the public vector benchmarks the paper evaluates on (Table 2:
96-, 128-, 960-dimensional descriptors, one million base vectors, Euclidean metric) with
uniformly distributed synthetic scalar attributes (Section 5.1, "Datasets").  None of
those data sets is read here; every value comes from ``numpy.random.Generator(PCG64)``.

The graph builder plays the role of the paper's two-pass construction (Section 4.3):
dense local edges inside each bucket from exact k-NN plus diversity pruning and a
forward/reverse interleave, and sparse remote edges to the nearest node of a few other
buckets.  It is input synthesis, not the method under test: its output is given
unchanged to the oracle and to the library, so graph quality moves recall, never parity.
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


# ----------------------------------------------------------------------------- graph

def remote_targets(b: int, n_buckets: int, k_remote: int) -> list:
    """Buckets that bucket ``b`` sends remote edges to: nearest offsets first
    (+-1, +-2: smooth transitions to adjacent attribute intervals), then doubling
    offsets (+-4, +-8, ...: long jumps), then whatever is left, skipping offsets that
    fall outside ``[0, n_buckets)``."""
    if k_remote <= 0:
        return []
    prefs = []
    o = 1
    while o < n_buckets:
        prefs += [o, -o]
        o *= 2
    rest = [s * x for x in range(1, n_buckets) for s in (1, -1) if s * x not in prefs]
    out = []
    for off in prefs + rest:
        t = b + off
        if 0 <= t < n_buckets and t not in out:
            out.append(t)
        if len(out) == k_remote:
            break
    return out


def _pairwise(xa, xb, metric: int):
    """Distance block between two sets of rows (torch tensors): squared L2 or -dot."""
    import torch
    dots = xa @ xb.T
    if metric == IP:
        return -dots
    na = (xa * xa).sum(1, keepdim=True)
    nb = (xb * xb).sum(1, keepdim=True).T
    return torch.clamp(na + nb - 2.0 * dots, min=0.0)


def build_graph(vectors: np.ndarray, bucket_of: np.ndarray, n_buckets: int, k_local: int,
                k_remote: int, *, metric: int = L2SQ, pool: Optional[int] = None,
                device: str = "cpu", chunk: int = 4096,
                progress=None) -> Tuple[np.ndarray, np.ndarray]:
    """A proximity graph for ``load_graph``: ``(local_adj[n, k_local], remote_adj[n, k_remote])``
    as uint32 external ids, ``EMPTY`` where no edge exists.

    Local rows (Section 4.3, first pass): exact k-NN inside the bucket over a pool of
    candidates (4 x k_local by default: wide enough to reach past the node's own cluster), greedy diversity selection (a candidate is kept when it is closer to the
    node than to every candidate already kept, Eq. 2), back-filled with the nearest
    rejected candidates, then interleaved with the reverse edges and cut to ``k_local``.
    Remote rows (second pass): the nearest node in each bucket of ``remote_targets``.
    ``bucket_of[i]`` is the bucket the index under test assigned to id ``i``; local
    edges stay inside it and remote edges leave it.
    """
    import torch
    n, _ = vectors.shape
    pool = pool or 4 * k_local
    local_adj = np.full((n, k_local), EMPTY, dtype=np.uint32)
    remote_adj = np.full((n, max(k_remote, 0)), EMPTY, dtype=np.uint32)
    order = np.argsort(bucket_of, kind="stable")
    counts = np.bincount(bucket_of, minlength=n_buckets)
    starts = np.concatenate([[0], np.cumsum(counts)])
    members = [order[starts[b]:starts[b + 1]] for b in range(n_buckets)]
    dev = torch.device(device)
    xdev = [None] * n_buckets

    def bucket_x(b):
        if xdev[b] is None:
            xdev[b] = torch.from_numpy(vectors[members[b]]).to(dev)
        return xdev[b]

    for b in range(n_buckets):
        ids = members[b]
        m = len(ids)
        if m == 0:
            continue
        xb = bucket_x(b)
        p = min(pool, m - 1)
        kl = min(k_local, m - 1)
        if p > 0:
            cand = torch.empty((m, p), dtype=torch.int64, device=dev)
            cdist = torch.empty((m, p), dtype=torch.float32, device=dev)
            for s in range(0, m, chunk):
                e = min(m, s + chunk)
                dm = _pairwise(xb[s:e], xb, metric)
                dm[torch.arange(e - s, device=dev), torch.arange(s, e, device=dev)] = float("inf")
                dv, di = torch.topk(dm, p, dim=1, largest=False, sorted=True)
                cand[s:e], cdist[s:e] = di, dv
            fwd = torch.empty((m, kl), dtype=torch.int64, device=dev)
            fdist = torch.empty((m, kl), dtype=torch.float32, device=dev)
            sub = max(1, chunk // 8)
            for s in range(0, m, sub):
                e = min(m, s + sub)
                cv = xb[cand[s:e]]                                   # (c, p, d)
                dots = torch.bmm(cv, cv.transpose(1, 2))
                if metric == IP:
                    pd = -dots
                else:
                    nn = (cv * cv).sum(2)
                    pd = torch.clamp(nn[:, :, None] + nn[:, None, :] - 2.0 * dots, min=0.0)
                kept = torch.zeros((e - s, p), dtype=torch.bool, device=dev)
                for t in range(p):
                    hidden = ((pd[:, t, :] <= cdist[s:e, t:t + 1]) & kept).any(1)
                    kept[:, t] = ~hidden
                rank = (~kept).to(torch.int64) * p + torch.arange(p, device=dev)[None, :]
                sel = torch.argsort(rank, dim=1)[:, :kl]
                fwd[s:e] = torch.gather(cand[s:e], 1, sel)
                fdist[s:e] = torch.gather(cdist[s:e], 1, sel)
            # reverse lists: for each target the nearest sources, at most kl of them
            src = torch.arange(m, device=dev)[:, None].expand(m, kl).reshape(-1)
            dst = fwd.reshape(-1)
            dd = fdist.reshape(-1)
            o1 = torch.argsort(dd, stable=True)
            o2 = torch.argsort(dst[o1], stable=True)
            perm = o1[o2]
            dst_s, src_s = dst[perm], src[perm]
            first = torch.searchsorted(dst_s, torch.arange(m, device=dev))
            pos = torch.arange(dst_s.numel(), device=dev) - first[dst_s]
            keep = pos < kl
            rev = torch.full((m, kl), -1, dtype=torch.int64, device=dev)
            rev[dst_s[keep], pos[keep]] = src_s[keep]
            merged = torch.stack([fwd, rev], dim=2).reshape(m, 2 * kl)
            w = merged.shape[1]
            bad = merged < 0
            for s in range(0, m, chunk):
                e = min(m, s + chunk)
                eq = merged[s:e, :, None] == merged[s:e, None, :]
                lower = torch.tril(torch.ones((w, w), dtype=torch.bool, device=dev), diagonal=-1)
                bad[s:e] |= (eq & lower[None]).any(2)
            rank = bad.to(torch.int64) * w + torch.arange(w, device=dev)[None, :]
            sel = torch.argsort(rank, dim=1)[:, :kl]
            final = torch.gather(merged, 1, sel)
            final_bad = torch.gather(bad, 1, sel)
            ids_t = torch.from_numpy(ids.astype(np.int64)).to(dev)
            out = ids_t[final.clamp(min=0)]
            out[final_bad] = int(EMPTY)
            local_adj[ids, :kl] = out.cpu().numpy().astype(np.uint32)
        # remote edges: nearest node of each target bucket
        for j, tb in enumerate(remote_targets(b, n_buckets, k_remote)):
            if len(members[tb]) == 0:
                continue
            xt = bucket_x(tb)
            best = torch.empty(m, dtype=torch.int64, device=dev)
            for s in range(0, m, chunk):
                e = min(m, s + chunk)
                best[s:e] = torch.argmin(_pairwise(xb[s:e], xt, metric), dim=1)
            remote_adj[ids, j] = members[tb][best.cpu().numpy()].astype(np.uint32)
        if progress is not None:
            progress(b)
    return local_adj, remote_adj
