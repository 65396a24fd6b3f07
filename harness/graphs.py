"""A proximity graph for ``load_graph``, made by the test and benchmark harness with torch.

This is neither the library nor the oracle: it is a third, independent construction in the
spirit of the paper's two-pass build (Section 4.3: dense local edges inside each bucket from
exact k-NN, diversity pruning and a forward/reverse interleave; sparse remote edges to the
nearest node of a few other buckets).  Its output is handed unchanged to the oracle and to the
library, so that search and insertion can be compared on a graph neither of them built: graph
quality moves recall, never parity.
"""
from __future__ import annotations

from typing import Optional, Tuple

import numpy as np

EMPTY = np.uint32(0xFFFFFFFF)
L2SQ = 0
IP = 1




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
