"""Exhaustive filtered k-NN on the GPU with torch matmul + top-k, used by the harness only to
score Recall@k (Eq. 1) of full query sets.  It is not part of the search path and shares no
code with it; tests cross-check it against the CPU oracle's float64 exhaustive answer."""
from __future__ import annotations

import numpy as np


def exact_filtered_knn(vectors, attrs, queries, lo, hi, k: int, metric: int = 0, chunk: int = 512):
    """vectors[n,d], attrs[n], queries[nq,d], lo/hi[nq]: torch tensors on one device.
    Returns ids[nq,k] (int64, -1 where fewer than k objects satisfy the range)."""
    import torch
    n = vectors.shape[0]
    chunk = max(1, min(chunk, (1 << 29) // max(1, n)))   # score blocks stay under 2 GiB
    out = torch.full((queries.shape[0], k), -1, dtype=torch.int64, device=vectors.device)
    vn = (vectors * vectors).sum(1) if metric == 0 else None
    for s in range(0, queries.shape[0], chunk):
        q = queries[s:s + chunk]
        d = -(q @ vectors.T) if metric != 0 else (vn[None, :] - 2.0 * (q @ vectors.T))
        bad = (attrs[None, :] < lo[s:s + chunk, None]) | (attrs[None, :] > hi[s:s + chunk, None])
        d.masked_fill_(bad, float("inf"))
        dv, di = torch.topk(d, min(k, n), dim=1, largest=False)
        di = torch.where(torch.isinf(dv), torch.full_like(di, -1), di)
        out[s:s + chunk, :di.shape[1]] = di
    return out


def recall(result_ids, truth_ids) -> float:
    """Eq. 1 averaged over queries.  result_ids: uint32-as-int32 tensor/array [nq,k] with
    0xFFFFFFFF padding; truth_ids: int64 [nq,k] with -1 padding."""
    import torch
    r = torch.as_tensor(np.asarray(result_ids.cpu() if hasattr(result_ids, "cpu") else result_ids).astype(np.int64) & 0xFFFFFFFF)
    t = torch.as_tensor(truth_ids.cpu() if hasattr(truth_ids, "cpu") else truth_ids)
    r = torch.where(r == 0xFFFFFFFF, torch.full_like(r, -2), r)
    hit = (r[:, :, None] == t[:, None, :]) & (t[:, None, :] >= 0)
    return float(hit.any(2).sum().item()) / max(1, int((t >= 0).sum().item()))
