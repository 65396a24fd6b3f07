"""Graph-quality diagnostics on the host (harness only): the number of strongly connected
components of a fixed-degree adjacency, the paper's measure of topological integrity
(Section 5.4: one component means every node is reachable from every other)."""
from __future__ import annotations

import numpy as np


def strong_components(adj_slots: np.ndarray, occupied: np.ndarray) -> int:
    """adj_slots[n_slots, K] (0xFFFFFFFF = no edge), occupied[n_slots] bool.  Counts strongly
    connected components among occupied slots."""
    from scipy.sparse import csr_matrix
    from scipy.sparse.csgraph import connected_components
    n = adj_slots.shape[0]
    src = np.repeat(np.arange(n, dtype=np.int64), adj_slots.shape[1])
    dst = adj_slots.reshape(-1).astype(np.int64)
    keep = (dst != 0xFFFFFFFF) & occupied[src]
    g = csr_matrix((np.ones(int(keep.sum()), dtype=np.int8), (src[keep], dst[keep])), shape=(n, n))
    _, labels = connected_components(g, directed=True, connection="strong")
    return int(len(np.unique(labels[occupied])))


def in_degrees(adj_slots: np.ndarray, occupied: np.ndarray) -> np.ndarray:
    """In-degree of every slot (edges out of occupied slots only); 0 for an occupied slot means an
    orphan: no search can reach it except as a seed (Section 5.3 tests that insertion leaves none)."""
    n = adj_slots.shape[0]
    rows = adj_slots[occupied]
    dst = rows[rows != 0xFFFFFFFF].astype(np.int64)
    return np.bincount(dst, minlength=n)


def orphans(adj_slots: np.ndarray, occupied: np.ndarray) -> int:
    """Occupied slots that no edge points to."""
    return int(((in_degrees(adj_slots, occupied) == 0) & occupied).sum())
