"""CPU oracle, Python side: bucketing, graph loading, exhaustive ground truth, recall,
and a ctypes front for the scalar C search/append in ``grab_oracle.c``.

THIS IS TEST INFRASTRUCTURE (see the C file's header).  It imports nothing from the
product package and the product package imports nothing from here.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

EMPTY = np.uint32(0xFFFFFFFF)
L2SQ, IP = 0, 1
_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libgrab_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no fast-math, no contraction: the fp32 order is fixed)."""
    src = os.path.join(_HERE, "grab_oracle.c")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
                               "-Wall", "-o", _LIB_PATH, src, "-lm"])
    return _LIB_PATH


class _Index(ctypes.Structure):
    _fields_ = [("dim", ctypes.c_int32), ("metric", ctypes.c_int32), ("k_local", ctypes.c_int32),
                ("k_remote", ctypes.c_int32), ("n_buckets", ctypes.c_int32), ("pad_", ctypes.c_int32),
                ("n_cap", ctypes.c_int64), ("X", ctypes.c_void_p), ("attr", ctypes.c_void_p),
                ("A", ctypes.c_void_p), ("slot2id", ctypes.c_void_p), ("table", ctypes.c_void_p)]


class _Params(ctypes.Structure):
    _fields_ = [("search_width", ctypes.c_int32), ("max_iter", ctypes.c_int32),
                ("n_seeds", ctypes.c_int32), ("visited_cap", ctypes.c_int32),
                ("seed_salt", ctypes.c_uint32)]


APPEND_STATS = ["requests_local", "requests_remote", "groups_local", "groups_remote", "applied_local", "applied_remote",
                "candidates_scanned", "remote_rows_evaluated", "local_requests_passed", "search_evals", "search_parents"]


class _RemoteRule(ctypes.Structure):
    _fields_ = [("mode", ctypes.c_int32), ("n_proximal", ctypes.c_int32), ("window", ctypes.c_int64)]


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB_PATH)
        _lib.oracle_distance.restype = ctypes.c_float
        _lib.oracle_distance.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32]
        _lib.oracle_search.restype = ctypes.c_int
        _lib.oracle_max_threads.restype = ctypes.c_int
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def distance(q: np.ndarray, v: np.ndarray, metric: int = L2SQ) -> np.float32:
    """fp32 distance with the fixed summation tree (see the C file)."""
    q = np.ascontiguousarray(q, dtype=np.float32)
    v = np.ascontiguousarray(v, dtype=np.float32)
    return np.float32(_load().oracle_distance(_ptr(q), _ptr(v), q.shape[0], metric))


# ------------------------------------------------------------------------ bucketing (A1)

def float_order_key(values) -> np.ndarray:
    """int32 keys that order exactly like the fp32 values (the filter of Section 3 on a float
    attribute, as in the experiments of Section 5.1, reduced to the integer case).

    An IEEE-754 binary32 number is sign and magnitude: among non-negative numbers a larger
    value has a larger bit pattern, among negative numbers a larger magnitude (a smaller
    value) has a larger bit pattern.  So the key of x >= 0 is its bit pattern read as int32,
    and the key of x < 0 is the bit pattern with the 31 magnitude bits inverted (still
    negative, and now growing with x).  Both zeros get key 0.  NaN has no order: refused.
    """
    v = np.ascontiguousarray(values, dtype=np.float32)
    if np.isnan(v).any():
        raise ValueError("NaN has no place in an ordered attribute")
    bits = v.view(np.int32).astype(np.int64)
    key = np.where(bits >= 0, bits, bits ^ 0x7FFFFFFF)
    key = np.where(v == 0.0, 0, key)
    return key.astype(np.int32)


def float_range_keys(lo, hi) -> Tuple[np.ndarray, np.ndarray]:
    """Keys of closed float ranges; a range with a NaN bound holds nothing (keys 1 > 0)."""
    lo = np.ascontiguousarray(lo, dtype=np.float32)
    hi = np.ascontiguousarray(hi, dtype=np.float32)
    bad = np.isnan(lo) | np.isnan(hi)
    klo = float_order_key(np.where(bad, np.float32(0), lo))
    khi = float_order_key(np.where(bad, np.float32(0), hi))
    return np.where(bad, 1, klo).astype(np.int32), np.where(bad, 0, khi).astype(np.int32)


def bucket_layout(attrs: np.ndarray, n_buckets: int, n_cap: int):
    """Section 4.2.1: partition into ``n_buckets`` disjoint ordered buckets by the scalar.

    reading: ids sorted by (attribute, id); bucket b takes sorted ranks
    [floor(b*n/B), floor((b+1)*n/B)) (equal counts, ties split by id); bucket b owns the slot
    slab [base[b], base[b]+cap[b]) with cap[b] = count[b] + floor((n_cap-n)/B) and
    base[b] = sum of earlier caps.  Returns (table[B,6] int32, id2slot[n], slot2id[total]).
    """
    n = len(attrs)
    B = n_buckets
    if B < 1 or n < B or n_cap < n:
        raise ValueError("need 1 <= B <= n <= n_cap")
    order = np.lexsort((np.arange(n), attrs))
    slack = (n_cap - n) // B
    starts = (np.arange(B + 1, dtype=np.int64) * n) // B
    counts = np.diff(starts)
    caps = counts + slack
    bases = np.concatenate([[0], np.cumsum(caps)[:-1]])
    total = int(caps.sum())
    table = np.zeros((B, 6), dtype=np.int32)
    id2slot = np.empty(n, dtype=np.uint32)
    slot2id = np.full(total, EMPTY, dtype=np.uint32)
    for b in range(B):
        ids = order[starts[b]:starts[b + 1]]
        slots = bases[b] + np.arange(counts[b])
        id2slot[ids] = slots
        slot2id[slots] = ids
        table[b] = (bases[b], counts[b], counts[b], caps[b], attrs[ids[0]], attrs[ids[-1]])
    return table, id2slot, slot2id


class Index:
    """Slot-space arrays of one index plus the calls that act on them."""

    def __init__(self, vectors: np.ndarray, attrs: np.ndarray, n_buckets: int,
                 n_cap: Optional[int] = None, metric: int = L2SQ):
        vectors = np.ascontiguousarray(vectors, dtype=np.float32)
        attrs = np.ascontiguousarray(attrs, dtype=np.int32)
        n, d = vectors.shape
        if d % 32:
            raise ValueError("dim must be a multiple of 32")
        n_cap = n if n_cap is None else n_cap
        self.dim, self.metric, self.n, self.n_buckets = d, metric, n, n_buckets
        self.table, self.id2slot, self.slot2id = bucket_layout(attrs, n_buckets, n_cap)
        self.n_cap = len(self.slot2id)
        self.id2slot = np.concatenate([self.id2slot, np.full(self.n_cap - n, EMPTY, np.uint32)])
        self.X = np.zeros((self.n_cap, d), dtype=np.float32)
        self.attr = np.zeros(self.n_cap, dtype=np.int32)
        live = self.slot2id != EMPTY
        self.X[live] = vectors[self.slot2id[live]]
        self.attr[live] = attrs[self.slot2id[live]]
        self.k_local = self.k_remote = 0
        self.A = None
        # remote_mode 0: remote entry j belongs to the j-th target bucket; 1: proximal / global split
        # (n_proximal None = ceil(k_remote / 2); remote_window = fraction of the attribute span)
        self.params = dict(search_width=1, max_iter=None, n_seeds=None, visited_cap=2800,
                           seed_salt=0, alpha=0.6, append_beam=64, remote_mode=0, n_proximal=None,
                           remote_window=0.2, append_remote_cands=0)

    # -- M_I2B: bucket of every external id
    def bucket_of_ids(self) -> np.ndarray:
        return self.bucket_of_slots(self.id2slot[:self.n])

    def bucket_of_slots(self, slots: np.ndarray) -> np.ndarray:
        ends = self.table[:, 0].astype(np.int64) + self.table[:, 3]
        return np.searchsorted(ends, np.asarray(slots, dtype=np.int64), side="right")

    # -- load_graph: ids -> slots, [local | remote] per row, checked (Section 4.2.2)
    def load_graph(self, local_adj: np.ndarray, remote_adj: np.ndarray):
        n = self.n
        kl, kr = local_adj.shape[1], remote_adj.shape[1]
        if local_adj.shape[0] != n or remote_adj.shape[0] != n:
            raise ValueError("adjacency must have one row per base vector")
        adj = np.concatenate([local_adj, remote_adj], axis=1).astype(np.uint32)
        live = adj != EMPTY
        if (adj[live] >= n).any():
            raise ValueError("neighbour id out of range")
        slots = np.full(adj.shape, EMPTY, dtype=np.uint32)
        slots[live] = self.id2slot[adj[live]]
        own = self.bucket_of_ids()[:, None]
        nb = np.where(live, self.bucket_of_slots(np.where(live, slots, 0)), -1)
        if ((nb[:, :kl] != own) & live[:, :kl]).any():
            raise ValueError("a local edge leaves its bucket")
        if self.params["remote_mode"] == 0 and ((nb[:, kl:] == own) & live[:, kl:]).any():
            raise ValueError("a remote edge stays in its bucket")   # mode 1 keeps redundant local edges there
        self.k_local, self.k_remote = kl, kr
        self.A = np.full((self.n_cap, kl + kr), EMPTY, dtype=np.uint32)
        self.A[self.id2slot[:n]] = slots

    # -- ctypes views
    def _c_index(self) -> _Index:
        A = self.A if self.A is not None else np.zeros((1, 1), np.uint32)
        return _Index(self.dim, self.metric, self.k_local, self.k_remote, self.n_buckets, 0,
                      self.n_cap, _ptr(self.X).value, _ptr(self.attr).value, _ptr(A).value,
                      _ptr(self.slot2id).value, _ptr(self.table).value)

    def _c_params(self, beam: int) -> _Params:
        p = self.params
        max_iter = p["max_iter"] if p["max_iter"] is not None else 2 * beam
        n_seeds = p["n_seeds"] if p["n_seeds"] is not None else min(beam, 64)
        return _Params(p["search_width"], max_iter, n_seeds, p["visited_cap"], p["seed_salt"])

    def _c_remote_rule(self) -> _RemoteRule:
        """The remote wiring in force.  The proximal window is `remote_window` times the span of
        the attributes in the index now (largest minus smallest), rounded down."""
        p = self.params
        kp = p["n_proximal"] if p["n_proximal"] is not None else (self.k_remote + 1) // 2
        span = int(self.table[-1, 5]) - int(self.table[0, 4])
        return _RemoteRule(p["remote_mode"], kp, int(np.floor(float(p["remote_window"]) * float(span))))

    def search_scoped(self, queries: np.ndarray, scope: np.ndarray, beam: int):
        """Candidate search of insertion / construction: scope b >= 0 = inside bucket b,
        -2 - b = outside bucket b.  Returns the whole final queues (slots[nq,beam], dist[nq,beam])."""
        queries = np.ascontiguousarray(queries, dtype=np.float32)
        scope = np.ascontiguousarray(scope, dtype=np.int32)
        nq = len(scope)
        slots = np.empty((nq, beam), dtype=np.uint32)
        dist = np.empty((nq, beam), dtype=np.float32)
        ix, pr = self._c_index(), self._c_params(beam)
        _load().oracle_search_scoped(ctypes.byref(ix), ctypes.byref(pr), _ptr(queries), _ptr(scope),
                                     ctypes.c_int64(nq), ctypes.c_int32(beam), _ptr(slots), _ptr(dist))
        return slots, dist

    def select(self, lo: int, hi: int, beam: int = 64):
        """(info[6], seeds): bucket run, population size, valid sorted span ends, seed slots."""
        pr = self._c_params(beam)
        info = np.zeros(6, dtype=np.int64)
        seeds = np.full(pr.n_seeds, EMPTY, dtype=np.uint32)
        ix = self._c_index()
        _load().oracle_select(ctypes.byref(ix), ctypes.byref(pr), ctypes.c_int32(lo), ctypes.c_int32(hi),
                              _ptr(info), _ptr(seeds))
        return info, seeds

    def search(self, queries: np.ndarray, lo: np.ndarray, hi: np.ndarray, k: int, beam: int,
               threads: int = 1):
        """Algorithm 2 for a batch.  Returns (ids[nq,k] uint32, dist[nq,k] fp32, counters[nq,8])."""
        if self.A is None:
            raise RuntimeError("load_graph first")
        queries = np.ascontiguousarray(queries, dtype=np.float32)
        lo = np.ascontiguousarray(lo, dtype=np.int32)
        hi = np.ascontiguousarray(hi, dtype=np.int32)
        nq = queries.shape[0]
        ids = np.empty((nq, k), dtype=np.uint32)
        dist = np.empty((nq, k), dtype=np.float32)
        ctr = np.zeros((nq, 8), dtype=np.uint32)
        ix, pr = self._c_index(), self._c_params(beam)
        rc = _load().oracle_search(ctypes.byref(ix), ctypes.byref(pr), _ptr(queries), _ptr(lo), _ptr(hi),
                                   ctypes.c_int64(nq), ctypes.c_int32(k), ctypes.c_int32(beam),
                                   _ptr(ids), _ptr(dist), _ptr(ctr), ctypes.c_int32(threads))
        if rc:
            raise ValueError("oracle_search rejected its arguments")
        return ids, dist, ctr


    # -- Section 4.3: two-pass construction (see the reading in grab_oracle.c)
    def knn(self, slot: int, target_bucket: int, P: int):
        """(slots[P], dist[P]) of the P nearest objects of a bucket to the row at `slot`."""
        out_s = np.full(P, EMPTY, dtype=np.uint32)
        out_d = np.full(P, np.inf, dtype=np.float32)
        ix = self._c_index()
        _load().oracle_knn(ctypes.byref(ix), ctypes.c_uint32(slot), ctypes.c_int32(target_bucket), ctypes.c_int32(P),
                           _ptr(out_s), _ptr(out_d))
        return out_s, out_d

    def remote_targets(self, b: int, k_remote: int):
        out = np.zeros(max(k_remote, 1), dtype=np.int32)
        f = _load().oracle_remote_targets
        f.restype = ctypes.c_int
        n = f(ctypes.c_int32(b), ctypes.c_int32(self.n_buckets), ctypes.c_int32(k_remote), _ptr(out))
        return out[:n].tolist()

    def build_graph(self, k_local: int, k_remote: int, pool: Optional[int] = None, threads: int = 1,
                    want_lists: bool = False):
        """Builds the adjacency in place.  Returns (F, R) when want_lists."""
        pool = pool or min(4 * k_local, 128)
        self.k_local, self.k_remote = k_local, k_remote
        self.A = np.full((self.n_cap, k_local + k_remote), EMPTY, dtype=np.uint32)
        F = np.empty((self.n_cap, pool), dtype=np.uint32) if want_lists else None
        R = np.empty((self.n_cap, k_local), dtype=np.uint32) if want_lists else None
        ix = self._c_index()
        rr, pr = self._c_remote_rule(), self._resolved_append_params()
        f = _load().oracle_build_graph
        f.restype = ctypes.c_int
        rc = f(ctypes.byref(ix), ctypes.c_int32(pool), _ptr(F) if want_lists else None,
               _ptr(R) if want_lists else None, ctypes.c_int32(threads), ctypes.byref(rr), ctypes.byref(pr),
               ctypes.c_int32(self.params["append_beam"]))
        if rc:
            raise ValueError("oracle_build_graph rejected its arguments")
        return (F, R) if want_lists else None

    def build_remote(self, threads: int = 1):
        """Pass 2 of the construction alone: rewrites the remote part of every row of the graph
        the index holds (see the reading in grab_oracle.c)."""
        if self.A is None:
            raise RuntimeError("load_graph first")
        ix = self._c_index()
        rr, pr = self._c_remote_rule(), self._resolved_append_params()
        f = _load().oracle_build_remote
        f.restype = ctypes.c_int
        rc = f(ctypes.byref(ix), ctypes.byref(rr), ctypes.byref(pr), ctypes.c_int32(self.params["append_beam"]),
               ctypes.c_int32(threads))
        if rc:
            raise ValueError("oracle_build_remote rejected its arguments")

    def _resolved_append_params(self) -> _Params:
        return self._c_params(self.params["append_beam"])

    def append(self, vectors: np.ndarray, attrs: np.ndarray, threads: int = 1):
        """Section 4.4 batched insertion (see the reading in grab_oracle.c).  Raises
        OverflowError, leaving the index untouched, if a bucket has no tail room.
        Returns kept[m,2]: entries of each new row kept by the diversity rule (local, remote)."""
        if self.A is None:
            raise RuntimeError("load_graph first")
        vectors = np.ascontiguousarray(vectors, dtype=np.float32)
        attrs = np.ascontiguousarray(attrs, dtype=np.int32)
        m = len(attrs)
        if vectors.shape != (m, self.dim):
            raise ValueError("bad shape")
        if self.n + m > len(self.id2slot):
            raise OverflowError("more objects than slots")
        kept = np.zeros((m, 2), dtype=np.int32)
        stats = np.zeros(12, dtype=np.uint64)
        ix, pr, rr = self._c_index(), self._resolved_append_params(), self._c_remote_rule()
        f = _load().oracle_append
        f.restype = ctypes.c_int
        rc = f(ctypes.byref(ix), ctypes.byref(pr), ctypes.c_float(self.params["alpha"]),
               ctypes.c_int32(self.params["append_beam"]), _ptr(vectors), _ptr(attrs), ctypes.c_int64(m),
               ctypes.c_int64(self.n), _ptr(self.id2slot), _ptr(kept), ctypes.c_int32(threads), ctypes.byref(rr),
               _ptr(stats), ctypes.c_int32(self.params["append_remote_cands"]))
        self.last_append_stats = dict(zip(APPEND_STATS, (int(x) for x in stats)))
        if rc == 3:
            raise OverflowError("a bucket is out of tail room")
        if rc:
            raise ValueError("oracle_append rejected its arguments")
        self.n += m
        return kept


def mix32(x: int) -> int:
    f = _load().oracle_mix32
    f.restype = ctypes.c_uint32
    return int(f(ctypes.c_uint32(x)))


def max_threads() -> int:
    return int(_load().oracle_max_threads())


# ------------------------------------------------------------- exact answer (Definition, Eq. 1)

def exact_filtered_knn(vectors: np.ndarray, attrs: np.ndarray, queries: np.ndarray, lo, hi,
                       k: int, metric: int = L2SQ) -> Tuple[np.ndarray, np.ndarray]:
    """Hybrid Search definition (Section 2.4): among objects with lo <= s_i <= hi the k with
    the smallest distance, in float64, ties by id.  Missing entries: (EMPTY, +inf)."""
    v64 = vectors.astype(np.float64)
    nq = len(queries)
    ids = np.full((nq, k), EMPTY, dtype=np.uint32)
    dist = np.full((nq, k), np.inf, dtype=np.float64)
    for i in range(nq):
        ok = np.nonzero((attrs >= lo[i]) & (attrs <= hi[i]))[0]
        if len(ok) == 0:
            continue
        q = queries[i].astype(np.float64)
        if metric == L2SQ:
            diff = v64[ok] - q
            d = np.einsum("ij,ij->i", diff, diff)
        else:
            d = -(v64[ok] @ q)
        o = np.lexsort((ok, d))[:k]
        ids[i, :len(o)] = ok[o]
        dist[i, :len(o)] = d[o]
    return ids, dist


def recall_at_k(result_ids: np.ndarray, truth_ids: np.ndarray) -> float:
    """Eq. 1 averaged over queries: |R intersect R*| / k; padding never counts as a hit and
    a query with fewer than k valid objects is scored against the number it has."""
    hits, total = 0, 0
    for r, t in zip(result_ids, truth_ids):
        t = t[t != EMPTY]
        total += len(t)
        hits += len(np.intersect1d(r[r != EMPTY], t))
    return hits / max(total, 1)
