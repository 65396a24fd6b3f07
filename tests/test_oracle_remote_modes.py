"""Pins for the oracle's second reading of the remote wiring: candidates from the global scope,
remote budget split into proximal and global picks, redundant local edges kept where a class has
no pick (Section 4.3, Remote Edge Construction; Section 4.4, Parallel Candidate Search), and for
the freshness bias under the inner-product metric (Eq. 3)."""
import json
import os

import numpy as np
import pytest

from oracle import oracle as O
from paper_2604_16402_amd import workloads as W

GOLD = os.path.join(os.path.dirname(__file__), "golden")
E = int(O.EMPTY)


def _pad(points, dim=32):
    out = np.zeros((len(points), dim), np.float32)
    out[:, :len(points[0])] = np.asarray(points, np.float32)
    return out


@pytest.mark.parametrize("alpha", [0.6, 1.0])
def test_hand_worked_append_with_proximal_and_global_picks(alpha):
    g = json.load(open(os.path.join(GOLD, "append_proximal_2d.json")))
    ix = O.Index(_pad(g["points"]), np.asarray(g["attrs"], np.int32), g["n_buckets"], n_cap=g["n_cap"])
    ix.params.update(remote_mode=1, n_proximal=g["n_proximal"], remote_window=g["remote_window"])
    ix.load_graph(np.asarray(g["local"], np.uint32), np.asarray(g["remote"], np.uint32))
    ix.params.update(n_seeds=g["n_seeds"], append_beam=g["append_beam"], visited_cap=g["visited_cap"], alpha=alpha)
    kept = ix.append(_pad(g["new_points"]), np.asarray(g["new_attrs"], np.int32))
    want = g[f"alpha_{alpha}"]
    assert ix.id2slot[8:10].tolist() == g["new_slots"]
    assert kept.tolist() == g["kept"]
    assert ix.A.tolist() == want["adj_slots"]
    assert ix.table.tolist() == want["table"]
    assert ix.last_append_stats == want["stats"]


def test_scoped_searches_see_exactly_their_scope():
    # with more seeds than objects every member of the scope is a seed: the queue of a scoped
    # search is then the scope itself, ordered by (distance, slot) - brute force in float64
    cfg = W.scaled(W.CONFIGS["c1"], 96, n_queries=12, buckets=4)
    X, a = W.base_vectors(cfg), W.attributes(cfg)
    ix = O.Index(X, a, cfg.buckets, n_cap=120)
    ix.build_graph(6, 2, pool=12)
    ix.params.update(n_seeds=128, visited_cap=4000)
    q = W.query_vectors(cfg)
    for b in range(4):
        for scope, members in ((b, np.arange(ix.table[b, 0], ix.table[b, 0] + ix.table[b, 2])),
                               (-2 - b, np.concatenate([np.arange(t[0], t[0] + t[2]) for c, t in enumerate(ix.table) if c != b]))):
            slots, dist = ix.search_scoped(q, np.full(len(q), scope, np.int32), 128)
            for i in range(len(q)):
                d64 = ((ix.X[members].astype(np.float64) - q[i].astype(np.float64)) ** 2).sum(1)
                got = slots[i][slots[i] != O.EMPTY]
                assert sorted(got.tolist()) == members.tolist()
                assert (np.diff(dist[i][:len(got)]) >= 0).all()
                assert np.allclose(dist[i][:len(got)], np.sort(d64), rtol=1e-5)
    # one bucket: nothing lies outside it
    one = O.Index(X, a, 1)
    one.build_graph(6, 0, pool=12)
    slots, _ = one.search_scoped(q[:2], np.full(2, -2, np.int32), 16)
    assert (slots == O.EMPTY).all()


@pytest.fixture(scope="module")
def small_built():
    """96 objects in 4 buckets; every candidate search sees its whole scope (seeds >= objects), so
    the construction's picks can be re-derived by brute force."""
    cfg = W.scaled(W.CONFIGS["c1"], 96, n_queries=12, buckets=4)
    X = W.base_vectors(cfg)
    a = (np.random.default_rng(5).permutation(96) * 7).astype(np.int32)      # distinct attributes
    out = {}
    for name, kw in (("pass1", dict(n_proximal=3, remote_window=0.0)),       # distinct attributes: nobody within 0
                     ("split", dict(n_proximal=2, remote_window=0.5)),
                     ("narrow", dict(n_proximal=2, remote_window=0.02))):
        ix = O.Index(X, a, cfg.buckets, n_cap=120)
        ix.params.update(remote_mode=1, n_seeds=128, visited_cap=4000, append_beam=128, **kw)
        F, R = ix.build_graph(6, 3, pool=12, want_lists=True)
        out[name] = dict(ix=ix, F=F, R=R)
    return dict(cfg=cfg, X=X, attrs=a, **out)


def test_redundant_local_edges_continue_the_interleaved_merge(small_built):
    # n_proximal = K_remote with a window no attribute difference fits: no pick at all, the row is
    # what pass 1 leaves: K_local necessary entries, then the next distinct entries of the merge
    p = small_built["pass1"]
    ix, F, R = p["ix"], p["F"], p["R"]
    kl, K = 6, 9
    for u in np.nonzero(ix.slot2id != O.EMPTY)[0]:
        seq = [c for pair in zip(F[u][:kl], R[u][:kl]) for c in pair] + F[u][kl:].tolist()
        merged = []
        for c in seq:
            if c != O.EMPTY and int(c) not in merged:
                merged.append(int(c))
        assert ix.A[u].tolist() == (merged + [E] * K)[:K]
    own = ix.bucket_of_slots(np.arange(ix.n_cap))[:, None]
    live = ix.A != O.EMPTY
    assert (ix.bucket_of_slots(np.where(live, ix.A, 0)) == own)[live].all()     # local edges only
    # the first K_local columns are the local part of the first reading on the same data
    ref = O.Index(small_built["X"], small_built["attrs"], 4, n_cap=120)
    ref.build_graph(6, 3, pool=12)
    assert np.array_equal(ref.A[:, :kl], ix.A[:, :kl])


@pytest.mark.parametrize("name", ["split", "narrow"])
def test_remote_picks_are_the_brute_force_selection(small_built, name):
    p, base = small_built[name], small_built["pass1"]["ix"]
    ix = p["ix"]
    kl, kr, kp = 6, 3, 2
    span = int(ix.table[-1, 5]) - int(ix.table[0, 4])
    w = int(np.floor(ix.params["remote_window"] * span))
    occupied = np.nonzero(ix.slot2id != O.EMPTY)[0]
    fallbacks = 0
    for u in occupied:
        b = int(ix.bucket_of_slots([u])[0])
        outside = [int(s) for s in occupied if int(ix.bucket_of_slots([s])[0]) != b]
        outside.sort(key=lambda s: (float(O.distance(ix.X[u], ix.X[s])), s))
        prox = [s for s in outside if abs(int(ix.attr[s]) - int(ix.attr[u])) <= w][:kp]
        glob = [s for s in outside if abs(int(ix.attr[s]) - int(ix.attr[u])) > w][:kr - kp]
        want = base.A[u].tolist()                         # pass-1 row: redundant local edges in the remote part
        for j, s in enumerate(prox):
            want[kl + j] = s
        for j, s in enumerate(glob):
            want[kl + kp + j] = s
        fallbacks += kp - len(prox)
        assert ix.A[u].tolist() == want, u
    assert (fallbacks > 0) == (name == "narrow")          # the narrow window leaves proximal positions to local edges


def test_build_remote_alone_equals_the_second_pass(small_built):
    # pass 2 on a loaded graph = pass 2 inside build_graph, for both readings
    X, a = small_built["X"], small_built["attrs"]
    base = small_built["pass1"]["ix"]
    for mode, kw in ((1, dict(n_proximal=2, remote_window=0.5)), (0, {})):
        ix = O.Index(X, a, 4, n_cap=120)
        ix.params.update(remote_mode=mode, n_seeds=128, visited_cap=4000, append_beam=128, **kw)
        ix.k_local, ix.k_remote = 6, 3
        ix.A = base.A.copy()
        ix.build_remote()
        ref = O.Index(X, a, 4, n_cap=120)
        ref.params.update(ix.params)
        ref.build_graph(6, 3, pool=12)
        if mode == 1:
            assert np.array_equal(ix.A, small_built["split"]["ix"].A)
        else:
            assert np.array_equal(ix.A, ref.A)


def _grown(mode, metric=O.L2SQ, alpha=0.6, n=3000, batch=400):
    cfg = W.scaled(W.CONFIGS["c4" if metric == O.IP else "c5"], n, n_queries=100, buckets=4, components=8, append_batch=batch)
    if metric == O.IP:
        import dataclasses
        cfg = dataclasses.replace(cfg, attr_dist="uniform", domain=n)
    X, a = W.base_vectors(cfg), W.attributes(cfg)
    ix = O.Index(X, a, cfg.buckets, n_cap=n + 4 * batch, metric=metric)
    ix.params.update(remote_mode=mode, alpha=alpha, n_seeds=64, append_beam=64)
    ix.build_graph(12, 4, pool=32, threads=8)
    pre = ix.A.copy()
    nx, na = W.append_vectors(cfg, 0), W.append_attributes(cfg, 0)
    kept = ix.append(nx, na, threads=4)
    return dict(cfg=cfg, ix=ix, pre=pre, X=X, attrs=a, nx=nx, na=na, kept=kept)


def test_append_invariants_under_the_second_reading():
    g = _grown(1)
    ix, cfg = g["ix"], g["cfg"]
    n0, n = cfg.n, ix.n
    kl, kr = ix.k_local, ix.k_remote
    kp = (kr + 1) // 2
    span = int(g["attrs"].max()) - int(g["attrs"].min())
    w = int(np.floor(0.2 * span))
    new_slots = ix.id2slot[n0:n]
    own_new = ix.bucket_of_slots(new_slots)
    rows = ix.A[new_slots]
    for i in range(len(new_slots)):
        row = rows[i]
        live = row[row != O.EMPTY]
        assert len(set(live.tolist())) == len(live) and new_slots[i] not in live
        nb = ix.bucket_of_slots(row[:kl][row[:kl] != O.EMPTY])
        assert (nb == own_new[i]).all()                                        # local part stays in the bucket
        for j in range(kr):
            c = row[kl + j]
            if c == O.EMPTY:
                continue
            if ix.bucket_of_slots([c])[0] == own_new[i]:
                continue                                                       # redundant local edge
            diff = abs(int(ix.attr[c]) - int(g["na"][i]))
            assert (diff <= w) == (j < kp), (i, j)                             # class by position
        picked = [c for c in row[kl:] if c != O.EMPTY and ix.bucket_of_slots([c])[0] != own_new[i]]
        assert g["kept"][i, 1] == len(picked)
    # old rows change only by gaining fresh nodes, and fresh nodes are found by searches
    old = ix.id2slot[:n0]
    changed = ix.A[old] != g["pre"][old]
    assert np.isin(ix.A[old][changed], new_slots).all()
    indeg = np.bincount(ix.A[ix.A != O.EMPTY].astype(np.int64), minlength=ix.n_cap)
    assert (indeg[new_slots] > 0).mean() > 0.99
    allX, alla = np.concatenate([g["X"], g["nx"]]), np.concatenate([g["attrs"], g["na"]])
    q = W.query_vectors(cfg)
    lo, hi = W.ranges(cfg, 0.25)
    ids, _, _ = ix.search(q, lo, hi, 10, 64)
    gt, _ = O.exact_filtered_knn(allX, alla, q, lo, hi, 10)
    assert O.recall_at_k(ids, gt) > 0.9


def test_batch_of_one_follows_the_request_rules_of_the_second_reading():
    # alpha -> 0: every distance test passes, so what happens at a target is decided by its
    # positions alone and can be read off the row as it was before
    g = _grown(1, alpha=1e-6, batch=1)
    ix, cfg, pre = g["ix"], g["cfg"], g["pre"]
    s = int(ix.id2slot[cfg.n])
    kl, kr = ix.k_local, ix.k_remote
    kp = (kr + 1) // 2
    w = int(np.floor(0.2 * (int(g["attrs"].max()) - int(g["attrs"].min()))))
    mine = int(ix.bucket_of_slots([s])[0])
    seen_remote = 0
    for j in range(kr):
        t = int(ix.A[s][kl + j])
        if t == E or int(ix.bucket_of_slots([t])[0]) == mine:
            continue
        seen_remote += 1
        prox = abs(int(ix.attr[t]) - int(g["na"][0])) <= w
        j0, j1 = (0, kp) if prox else (kp, kr)
        part = pre[t][kl + j0:kl + j1].tolist()
        bt = int(ix.bucket_of_slots([t])[0])
        free = [x for x, c in enumerate(part) if c == E or int(ix.bucket_of_slots([c])[0]) == bt]
        now = ix.A[t][kl + j0:kl + j1].tolist()
        if free:
            want = list(part); want[free[0]] = s
        else:
            far = max(range(len(part)), key=lambda x: (float(O.distance(ix.X[t], ix.X[part[x]])), part[x]))
            want = list(part); want[far] = s
        assert now == want
        other = slice(kl + (kp if prox else 0), kl + (kr if prox else kp))
        assert ix.A[t][other].tolist() == pre[t][other].tolist()               # the other class is untouched
    assert seen_remote > 0


def test_bias_helps_newcomers_under_inner_product_too():
    # Eq. 3 is meant to open rows for fresh nodes: a smaller alpha must never cost them in-edges,
    # also when distances are negated inner products (negative for similar vectors)
    got = {}
    for alpha in (1.0, 0.6, 0.2):
        g = _grown(0, metric=O.IP, alpha=alpha)
        ix, cfg = g["ix"], g["cfg"]
        new = ix.id2slot[cfg.n:ix.n]
        got[alpha] = int(np.isin(ix.A[ix.id2slot[:cfg.n]], new).sum())
    assert got[0.2] >= got[0.6] >= got[1.0] and got[0.6] > got[1.0]


def test_inner_product_bias_is_the_euclidean_one_on_unit_vectors():
    # for unit vectors 1 + (-q.v) is half the squared Euclidean distance, so an inner-product index
    # and a squared-L2 index over the same unit vectors must take the same rewiring decisions
    out = {}
    for metric in (O.IP, O.L2SQ):
        cfg = W.scaled(W.CONFIGS["c4"], 1500, n_queries=10, buckets=3, components=6, append_batch=150)
        import dataclasses
        cfg = dataclasses.replace(cfg, attr_dist="uniform", domain=1500)
        X, a = W.base_vectors(cfg), W.attributes(cfg)
        ix = O.Index(X, a, cfg.buckets, n_cap=2100, metric=metric)
        ix.params.update(n_seeds=600, append_beam=64, visited_cap=8000)
        ref = O.Index(X, a, cfg.buckets, n_cap=2100, metric=O.L2SQ)
        ref.build_graph(10, 2, pool=24, threads=8)
        ix.k_local, ix.k_remote, ix.A = 10, 2, ref.A.copy()      # the same graph under both metrics
        ix.append(W.append_vectors(cfg, 0), W.append_attributes(cfg, 0), threads=4)
        out[metric] = ix.A.copy()
    same = (out[O.IP] == out[O.L2SQ]).mean()
    assert same > 0.995     # identical up to fp32 rounding of the two distance forms near ties
