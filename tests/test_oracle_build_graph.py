"""Pins for the oracle's two-pass graph construction (Section 4.3)."""
import numpy as np
import pytest

from oracle import oracle as O
from paper_2604_16402_amd import workloads as W


@pytest.fixture(scope="module")
def built():
    cfg = W.scaled(W.CONFIGS["c1"], 3000, n_queries=300, buckets=6)
    X, a = W.base_vectors(cfg), W.attributes(cfg)
    ix = O.Index(X, a, cfg.buckets)
    F, R = ix.build_graph(16, 4, pool=32, threads=8, want_lists=True)
    return dict(cfg=cfg, X=X, attrs=a, ix=ix, F=F, R=R)


def test_knn_against_float64_brute_force(built):
    ix, X = built["ix"], built["X"]
    rng = np.random.default_rng(0)
    for slot in rng.integers(0, 3000, 25):
        for tb in (int(ix.bucket_of_slots([slot])[0]), 0, 5):
            s, d = ix.knn(int(slot), tb, 20)
            t = ix.table[tb]
            members = np.arange(t[0], t[0] + t[2])
            members = members[members != slot]
            d64 = ((ix.X[members].astype(np.float64) - ix.X[slot].astype(np.float64)) ** 2).sum(1)
            order = np.argsort(d64, kind="stable")[:20]
            assert np.allclose(d, d64[order], rtol=1e-5)
            assert (np.diff(d) >= 0).all() and slot not in s
            assert set(s.tolist()) == set(members[order].tolist()) or np.isclose(d64[order][-1], np.sort(d64)[20], rtol=1e-5)
    # a bucket smaller than P pads with (EMPTY, inf)
    small = O.Index(X[:40], built["attrs"][:40], 4)
    s, d = small.knn(0, 0, 16)
    assert (s[9:] == O.EMPTY).all() and np.isinf(d[9:]).all() and (s[:9] != O.EMPTY).all()


def test_remote_target_order():
    ix = O.Index(np.zeros((64, 32), np.float32), np.arange(64, dtype=np.int32), 16)
    assert ix.remote_targets(8, 8) == [9, 7, 10, 6, 12, 4, 0, 11]      # +-1, +-2, +-4, (+8 outside) -8, then +3
    assert ix.remote_targets(0, 4) == [1, 2, 4, 8]
    assert ix.remote_targets(15, 4) == [14, 13, 11, 7]
    assert ix.remote_targets(1, 20) == [2, 0, 3, 5, 9, 4, 6, 7, 8, 10, 11, 12, 13, 14, 15]   # never more than B-1
    assert ix.remote_targets(3, 3) == [4, 2, 5]
    assert ix.remote_targets(0, 0) == []


def test_forward_lists_obey_the_diversity_rule(built):
    ix, F = built["ix"], built["F"]
    rng = np.random.default_rng(1)
    for u in rng.integers(0, 3000, 40):
        b = int(ix.bucket_of_slots([u])[0])
        cand, cd = ix.knn(int(u), b, 32)
        assert sorted(F[u].tolist()) == sorted(cand.tolist())               # a reordering of the candidates
        kept = []
        order_kept, order_rej = [], []
        for c, d in zip(cand, cd):
            if all(d < O.distance(ix.X[c], ix.X[n]) for n in kept):
                kept.append(c); order_kept.append(c)
            else:
                order_rej.append(c)
        assert F[u].tolist() == order_kept + order_rej


def test_reverse_lists_are_the_definition(built):
    ix, F, R = built["ix"], built["F"], built["R"]
    kl = 16
    occupied = np.nonzero(ix.slot2id != O.EMPTY)[0]
    src_of = {}
    for u in occupied:
        for v in F[u][:kl]:
            if v != O.EMPTY:
                src_of.setdefault(int(v), []).append(int(u))
    rng = np.random.default_rng(2)
    for v in rng.choice(occupied, 60, replace=False):
        srcs = src_of.get(int(v), [])
        key = sorted((float(O.distance(ix.X[u], ix.X[v])), u) for u in srcs)
        want = [u for _, u in key][:kl]
        got = R[v][R[v] != O.EMPTY].tolist()
        assert got == want


def test_interleaved_merge_and_remote_part(built):
    ix, F, R, cfg = built["ix"], built["F"], built["R"], built["cfg"]
    kl, kr = 16, 4
    for u in range(0, 3000, 37):
        merged = []
        for j in range(kl):
            for c in (F[u][j], R[u][j]):
                if c != O.EMPTY and c not in merged:
                    merged.append(int(c))
        assert ix.A[u][:kl].tolist() == (merged + [int(O.EMPTY)] * kl)[:kl]
        b = int(ix.bucket_of_slots([u])[0])
        for j, tb in enumerate(ix.remote_targets(b, kr)):
            assert ix.A[u][kl + j] == ix.knn(u, tb, 1)[0][0]
    A = ix.A
    own = ix.bucket_of_slots(np.arange(3000))[:, None]
    live = A != O.EMPTY
    nb = ix.bucket_of_slots(np.where(live, A, 0))
    assert ((nb[:, :kl] == own) | ~live[:, :kl]).all() and ((nb[:, kl:] != own) | ~live[:, kl:]).all()
    assert (A != np.arange(3000)[:, None]).all() and live.all()
    srt = np.sort(A.astype(np.int64), axis=1)
    assert (np.diff(srt, axis=1) != 0).all()


def test_search_on_the_built_graph_finds_neighbours(built):
    ix, cfg = built["ix"], built["cfg"]
    q = W.query_vectors(cfg)
    lo, hi = W.ranges(cfg, 0.2)
    ids, _, _ = ix.search(q, lo, hi, 10, 64, threads=4)
    gt, _ = O.exact_filtered_knn(built["X"], built["attrs"], q, lo, hi, 10)
    assert O.recall_at_k(ids, gt) > 0.95
