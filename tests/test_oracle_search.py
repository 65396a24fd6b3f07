"""Pins for the oracle's range-constrained beam search (Algorithm 2; Hybrid Search
definition, Section 2.4; Recall@k, Eq. 1)."""
import json
import os

import numpy as np
import pytest

from oracle import oracle as O
from paper_2604_16402_amd import workloads as W

GOLD = os.path.join(os.path.dirname(__file__), "golden")
NAMES = ["iters", "parents", "evals", "seed_evals", "rejects", "tail", "visited", "stop"]


def _pad(points, dim=32):
    out = np.zeros((len(points), dim), np.float32)
    out[:, :len(points[0])] = np.asarray(points, np.float32)
    return out


def test_hand_traced_example():
    g = json.load(open(os.path.join(GOLD, "trace_2d.json")))
    ix = O.Index(_pad(g["points"]), np.asarray(g["attrs"], np.int32), g["n_buckets"])
    ix.load_graph(np.asarray(g["local"], np.uint32), np.asarray(g["remote"], np.uint32))
    q = _pad([g["query"]])
    ix.params.update(n_seeds=g["n_seeds"], search_width=g["search_width"])
    info, seeds = ix.select(g["lo"], g["hi"], g["beam"])
    e = g["expected_select"]
    assert info.tolist() == [e["b0"], e["b1"], e["V"], e["first_valid_slot"], e["end_valid_slot"], len(e["seeds"])]
    assert seeds.tolist() == e["seeds"]
    for case in g["cases"]:
        ix.params.update(max_iter=case["max_iter"], visited_cap=case["visited_cap"])
        ids, dist, ctr = ix.search(q, np.array([g["lo"]]), np.array([g["hi"]]), g["k"], g["beam"])
        assert ids[0].tolist() == case["ids"], case
        assert dist[0].tolist() == case["dist"], case
        got = dict(zip(NAMES, ctr[0].tolist()))
        for name, want in case["counters"].items():
            assert got[name] == want, (name, case)


def _check_invariants(ids, dist, attrs, lo, hi):
    for r, d, l, h in zip(ids, dist, lo, hi):
        live = r != O.EMPTY
        n = int(live.sum())
        assert live[:n].all() and not live[n:].any()                 # padding only at the end
        assert np.isinf(d[n:]).all()
        assert ((attrs[r[:n]] >= l) & (attrs[r[:n]] <= h)).all()      # condition (2): lo <= s_i <= hi
        assert (np.diff(d[:n]) >= 0).all()                            # ascending distance
        assert len(set(r[:n].tolist())) == n                          # no duplicates


def test_invariants_on_config1(c1_small):
    c = c1_small
    ids, dist, _ = c["oracle"].search(c["queries"], c["lo"], c["hi"], 10, 64)
    _check_invariants(ids, dist, c["attrs"], c["lo"], c["hi"])
    # reported distances are the distances of the reported ids
    for i in range(0, 1000, 97):
        for j in range(10):
            assert dist[i, j] == O.distance(c["queries"][i], c["X"][ids[i, j]])


def test_small_population_gives_exact_answer(c1_small):
    # V <= S: every valid object is a seed, so the result is the exhaustive filtered k-NN
    c = c1_small
    ix = c["oracle"]
    rng = np.random.default_rng(1)
    lo = rng.integers(0, 9900, 200).astype(np.int32)
    hi = (lo + rng.integers(0, 60, 200)).astype(np.int32)
    ix.params.update(n_seeds=64)
    ids, dist, ctr = ix.search(c["queries"][:200], lo, hi, 10, 64)
    gt, gd = O.exact_filtered_knn(c["X"], c["attrs"], c["queries"][:200], lo, hi, 10)
    small = np.array([((c["attrs"] >= l) & (c["attrs"] <= h)).sum() <= 64 for l, h in zip(lo, hi)])
    assert small.sum() > 100
    assert (ids[small] == gt[small]).all()
    assert np.allclose(dist[small], gd[small], rtol=1e-5, atol=0, equal_nan=False) or \
        np.array_equal(np.isinf(dist[small]), np.isinf(gd[small]))
    ix.params.update(n_seeds=None)
    _check_invariants(ids, dist, c["attrs"], lo, hi)


def test_complete_graph_equals_brute_force():
    # K >= n-1 inside one bucket and the full range: one expansion reaches everything
    rng = np.random.default_rng(2)
    n, dim = 40, 32
    X = rng.standard_normal((n, dim)).astype(np.float32)
    attrs = rng.permutation(n).astype(np.int32)
    ix = O.Index(X, attrs, 1)
    local = np.array([[j for j in range(n) if j != i] for i in range(n)], np.uint32)
    ix.load_graph(local, np.zeros((n, 0), np.uint32))
    q = rng.standard_normal((25, dim)).astype(np.float32)
    lo = np.zeros(25, np.int32); hi = np.full(25, n, np.int32)
    ix.params.update(n_seeds=1, max_iter=1, visited_cap=1000)
    ids, dist, ctr = ix.search(q, lo, hi, 10, 64)
    gt, gd = O.exact_filtered_knn(X, attrs, q, lo, hi, 10)
    assert (ids == gt).all()
    assert (ctr[:, 2] == n).all()                                      # every object evaluated exactly once


def test_wide_beam_on_connected_valid_subgraph_is_exact():
    # beam >= V and a ring inside the valid set: the search must enumerate all of it
    rng = np.random.default_rng(4)
    n, dim = 300, 64
    X = rng.standard_normal((n, dim)).astype(np.float32)
    attrs = np.arange(n, dtype=np.int32)
    ix = O.Index(X, attrs, 3)
    local = np.full((n, 2), O.EMPTY, np.uint32)
    for b in range(3):
        for i in range(100):
            local[b * 100 + i] = [b * 100 + (i + 1) % 100, b * 100 + (i - 1) % 100]
    remote = np.array([[(i + 100) % n] for i in range(n)], np.uint32)
    ix.load_graph(local, remote)
    q = rng.standard_normal((20, dim)).astype(np.float32)
    lo = np.zeros(20, np.int32); hi = np.full(20, 299, np.int32)
    ix.params.update(n_seeds=2, max_iter=10000, visited_cap=5000)
    ids, dist, ctr = ix.search(q, lo, hi, 10, 512)
    gt, _ = O.exact_filtered_knn(X, attrs, q, lo, hi, 10)
    assert (ids == gt).all() and (ctr[:, 6] == n).all()
    # a filter that cuts the ring still never returns an object outside it
    lo[:] = 50; hi[:] = 249
    ids, dist, _ = ix.search(q, lo, hi, 10, 512)
    _check_invariants(ids, dist, attrs, lo, hi)


def test_degenerate_ranges(c1_small):
    c = c1_small
    q = c["queries"][:3]
    ids, dist, ctr = c["oracle"].search(q, np.array([10, 20000, -5], np.int32), np.array([5, 30000, -1], np.int32), 10, 64)
    assert (ids == O.EMPTY).all() and np.isinf(dist).all() and (ctr[:, 7] == 3).all()
    # a single-value range returns exactly the objects carrying that value
    val = int(c["attrs"][0])
    ids, dist, _ = c["oracle"].search(q[:1], np.array([val], np.int32), np.array([val], np.int32), 10, 64)
    want = np.nonzero(c["attrs"] == val)[0]
    got = ids[0][ids[0] != O.EMPTY]
    assert set(got.tolist()) == set(want[:10].tolist()) or len(want) > 10


def test_recall_is_high_and_rises_with_beam(c1_small):
    # Section 5 (hyper-parameter study): a larger candidate queue raises recall
    c = c1_small
    ix = c["oracle"]
    gt, _ = O.exact_filtered_knn(c["X"], c["attrs"], c["queries"], c["lo"], c["hi"], 10)
    rec = {}
    for beam in (16, 64):
        ids, _, _ = ix.search(c["queries"], c["lo"], c["hi"], 10, beam)
        rec[beam] = O.recall_at_k(ids, gt)
    assert rec[64] >= 0.95 and rec[64] >= rec[16]


def test_search_is_deterministic_and_thread_independent(c1_small):
    c = c1_small
    a = c["oracle"].search(c["queries"][:200], c["lo"][:200], c["hi"][:200], 10, 64, threads=1)
    b = c["oracle"].search(c["queries"][:200], c["lo"][:200], c["hi"][:200], 10, 64, threads=4)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


def test_search_width_and_caps_change_only_what_they_should(c1_small):
    c = c1_small
    ix = c["oracle"]
    q, lo, hi = c["queries"][:100], c["lo"][:100], c["hi"][:100]
    ix.params.update(search_width=4, max_iter=7)
    ids, dist, ctr = ix.search(q, lo, hi, 10, 64)
    assert (ctr[:, 0] <= 7).all() and (ctr[:, 1] <= 28).all() and (ctr[:, 7] == 1).any()
    _check_invariants(ids, dist, c["attrs"], lo, hi)
    ix.params.update(search_width=1, max_iter=None, visited_cap=200)
    ids, dist, ctr = ix.search(q, lo, hi, 10, 64)
    assert (ctr[:, 6] <= 200).all() and (ctr[:, 7] == 2).any()
    ix.params.update(visited_cap=2800)


def test_exact_knn_and_recall_definitions():
    X = _pad([[0, 0], [1, 0], [2, 0], [3, 0], [4, 0]])
    attrs = np.array([0, 1, 2, 3, 4], np.int32)
    q = _pad([[2.2, 0]])
    ids, d = O.exact_filtered_knn(X, attrs, q, [1], [4], 3)
    assert ids[0].tolist() == [2, 3, 1]
    assert np.allclose(d[0], [0.04, 0.64, 1.44])
    ids, d = O.exact_filtered_knn(X, attrs, q, [3], [4], 3)
    assert ids[0].tolist() == [3, 4, int(O.EMPTY)] and np.isinf(d[0, 2])
    assert O.recall_at_k(np.array([[2, 3, 0]], np.uint32), np.array([[2, 3, 1]], np.uint32)) == pytest.approx(2 / 3)
    assert O.recall_at_k(np.array([[3, 4, O.EMPTY]], np.uint32), ids) == 1.0
