"""Batched insertion on the GPU against the oracle, bit for bit (needs an MI355X)."""
import json
import os

import numpy as np
import pytest

from oracle import oracle as O
from harness import graphs as HG
from paper_2604_16402_amd import workloads as W

pytestmark = pytest.mark.gpu
GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _pad(points, dim=32):
    out = np.zeros((len(points), dim), np.float32)
    out[:, :len(points[0])] = np.asarray(points, np.float32)
    return out


def _same_index(ix, ora):
    table, id2slot, slot2id = ix.get_layout()
    assert np.array_equal(table, ora.table)
    assert np.array_equal(id2slot, ora.id2slot[:ora.n])
    assert np.array_equal(slot2id, ora.slot2id)
    x, a = ix.get_rows()
    live = ora.slot2id != O.EMPTY
    assert np.array_equal(x[live], ora.X[live]) and np.array_equal(a[live], ora.attr[live])
    got = ix.get_graph()
    if not np.array_equal(got, ora.A):
        bad = np.nonzero((got != ora.A).any(1))[0]
        raise AssertionError(f"{len(bad)} adjacency rows differ, first slot {bad[0]}: {got[bad[0]]} vs {ora.A[bad[0]]}")


@pytest.mark.parametrize("alpha", [0.6, 1.0])
def test_hand_worked_append_on_gpu(alpha):
    from paper_2604_16402_amd import binding as B
    g = json.load(open(os.path.join(GOLD, "append_2d.json")))
    ix = B.Index(32)
    ix.build_buckets(_pad(g["points"]), np.asarray(g["attrs"], np.int32), g["n_buckets"], g["n_cap"])
    ix.load_graph(np.asarray(g["local"], np.uint32), np.asarray(g["remote"], np.uint32))
    for k, v in [("n_seeds", g["n_seeds"]), ("append_beam", g["append_beam"]), ("visited_cap", g["visited_cap"]), ("alpha", alpha)]:
        ix.set_param(k, v)
    ix.append_batch(_pad(g["new_points"]), np.asarray(g["new_attrs"], np.int32))
    want = g[f"alpha_{alpha}"]
    table, id2slot, slot2id = ix.get_layout()
    assert id2slot[8:10].tolist() == g["new_slots"] and table.tolist() == want["table"]
    assert ix.get_graph().tolist() == want["adj_slots"]
    assert ix.sizes()["n"] == 10
    ix.close()


def test_hand_worked_victim_choice_on_gpu():
    from paper_2604_16402_amd import binding as B
    g = json.load(open(os.path.join(GOLD, "append_victim_1d.json")))

    def line(c):
        out = np.zeros((len(c), 32), np.float32)
        out[:, 0] = np.asarray(c, np.float32)
        return out
    ix = B.Index(32)
    ix.build_buckets(line(g["coords"]), np.asarray(g["attrs"], np.int32), g["n_buckets"], g["n_cap"])
    ix.load_graph(np.asarray(g["local"], np.uint32), None)
    for k, v in [("n_seeds", g["n_seeds"]), ("append_beam", g["append_beam"]), ("alpha", g["alpha"])]:
        ix.set_param(k, v)
    ix.append_batch(line([g["new_coord"]]), np.asarray([g["new_attr"]], np.int32))
    assert ix.get_graph().tolist() == g["adj_slots_after"]
    ix.close()


def _pair(n, dim, B, kl, kr, n_cap, seed, components=16, metric=W.L2SQ, batch=None):
    import torch
    from paper_2604_16402_amd import binding
    cfg = W.Config(f"a{seed}", n, dim, components, 0.3, n, B, kl, kr, 400, (0.1,), metric=metric, seed=seed,
                   append_rounds=3, append_batch=batch or max(64, n // 8))
    X, a = W.base_vectors(cfg), W.attributes(cfg)
    ora = O.Index(X, a, B, n_cap=n_cap, metric=metric)
    la, ra = HG.build_graph(X, ora.bucket_of_ids(), B, kl, kr, metric=metric,
                           device="cuda:0" if n > 20000 else "cpu", chunk=8192)
    ora.load_graph(la, ra)
    ix = binding.Index(dim, metric)
    ix.build_buckets(X, a, B, n_cap)
    ix.load_graph(la, ra)
    return cfg, ix, ora, X, a


@pytest.mark.parametrize("n,dim,B,kl,kr,n_cap,beam,width,rcands", [
    (6000, 128, 8, 16, 4, 9000, 64, 1, 0),
    (5000, 64, 5, 24, 8, 8000, 32, 2, 0),
    (3000, 960, 3, 20, 4, 4500, 48, 1, 0),
    (100000, 128, 16, 32, 8, 150000, 64, 1, 0),
    (6000, 128, 8, 16, 4, 9000, 128, 2, 24),      # remote parts from the nearest 24 of 128 candidates
    (4000, 160, 4, 12, 4, 6000, 64, 1, 0),        # five 128-byte lines per row
    (4000, 384, 4, 12, 4, 6000, 64, 1, 8),
])
def test_append_matches_oracle(n, dim, B, kl, kr, n_cap, beam, width, rcands):
    cfg, ix, ora, X, a = _pair(n, dim, B, kl, kr, n_cap, seed=n + dim)
    for k, v in [("append_beam", beam), ("search_width", width), ("append_remote_cands", rcands)]:
        ix.set_param(k, v)
        ora.params[k] = v
    allX, alla = [X], [a]
    for r in range(3):
        nx, na = W.append_vectors(cfg, r), W.append_attributes(cfg, r)
        if r == 2:                                  # attributes outside every bucket interval widen the edge buckets
            na = na.copy(); na[:12] = -7 - np.arange(12); na[12:24] = n + 100 + np.arange(12)
        ix.append_batch(nx, na)
        ora.append(nx, na, threads=O.max_threads())
        _same_index(ix, ora)
        assert ix.get_append_stats() == ora.last_append_stats      # the same work, counted the same way
        allX.append(nx); alla.append(na)
    # searches over the grown index: tails are live, so the attribute-read path is exercised
    q = W.query_vectors(cfg)
    rng = np.random.default_rng(1)
    lo = rng.integers(-20, n, len(q)).astype(np.int32)
    hi = (lo + rng.integers(1, n // 2, len(q))).astype(np.int32)
    ids, dist = ix.search_range(q, lo, hi, 10, 64)
    ctr = ix.get_counters(len(q))
    w_ids, w_dist, w_ctr = ora.search(q, lo, hi, 10, 64, threads=O.max_threads())
    assert np.array_equal(dist, w_dist) and np.array_equal(ids, w_ids) and np.array_equal(ctr, w_ctr)
    assert ctr[:, 5].sum() > 0                      # some pre-checks had to read a tail attribute
    allX, alla = np.concatenate(allX), np.concatenate(alla)
    gt, _ = O.exact_filtered_knn(allX, alla, q[:100], lo[:100], hi[:100], 10)
    assert O.recall_at_k(ids[:100], gt) > 0.75     # soft: the graph is small and shallow here
    assert (ids[ids != 0xFFFFFFFF] >= n).any()
    ix.close()


@pytest.mark.parametrize("mode", [0, 1])
def test_targets_with_more_than_64_requests(mode):
    # a small index and a large batch: every existing object is asked for an edge by far more new
    # objects than one wavefront holds at once, so the rewiring walks its request lists in pages
    cfg, ix, ora, X, a = _pair(400, 64, 4, 8, 4, 400 + 4 * 3600, seed=31, components=4, batch=6000)
    for k, v in [("append_beam", 32), ("n_seeds", 32), ("remote_mode", mode)]:
        ix.set_param(k, v)
        ora.params[k] = v
    for r in range(2):
        nx, na = W.append_vectors(cfg, r), W.append_attributes(cfg, r)
        ix.append_batch(nx, na)
        ora.append(nx, na, threads=O.max_threads())
        _same_index(ix, ora)
        st = ix.get_append_stats()
        assert st == ora.last_append_stats
        if r == 0:
            assert st["requests_local"] > 64 * st["groups_local"] and st["requests_remote"] > 0
    ix.close()


def test_full_bucket_reports_efull_and_writes_nothing():
    from paper_2604_16402_amd import binding as B
    cfg, ix, ora, X, a = _pair(3000, 64, 4, 12, 3, 3000 + 4 * 20, seed=77)
    before = (ix.get_layout(), ix.get_graph(), ix.get_rows())
    nx, na = W.append_vectors(cfg, 0), W.append_attributes(cfg, 0)
    with pytest.raises(B.GrabError) as e:
        ix.append_batch(nx, na)
    assert e.value.status == B.EFULL
    after = (ix.get_layout(), ix.get_graph(), ix.get_rows())
    for x, y in zip(before, after):
        if isinstance(x, tuple):
            assert all(np.array_equal(p, q) for p, q in zip(x, y))
        else:
            assert np.array_equal(x, y)
    ix.append_batch(nx[:30], na[:30])               # a batch that fits still goes through
    ora.append(nx[:30], na[:30])
    _same_index(ix, ora)
    with pytest.raises(B.GrabError) as e:
        ix.append_batch(nx[:0].reshape(0, 64), na[:0]) if False else ix.append_batch(nx[:200], na[:200])
    assert e.value.status == B.EFULL
    ix.close()


def test_append_twice_from_the_same_state_gives_identical_bytes():
    outs = []
    for _ in range(2):
        cfg, ix, ora, X, a = _pair(4000, 128, 4, 16, 4, 6000, seed=5)
        ix.append_batch(W.append_vectors(cfg, 0), W.append_attributes(cfg, 0))
        outs.append((ix.get_graph(), ix.get_layout()[0], ix.get_layout()[1]))
        ix.close()
    assert all(np.array_equal(x, y) for x, y in zip(*outs))
