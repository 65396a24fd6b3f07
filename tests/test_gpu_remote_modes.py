"""The proximal/global reading of the remote wiring (construction pass 2 and insertion with a
global-scope candidate search) and the inner-product bias, GPU against oracle, bit for bit
(needs an MI355X)."""
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
    got = ix.get_graph()
    if not np.array_equal(got, ora.A):
        bad = np.nonzero((got != ora.A).any(1))[0]
        raise AssertionError(f"{len(bad)} adjacency rows differ, first slot {bad[0]}: {got[bad[0]]} vs {ora.A[bad[0]]}")


def _set(ix, ora, **kw):
    for k, v in kw.items():
        ix.set_param(k, v)
        ora.params[k] = v


@pytest.mark.parametrize("alpha", [0.6, 1.0])
def test_hand_worked_append_with_proximal_and_global_picks_on_gpu(alpha):
    from paper_2604_16402_amd import binding as B
    g = json.load(open(os.path.join(GOLD, "append_proximal_2d.json")))
    ix = B.Index(32)
    ix.build_buckets(_pad(g["points"]), np.asarray(g["attrs"], np.int32), g["n_buckets"], g["n_cap"])
    for k, v in [("remote_mode", 1), ("n_proximal", g["n_proximal"]), ("remote_window", g["remote_window"]),
                 ("n_seeds", g["n_seeds"]), ("append_beam", g["append_beam"]), ("visited_cap", g["visited_cap"]), ("alpha", alpha)]:
        ix.set_param(k, v)
    ix.load_graph(np.asarray(g["local"], np.uint32), np.asarray(g["remote"], np.uint32))
    ix.append_batch(_pad(g["new_points"]), np.asarray(g["new_attrs"], np.int32))
    want = g[f"alpha_{alpha}"]
    table, id2slot, _ = ix.get_layout()
    assert id2slot[8:10].tolist() == g["new_slots"] and table.tolist() == want["table"]
    assert ix.get_graph().tolist() == want["adj_slots"]
    assert ix.get_append_stats() == want["stats"]
    ix.close()


def _fresh_pair(n, dim, B, n_cap, seed, metric=W.L2SQ, components=16):
    from paper_2604_16402_amd import binding
    cfg = W.Config(f"r{seed}", n, dim, components, 0.3, n, B, 0, 0, 300, (0.1,), metric=metric, seed=seed,
                   normalise=metric == W.IP, append_rounds=3, append_batch=max(64, n // 8))
    X, a = W.base_vectors(cfg), W.attributes(cfg)
    ora = O.Index(X, a, B, n_cap=n_cap, metric=metric)
    ix = binding.Index(dim, metric)
    ix.build_buckets(X, a, B, n_cap)
    return cfg, ix, ora, X, a


@pytest.mark.parametrize("n,dim,B,kl,kr,pool,kp,window,beam,seeds,width", [
    (6000, 128, 8, 16, 4, 32, -1, 0.2, 64, 128, 2),
    (4000, 64, 5, 12, 6, 24, 4, 0.35, 40, 64, 1),       # a queue shorter than 64, a wider window
    (3000, 96, 6, 10, 3, 16, 3, 0.01, 64, 256, 4),      # proximal positions only, a window few candidates fit: fallbacks
    (2500, 960, 3, 12, 4, 20, 0, 0.2, 48, 64, 1),       # no proximal position; long rows
])
def test_two_pass_construction_under_the_second_reading(n, dim, B, kl, kr, pool, kp, window, beam, seeds, width):
    cfg, ix, ora, X, a = _fresh_pair(n, dim, B, n + B * 10, seed=n + dim)
    _set(ix, ora, remote_mode=1, remote_window=window, append_beam=beam, n_seeds=seeds, search_width=width)
    ix.set_param("n_proximal", kp)
    ora.params["n_proximal"] = None if kp < 0 else kp
    ix.build_graph(kl, kr, pool)
    ora.build_graph(kl, kr, pool=pool, threads=O.max_threads())
    _same_index(ix, ora)
    own = ora.bucket_of_slots(np.arange(ora.n_cap))[:, None]
    live = ora.A != O.EMPTY
    leaves = (ora.bucket_of_slots(np.where(live, ora.A, 0)) != own) & live
    assert leaves[:, kl:].any() and not leaves[:, :kl].any()
    if window < 0.05:
        assert (live[:, kl:] & ~leaves[:, kl:]).any()        # redundant local edges were kept somewhere
    # searches over the fused graph agree as well
    q = W.query_vectors(cfg)
    lo, hi = W.ranges(cfg, 0.3)
    ix.set_param("n_seeds", 0); ora.params["n_seeds"] = None
    ids, dist = ix.search_range(q, lo, hi, 10, 64)
    w_ids, w_dist, _ = ora.search(q, lo, hi, 10, 64, threads=O.max_threads())
    assert np.array_equal(dist, w_dist) and np.array_equal(ids, w_ids)
    ix.close()


@pytest.mark.parametrize("mode", [0, 1])
def test_second_pass_alone_on_a_loaded_graph(mode):
    # grab_build_remote on a graph the harness made: 100,000 objects, 16 buckets
    n, B, kl, kr = 100_000, 16, 32, 8
    cfg, ix, ora, X, a = _fresh_pair(n, 128, B, n, seed=4242, components=64)
    la, ra = HG.build_graph(X, ora.bucket_of_ids(), B, kl, kr, device="cuda:0", chunk=8192)
    ix.load_graph(la, ra)
    ora.load_graph(la, ra)
    _set(ix, ora, remote_mode=mode, append_beam=64, n_seeds=128, search_width=2, max_iter=24)
    before = ora.A.copy()
    ix.build_remote()
    if mode == 1:
        ora.build_remote(threads=O.max_threads())
        _same_index(ix, ora)
        assert (ora.A[:, kl:] != before[:, kl:]).mean() > 0.5
    else:
        # the exact nearest object of each target bucket: the oracle's brute force on a sample of rows
        got = ix.get_graph()
        assert np.array_equal(got[:, :kl], before[:, :kl])
        rng = np.random.default_rng(3)
        for u in rng.integers(0, n, 200):
            b = int(ora.bucket_of_slots([u])[0])
            want = [int(ora.knn(int(u), tb, 1)[0][0]) for tb in ora.remote_targets(b, kr)]
            assert got[u, kl:].tolist() == want
    ix.close()


@pytest.mark.parametrize("n,dim,B,kl,kr,n_cap,beam,width,metric,mode", [
    (6000, 128, 8, 16, 4, 9000, 64, 1, W.L2SQ, 1),
    (5000, 64, 5, 24, 8, 8000, 32, 2, W.L2SQ, 1),
    (3000, 960, 3, 20, 4, 4500, 48, 1, W.L2SQ, 1),
    (6000, 96, 6, 16, 4, 9000, 64, 2, W.IP, 1),          # inner product: the shifted bias of Eq. 3
    (6000, 96, 6, 16, 4, 9000, 64, 2, W.IP, 0),
    (100000, 128, 16, 32, 8, 150000, 64, 2, W.L2SQ, 1),
])
def test_append_matches_oracle_under_both_readings(n, dim, B, kl, kr, n_cap, beam, width, metric, mode):
    cfg, ix, ora, X, a = _fresh_pair(n, dim, B, n_cap, seed=n + dim + mode, metric=metric)
    _set(ix, ora, remote_mode=mode, append_beam=beam, search_width=width, n_seeds=96)
    la, ra = HG.build_graph(X, ora.bucket_of_ids(), B, kl, kr, metric=metric, device="cuda:0" if n > 20000 else "cpu", chunk=8192)
    ix.load_graph(la, ra)
    ora.load_graph(la, ra)
    if mode == 1:                        # remote parts as the second reading builds them, on both sides
        ix.build_remote()
        ora.build_remote(threads=O.max_threads())
        _same_index(ix, ora)
    for r in range(3):
        nx, na = W.append_vectors(cfg, r), W.append_attributes(cfg, r)
        if r == 2:
            na = na.copy(); na[:12] = -7 - np.arange(12); na[12:24] = n + 100 + np.arange(12)
        ix.append_batch(nx, na)
        ora.append(nx, na, threads=O.max_threads())
        _same_index(ix, ora)
        assert ix.get_append_stats() == ora.last_append_stats      # the same work, counted the same way
    new = ora.id2slot[n:ora.n]
    indeg = np.bincount(ora.A[ora.A != O.EMPTY].astype(np.int64), minlength=ora.n_cap)
    assert (indeg[new] > 0).mean() > 0.98
    q = W.query_vectors(cfg)
    rng = np.random.default_rng(1)
    lo = rng.integers(-20, n, len(q)).astype(np.int32)
    hi = (lo + rng.integers(1, n // 2, len(q))).astype(np.int32)
    ix.set_param("n_seeds", 0); ora.params["n_seeds"] = None
    ids, dist = ix.search_range(q, lo, hi, 10, 64)
    w_ids, w_dist, w_ctr = ora.search(q, lo, hi, 10, 64, threads=O.max_threads())
    assert np.array_equal(dist, w_dist) and np.array_equal(ids, w_ids) and np.array_equal(ix.get_counters(len(q)), w_ctr)
    ix.close()


def test_bad_rule_parameters_are_refused():
    from paper_2604_16402_amd import binding as B
    cfg, ix, ora, X, a = _fresh_pair(2000, 64, 4, 2400, seed=9)
    ix.set_param("remote_mode", 1)
    ix.set_param("n_proximal", 5)
    with pytest.raises(B.GrabError) as e:
        ix.build_graph(8, 4, 16)
    assert e.value.status == B.EINVAL and ix.sizes()["has_graph"] == 0
    for name, bad in [("remote_mode", 2), ("n_proximal", 65), ("n_proximal", -2), ("remote_window", 1.5), ("remote_window", -0.1)]:
        with pytest.raises(B.GrabError):
            ix.set_param(name, bad)
    with pytest.raises(B.GrabError) as e:
        ix.build_remote()
    assert e.value.status == B.ESTATE
    ix.close()
