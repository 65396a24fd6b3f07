"""Two-pass graph construction on the GPU against the oracle (needs an MI355X)."""
import numpy as np
import pytest

from oracle import oracle as O
from paper_2604_16402_amd import workloads as W

pytestmark = pytest.mark.gpu


def _case(n, dim, B, metric, seed, n_cap=None):
    cfg = W.Config(f"g{seed}", n, dim, 12, 0.4, n, B, 0, 0, 300, (0.2,), metric=metric,
                   normalise=(metric == W.IP), seed=seed)
    X, a = W.base_vectors(cfg), W.attributes(cfg)
    return cfg, X, a


@pytest.mark.parametrize("n,dim,B,kl,kr,pool,metric,n_cap", [
    (3000, 128, 6, 16, 4, 32, W.L2SQ, None),
    (2500, 64, 5, 12, 8, 0, W.L2SQ, 3000),      # pool default, more remote entries than buckets allow, slack
    (2000, 96, 4, 20, 2, 40, W.IP, None),
    (1500, 960, 3, 8, 2, 24, W.L2SQ, None),
    (1500, 160, 3, 12, 3, 24, W.L2SQ, None),
    (1500, 640, 3, 12, 3, 24, W.L2SQ, None),
    (1500, 384, 3, 12, 3, 24, W.IP, 1800),
    (700, 32, 9, 33, 5, 64, W.L2SQ, None),      # buckets (~78 rows) barely larger than the pool
    (300, 32, 6, 32, 3, 64, W.L2SQ, None),      # buckets (50 rows) smaller than the pool: short lists
    (4000, 128, 5, 32, 4, 128, W.L2SQ, None),   # 128 candidates: two per lane
    (2600, 64, 4, 20, 3, 100, W.L2SQ, 3000),    # a pool that is not a power of two
])
def test_build_graph_matches_oracle(n, dim, B, kl, kr, pool, metric, n_cap):
    from paper_2604_16402_amd import binding
    cfg, X, a = _case(n, dim, B, metric, seed=n + dim)
    ora = O.Index(X, a, B, n_cap=n_cap, metric=metric)
    ora.build_graph(kl, kr, pool=pool or min(4 * kl, 128), threads=O.max_threads())
    ix = binding.Index(dim, metric)
    ix.build_buckets(X, a, B, n_cap)
    ix.build_graph(kl, kr, pool)
    got = ix.get_graph()
    if not np.array_equal(got, ora.A):
        bad = np.nonzero((got != ora.A).any(1))[0]
        raise AssertionError(f"{len(bad)} rows differ; slot {bad[0]}: {got[bad[0]].tolist()} vs {ora.A[bad[0]].tolist()}")
    assert ix.sizes()["has_graph"] == 1 and ix.sizes()["k_local"] == kl
    # the built graph is searchable and the search still matches the oracle on it
    q = W.query_vectors(cfg)
    lo, hi = W.ranges(cfg, 0.3)
    ids, dist = ix.search_range(q, lo, hi, 10, 64)
    w_ids, w_dist, _ = ora.search(q, lo, hi, 10, 64)
    assert np.array_equal(ids, w_ids) and np.array_equal(dist, w_dist)
    ix.close()


@pytest.mark.parametrize("kind", ["copies", "far_from_origin", "a_few_copies"])
def test_build_graph_where_the_score_filter_cannot_decide(kind):
    # construction filters nearest-neighbour candidates by low-precision scores with a proven margin and
    # re-ranks the survivors exactly; where the margin admits more candidates than its lists hold (hundreds
    # of equal distances; distances tiny against the norms) it must fall back to evaluating every pair
    from paper_2604_16402_amd import binding
    rng = np.random.default_rng(17)
    n, dim, B, kl, kr, pool = 3000, 64, 3, 16, 3, 32
    if kind == "copies":                 # two distinct vectors: about 500 ties at distance zero per bucket
        X = rng.standard_normal((2, dim)).astype(np.float32)[rng.integers(0, 2, n)]
    elif kind == "a_few_copies":         # 40 distinct vectors: ties well inside what the lists hold
        X = rng.standard_normal((40, dim)).astype(np.float32)[rng.integers(0, 40, n)]
    else:                                # a tight cloud a thousand units from the origin
        X = (1000.0 + 0.01 * rng.standard_normal((n, dim))).astype(np.float32)
    a = rng.integers(0, n, n).astype(np.int32)
    ora = O.Index(X, a, B)
    ora.build_graph(kl, kr, pool=pool, threads=O.max_threads())
    ix = binding.Index(dim)
    ix.build_buckets(X, a, B)
    ix.build_graph(kl, kr, pool)
    assert np.array_equal(ix.get_graph(), ora.A)
    ix.close()


def test_build_graph_after_append_covers_the_tails():
    from paper_2604_16402_amd import binding
    cfg, X, a = _case(2400, 64, 4, W.L2SQ, seed=9)
    ora = O.Index(X[:2000], a[:2000], 4, n_cap=2600)
    ix = binding.Index(64)
    ix.build_buckets(X[:2000], a[:2000], 4, 2600)
    ora.build_graph(12, 3, pool=24)
    ix.build_graph(12, 3, 24)
    ora.append(X[2000:], a[2000:])
    ix.append_batch(X[2000:], a[2000:])
    assert np.array_equal(ix.get_graph(), ora.A)
    ora.build_graph(12, 3, pool=24)             # rebuild over sorted prefixes and appended tails alike
    ix.build_graph(12, 3, 24)
    assert np.array_equal(ix.get_graph(), ora.A)
    ix.close()


def test_build_graph_rejects_bad_arguments():
    from paper_2604_16402_amd import binding as B
    ix = B.Index(32)
    with pytest.raises(B.GrabError) as e:
        ix.build_graph(8, 2, 16)
    assert e.value.status == B.ESTATE
    ix.build_buckets(np.zeros((50, 32), np.float32), np.arange(50, dtype=np.int32), 2)
    for kl, kr, pool in [(0, 2, 8), (70, 2, 64), (8, 70, 16), (8, 2, 4), (8, 2, 200)]:
        with pytest.raises(B.GrabError) as e:
            ix.build_graph(kl, kr, pool)
        assert e.value.status == B.EINVAL
    ix.close()


def test_full_size_build_properties_and_recall():
    # 1M x 128, 64 buckets, degree 32+8: sampled rows against what the oracle can compute one by
    # one, structural properties on every row, and search recall on the built graph
    import time
    import torch
    from harness import groundtruth as GT
    from paper_2604_16402_amd import binding
    dev = torch.device("cuda:0")
    cfg = W.CONFIGS["c2"]
    X, a, q = W.base_vectors(cfg), W.attributes(cfg), W.query_vectors(cfg)
    kl, kr, pool = cfg.k_local, cfg.k_remote, 128
    ix = binding.Index(cfg.dim, cfg.metric, stream=torch.cuda.current_stream(dev).cuda_stream)
    Xd, ad = torch.from_numpy(X).to(dev), torch.from_numpy(a).to(dev)
    ix.build_buckets(Xd, ad, cfg.buckets)
    t0 = time.time()
    ix.build_graph(kl, kr, pool)
    print(f"build_graph 1M x 128: {time.time() - t0:.2f}s")
    ora = O.Index(X, a, cfg.buckets)
    A = ix.get_graph()
    n = cfg.n
    own = ora.bucket_of_slots(np.arange(n))
    live = A != O.EMPTY
    nb = ora.bucket_of_slots(np.where(live, A, 0))
    assert live.all()
    assert (nb[:, :kl] == own[:, None]).all() and (nb[:, kl:] != own[:, None]).all()
    assert (A != np.arange(n)[:, None]).all()
    assert (np.diff(np.sort(A.astype(np.int64), axis=1), axis=1) != 0).all()

    def forward(u):
        cand, cd = ora.knn(int(u), int(own[u]), pool)
        kept, rej = [], []
        for c, d in zip(cand, cd):
            (kept if all(d < O.distance(ora.X[c], ora.X[m]) for m in kept) else rej).append(int(c))
        return kept + rej

    rng = np.random.default_rng(0)
    for u in rng.integers(0, n, 40):
        F = forward(u)
        row = A[u][:kl].tolist()
        assert row[0] == F[0]                                          # the nearest neighbour leads the row
        missing = [c for c in F[:kl] if c not in row]
        assert len(missing) <= sum(1 for v in row if v not in F[:kl])   # forward entries only yield to reverse edges
        for v in row:
            if v not in F[:kl]:
                assert int(u) in forward(v)[:kl]                       # every other entry is a reverse edge
        for j, tb in enumerate(ora.remote_targets(int(own[u]), kr)):
            assert A[u][kl + j] == ora.knn(int(u), tb, 1)[0][0]        # nearest node of the target bucket
    lo, hi = W.ranges(cfg, 0.1)
    qd, lod, hid = torch.from_numpy(q).to(dev), torch.from_numpy(lo).to(dev), torch.from_numpy(hi).to(dev)
    ids = torch.empty((len(q), 10), dtype=torch.int32, device=dev)
    dist = torch.empty((len(q), 10), dtype=torch.float32, device=dev)
    ix.set_param("visited_cap", 1400); ix.set_param("n_seeds", 64); ix.set_param("search_width", 2)
    ix.search_range(qd, lod, hid, 10, 32, ids, dist)
    gt = GT.exact_filtered_knn(Xd, ad, qd, lod, hid, 10)
    rec = GT.recall(ids, gt)
    print(f"recall@10 on the library-built graph: {rec:.4f}")
    assert rec >= 0.95
    ix.close()
