"""HIP path against the CPU oracle, element by element, through the C ABI (needs an MI355X)."""
import numpy as np
import pytest

from oracle import oracle as O
from harness import graphs as HG
from paper_2604_16402_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_dev():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return torch.device("cuda:0")


def _gpu_index(c, dev, n_cap=None):
    import torch
    from paper_2604_16402_amd import binding
    cfg = c["cfg"]
    ix = binding.Index(cfg.dim, cfg.metric, stream=torch.cuda.current_stream(dev).cuda_stream)
    ix.build_buckets(torch.from_numpy(c["X"]).to(dev), torch.from_numpy(c["attrs"]).to(dev), cfg.buckets, n_cap)
    ix.load_graph(torch.from_numpy(c["local"].view(np.int32)).to(dev), torch.from_numpy(c["remote"].view(np.int32)).to(dev))
    return ix


def _search_gpu(ix, dev, q, lo, hi, k, beam):
    import torch
    ids = torch.empty((len(q), k), dtype=torch.int32, device=dev)
    dist = torch.empty((len(q), k), dtype=torch.float32, device=dev)
    ix.search_range(torch.from_numpy(q).to(dev), torch.from_numpy(lo).to(dev), torch.from_numpy(hi).to(dev), k, beam, ids, dist)
    torch.cuda.synchronize()
    return ids.cpu().numpy().view(np.uint32), dist.cpu().numpy(), ix.get_counters(len(q))


def test_layout_is_bit_exact(c1_small, torch_dev):
    ix = _gpu_index(c1_small, torch_dev)
    ora = c1_small["oracle"]
    table, id2slot, slot2id = ix.get_layout()
    assert np.array_equal(table, ora.table)
    assert np.array_equal(id2slot, ora.id2slot[:ora.n])
    assert np.array_equal(slot2id, ora.slot2id)
    x, a = ix.get_rows()
    assert np.array_equal(x, ora.X) and np.array_equal(a, ora.attr)
    assert np.array_equal(ix.get_graph(), ora.A)
    ix.close()


def test_selection_and_seeds_are_bit_exact(c1_small, torch_dev):
    ix = _gpu_index(c1_small, torch_dev)
    ora = c1_small["oracle"]
    rng = np.random.default_rng(0)
    lo = np.concatenate([c1_small["lo"][:200], rng.integers(-50, 10050, 300)]).astype(np.int32)
    hi = np.concatenate([c1_small["hi"][:200], lo[200:] + rng.integers(-5, 6000, 300)]).astype(np.int32)
    info, seeds = ix.select_range(lo, hi, 64)
    for i in range(len(lo)):
        want_info, want_seeds = ora.select(int(lo[i]), int(hi[i]), 64)
        assert info[i].tolist() == want_info.tolist(), (i, lo[i], hi[i])
        assert np.array_equal(seeds[i], want_seeds), (i, lo[i], hi[i])
    ix.close()


@pytest.mark.parametrize("domain", [25, 1 << 20])
def test_selection_across_the_fence_of_an_edge_bucket(torch_dev, domain):
    """Buckets of 20,000 objects: more than 128 fence entries (the fence itself needs two probing steps), a sorted
    prefix that is no multiple of the fence distance, and, with 25 distinct attribute values, runs of equal
    attributes that span a dozen fence entries; bounds on, just below and just above stored values."""
    import torch
    from paper_2604_16402_amd import binding
    n, B, dim = 80_001, 4, 32
    rng = np.random.default_rng(domain)
    X = rng.standard_normal((n, dim)).astype(np.float32)
    a = rng.integers(0, domain, n).astype(np.int32)
    ora = O.Index(X, a, B, n_cap=n)
    ix = binding.Index(dim, W.L2SQ, stream=torch.cuda.current_stream(torch_dev).cuda_stream)
    ix.build_buckets(torch.from_numpy(X).to(torch_dev), torch.from_numpy(a).to(torch_dev), B, n)
    if domain == 25:
        v = np.arange(-2, 28, dtype=np.int32)
        lo, hi = [g.ravel() for g in np.meshgrid(v, v, indexing="ij")]
    else:
        srt = np.sort(a)
        at = srt[rng.integers(0, n, 400)]                      # stored values, many of them next to a fence entry
        at[:200] = srt[(rng.integers(0, n // 128, 200) * 128) % n]
        lo = (at + rng.integers(-1, 2, 400)).astype(np.int32)
        hi = (lo + rng.integers(-3, domain // 3, 400)).astype(np.int32)
        hi[::7] = srt[rng.integers(0, n, len(hi[::7]))]
    info, seeds = ix.select_range(lo.astype(np.int32), hi.astype(np.int32), 64)
    for i in range(len(lo)):
        want_info, want_seeds = ora.select(int(lo[i]), int(hi[i]), 64)
        assert info[i].tolist() == want_info.tolist(), (i, lo[i], hi[i])
        assert np.array_equal(seeds[i], want_seeds), (i, lo[i], hi[i])
    ix.close()


@pytest.mark.parametrize("beam,width", [(64, 1), (128, 1), (64, 4), (40, 2)])
def test_search_matches_oracle_exactly(c1_small, torch_dev, beam, width):
    c = c1_small
    ix = _gpu_index(c, torch_dev)
    ora = c["oracle"]
    ix.set_param("search_width", width)
    ora.params.update(search_width=width)
    try:
        ids, dist, ctr = _search_gpu(ix, torch_dev, c["queries"], c["lo"], c["hi"], 10, beam)
        want_ids, want_dist, want_ctr = ora.search(c["queries"], c["lo"], c["hi"], 10, beam)
    finally:
        ora.params.update(search_width=1)
        ix.close()
    assert np.array_equal(dist, want_dist)           # fp32 bits equal: same summation tree
    assert np.array_equal(ids, want_ids)
    assert np.array_equal(ctr, want_ctr)             # same traversal, step for step


def test_launch_order_survives_batches_of_changing_size(c1_small, torch_dev):
    """Batches of 2,048 queries and more run in bucket order, filed by counters that two calls use in turn and the
    later call clears: batches of different sizes, one after the other on one index, must all match the oracle (a
    rank left over from an earlier call would send two queries to one place of the order and leave one unanswered)."""
    c = c1_small
    ix = _gpu_index(c, torch_dev)
    ora = c["oracle"]
    rng = np.random.default_rng(5)
    try:
        want = {}
        for nq in (2300, 4100, 2300, 300, 2048, 4100):
            pick = rng.integers(0, len(c["queries"]), nq)
            q, lo, hi = c["queries"][pick], c["lo"][pick].copy(), c["hi"][pick].copy()
            lo[::9] = 20000                                   # some queries select nothing: the extra bin
            ids, dist, ctr = _search_gpu(ix, torch_dev, q, lo, hi, 10, 32)
            if "all" not in want:
                want["all"] = ora.search(c["queries"], c["lo"], c["hi"], 10, 32)
            w_ids, w_dist, w_ctr = (x[pick] for x in want["all"])
            none = np.arange(nq) % 9 == 0
            assert np.array_equal(ids[~none], w_ids[~none]) and np.array_equal(dist[~none], w_dist[~none])
            assert np.array_equal(ctr[~none], w_ctr[~none])
            assert (ids[none] == 0xFFFFFFFF).all() and np.isinf(dist[none]).all()
    finally:
        ix.close()


def _random_case(n, dim, B, kl, kr, metric, seed, n_cap=None, nq=300, domain=None):
    cfg = W.Config(f"t{seed}", n, dim, 8, 0.4, domain or n, B, kl, kr, nq, (0.2,), metric=metric,
                   normalise=(metric == W.IP), seed=seed)
    X, a, q = W.base_vectors(cfg), W.attributes(cfg), W.query_vectors(cfg)
    ora = O.Index(X, a, B, n_cap=n_cap, metric=metric)
    la, ra = HG.build_graph(X, ora.bucket_of_ids(), B, kl, kr, metric=metric)
    ora.load_graph(la, ra)
    return dict(cfg=cfg, X=X, attrs=a, queries=q, local=la, remote=ra, oracle=ora)


@pytest.mark.parametrize("dim,metric,n,B,kl,kr,n_cap", [
    (32, W.L2SQ, 3001, 7, 12, 3, None),        # ragged sizes, one 128-byte line per row
    (64, W.L2SQ, 2500, 5, 16, 4, 3100),        # slack between slabs
    (96, W.IP, 4000, 9, 24, 8, None),          # inner product on unit vectors, 3 lines per row
    (256, W.L2SQ, 1500, 4, 20, 2, None),       # 8 lines per row (still register-resident query)
    (960, W.L2SQ, 1200, 3, 48, 8, None),       # 30 lines per row, query staged in LDS
    (128, W.L2SQ, 2000, 4, 61, 3, None),       # degree 64
    (160, W.L2SQ, 2000, 4, 16, 4, None),       # 5 lines per row
    (192, W.IP, 2000, 4, 16, 4, 2400),         # 6 lines per row
    (384, W.L2SQ, 1500, 3, 20, 4, None),       # 12 lines per row: query staged in LDS, two batches of pieces
    (640, W.L2SQ, 1500, 3, 20, 4, None),       # 20 lines per row
])
def test_other_shapes_match_oracle(torch_dev, dim, metric, n, B, kl, kr, n_cap):
    c = _random_case(n, dim, B, kl, kr, metric, seed=dim + n, n_cap=n_cap)
    ix = _gpu_index(c, torch_dev, n_cap)
    ora = c["oracle"]
    table, id2slot, slot2id = ix.get_layout()
    assert np.array_equal(table, ora.table) and np.array_equal(slot2id, ora.slot2id)
    rng = np.random.default_rng(dim)
    nq = len(c["queries"])
    width = rng.integers(1, n, nq)
    lo = rng.integers(-10, n, nq).astype(np.int32)
    hi = (lo + width).astype(np.int32)
    for beam, w, S in [(64, 1, 0), (33, 3, 200)]:
        if w * (kl + kr) > 512:
            continue
        ix.set_param("search_width", w); ix.set_param("n_seeds", S)
        ora.params.update(search_width=w, n_seeds=S or None)
        ids, dist, ctr = _search_gpu(ix, torch_dev, c["queries"], lo, hi, 10, beam)
        want_ids, want_dist, want_ctr = ora.search(c["queries"], lo, hi, 10, beam)
        assert np.array_equal(dist, want_dist), (beam, w, S)
        assert np.array_equal(ids, want_ids), (beam, w, S)
        assert np.array_equal(ctr, want_ctr), (beam, w, S)
    ix.close()


def test_edge_cases(c1_small, torch_dev):
    import torch
    c = c1_small
    ix = _gpu_index(c, torch_dev)
    ora = c["oracle"]
    q = c["queries"][:8]
    # empty, inverted and out-of-domain ranges; single-value range; whole domain
    lo = np.array([10, 20000, -5, 5000, 0, 9999, 777, -100], np.int32)
    hi = np.array([5, 30000, -1, 5000, 9999, 9999, 790, 100000], np.int32)
    ids, dist, ctr = _search_gpu(ix, torch_dev, q, lo, hi, 10, 64)
    want = ora.search(q, lo, hi, 10, 64)
    assert np.array_equal(ids, want[0]) and np.array_equal(dist, want[1]) and np.array_equal(ctr, want[2])
    assert (ids[:3] == 0xFFFFFFFF).all() and np.isinf(dist[:3]).all() and (ctr[:3, 7] == 3).all()
    # V <= S: the answer is the exhaustive filtered k-NN
    rng = np.random.default_rng(3)
    lo2 = rng.integers(0, 9900, 256).astype(np.int32)
    hi2 = (lo2 + rng.integers(0, 50, 256)).astype(np.int32)
    ids2, dist2, _ = _search_gpu(ix, torch_dev, c["queries"][:256], lo2, hi2, 10, 64)
    gt, _ = O.exact_filtered_knn(c["X"], c["attrs"], c["queries"][:256], lo2, hi2, 10)
    small = np.array([((c["attrs"] >= l) & (c["attrs"] <= h)).sum() <= 64 for l, h in zip(lo2, hi2)])
    assert small.sum() > 100 and np.array_equal(ids2[small], gt[small])
    # k == beam, k == 1, host (numpy) buffers in and out, a single query, no query
    for k, beam in [(16, 16), (1, 64), (64, 64)]:
        got_ids, got_dist = ix.search_range(q, lo, hi, k, beam)
        w_ids, w_dist, _ = ora.search(q, lo, hi, k, beam)
        assert np.array_equal(got_ids, w_ids) and np.array_equal(got_dist, w_dist)
    one_ids, one_dist = ix.search_range(q[4:5], lo[4:5], hi[4:5], 10, 64)
    assert np.array_equal(one_ids, want[0][4:5]) and np.array_equal(one_dist, want[1][4:5])
    none_ids, _ = ix.search_range(q[:0], lo[:0], hi[:0], 10, 64)
    assert none_ids.shape == (0, 10)
    # stopping rules: iteration cap and visited capacity
    for name, val, oname in [("max_iter", 3, "max_iter"), ("visited_cap", 150, "visited_cap")]:
        ix.set_param(name, val); ora.params[oname] = val
        g = _search_gpu(ix, torch_dev, c["queries"][:200], c["lo"][:200], c["hi"][:200], 10, 64)
        w = ora.search(c["queries"][:200], c["lo"][:200], c["hi"][:200], 10, 64)
        assert all(np.array_equal(x, y) for x, y in zip(g, w))
        ix.set_param("max_iter", 0); ix.set_param("visited_cap", 2800)
        ora.params.update(max_iter=None, visited_cap=2800)
    # argument errors are reported, not executed
    from paper_2604_16402_amd import binding as B
    for k, beam in [(0, 64), (65, 64), (10, 1000)]:
        with pytest.raises(B.GrabError) as e:
            ix.search_range(q, lo, hi, k, beam)
        assert e.value.status == B.EINVAL
    ix.set_param("n_seeds", 5000)
    with pytest.raises(B.GrabError) as e:
        ix.search_range(q, lo, hi, 10, 64)
    assert e.value.status == B.EINVAL
    ix.close()


def test_malformed_graph_is_rejected(c1_small, torch_dev):
    from paper_2604_16402_amd import binding as B
    c = c1_small
    ix = _gpu_index(c, torch_dev)
    ora = c["oracle"]
    bad = c["local"].copy()
    other = np.nonzero(ora.bucket_of_ids() != ora.bucket_of_ids()[0])[0][0]
    bad[0, 0] = other                                     # a local edge that leaves its bucket
    with pytest.raises(B.GrabError) as e:
        ix.load_graph(bad, c["remote"])
    assert e.value.status == B.EINVAL and ix.sizes()["has_graph"] == 0
    bad = c["remote"].copy()
    bad[5, 0] = 10_000_000                                 # id out of range
    with pytest.raises(B.GrabError) as e:
        ix.load_graph(c["local"], bad)
    assert e.value.status == B.EINVAL
    ix.load_graph(c["local"], c["remote"])                 # a good graph still loads afterwards
    assert ix.sizes()["has_graph"] == 1
    ix.close()


def test_hand_traced_example_on_gpu(torch_dev):
    import json, os
    g = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "trace_2d.json")))
    pts = np.zeros((8, 32), np.float32); pts[:, :2] = np.asarray(g["points"], np.float32)
    qv = np.zeros((1, 32), np.float32); qv[0, :2] = g["query"]
    from paper_2604_16402_amd import binding as B
    ix = B.Index(32)
    ix.build_buckets(pts, np.asarray(g["attrs"], np.int32), g["n_buckets"])
    ix.load_graph(np.asarray(g["local"], np.uint32), np.asarray(g["remote"], np.uint32))
    ix.set_param("n_seeds", g["n_seeds"])
    info, seeds = ix.select_range(np.array([g["lo"]], np.int32), np.array([g["hi"]], np.int32), g["beam"])
    e = g["expected_select"]
    assert info[0].tolist() == [e["b0"], e["b1"], e["V"], e["first_valid_slot"], e["end_valid_slot"], len(e["seeds"])]
    assert seeds[0].tolist() == e["seeds"]
    for case in g["cases"]:
        if case["max_iter"] == 0:
            continue                                       # 0 means "default" at the C boundary
        ix.set_param("max_iter", case["max_iter"]); ix.set_param("visited_cap", case["visited_cap"])
        ids, dist = ix.search_range(qv, np.array([g["lo"]], np.int32), np.array([g["hi"]], np.int32), g["k"], g["beam"])
        assert ids[0].tolist() == case["ids"] and dist[0].tolist() == case["dist"]
        ctr = ix.get_counters(1)[0]
        names = ["iters", "parents", "evals", "seed_evals", "rejects", "tail", "visited", "stop"]
        for name, want in case["counters"].items():
            assert ctr[names.index(name)] == want, (name, case)
    ix.close()


def test_search_twice_gives_identical_bytes(c1_small, torch_dev):
    c = c1_small
    ix = _gpu_index(c, torch_dev)
    a = _search_gpu(ix, torch_dev, c["queries"], c["lo"], c["hi"], 10, 64)
    b = _search_gpu(ix, torch_dev, c["queries"], c["lo"], c["hi"], 10, 64)
    assert all(np.array_equal(x, y) for x, y in zip(a, b))
    ix.close()


@pytest.mark.parametrize("dim,kl,kr,beam,width,seeds,vcap", [
    (128, 64, 64, 512, 4, 512, 6000),     # degree 128 and a 512-entry queue (the paper's scalability setting)
    (2048, 24, 8, 128, 4, 128, 2800),     # 2048-dimensional rows (64 lines per row)
    (128, 100, 28, 256, 1, 0, 2800),      # unbalanced degree split, queue of 256
])
def test_wide_parameter_surface(torch_dev, dim, kl, kr, beam, width, seeds, vcap):
    n, B = (3000, 4) if dim <= 128 else (1200, 3)
    cfg = W.Config("wide", n, dim, 8, 0.4, n, B, min(kl, 64), min(kr, 64), 200, (0.3,), seed=dim + kl)
    X, a, q = W.base_vectors(cfg), W.attributes(cfg), W.query_vectors(cfg)
    ora = O.Index(X, a, B)
    la, ra = HG.build_graph(X, ora.bucket_of_ids(), B, min(kl, 64), kr, pool=min(2 * kl, 200))
    if kl > 64:      # pad the local part with further in-bucket neighbours to reach the requested width
        la2, _ = HG.build_graph(X, ora.bucket_of_ids(), B, kl, 0, pool=kl + 20)
        la = la2
    ora.load_graph(la, ra)
    c = dict(cfg=cfg, X=X, attrs=a, local=la, remote=ra)
    ix = _gpu_index(c, torch_dev)
    for name, val in [("visited_cap", vcap), ("n_seeds", seeds), ("search_width", width)]:
        ix.set_param(name, val)
    ora.params.update(visited_cap=vcap, n_seeds=seeds or None, search_width=width)
    lo, hi = W.ranges(cfg, 0.3)
    ids, dist, ctr = _search_gpu(ix, torch_dev, q, lo, hi, 10, beam)
    w = ora.search(q, lo, hi, 10, beam)
    assert np.array_equal(dist, w[1]) and np.array_equal(ids, w[0]) and np.array_equal(ctr, w[2])
    ix.close()


def test_gather_probe_reports_rows_read(c1_small, torch_dev):
    from paper_2604_16402_amd import binding
    ix = _gpu_index(c1_small, torch_dev)
    ms, nbytes = ix.probe_gather(1024, 4)
    # 128-d rows: 4 rows per lane group in flight, 8 groups per wavefront
    assert nbytes == 1024 * 4 * 8 * 4 * 128 * 4
    assert ms > 0.0
    with pytest.raises(binding.GrabError):
        ix.probe_gather(0, 4)
    with pytest.raises(binding.GrabError):
        ix.probe_gather(16, 1 << 20)
    # a search after the probe still matches the oracle (the probe shares the timing events)
    q, lo, hi = c1_small["queries"][:50], c1_small["lo"][:50], c1_small["hi"][:50]
    ids, dist, _ = _search_gpu(ix, torch_dev, q, lo, hi, 10, 64)
    want_ids, want_dist, _ = c1_small["oracle"].search(q, lo, hi, 10, 64)
    assert np.array_equal(ids, want_ids) and np.array_equal(dist, want_dist)
    ix.close()


@pytest.mark.parametrize("nq", [2048, 2051, 4097])
def test_batches_that_run_in_bucket_order_match_oracle(c1_small, torch_dev, nq):
    # from 2,048 queries on the library launches the queries grouped by first selected bucket; the
    # batch sizes leave zero, five and seven unused workgroups at the end of that order
    ix = _gpu_index(c1_small, torch_dev)
    rng = np.random.default_rng(nq)
    pick = rng.integers(0, len(c1_small["queries"]), nq)
    q = c1_small["queries"][pick]
    lo = rng.integers(-200, 10100, nq).astype(np.int32)
    hi = (lo + rng.integers(-3, 3000, nq)).astype(np.int32)          # some ranges are empty
    ids, dist, ctr = _search_gpu(ix, torch_dev, q, lo, hi, 10, 32)
    want_ids, want_dist, want_ctr = c1_small["oracle"].search(q, lo, hi, 10, 32, threads=O.max_threads())
    assert np.array_equal(ids, want_ids) and np.array_equal(dist, want_dist) and np.array_equal(ctr, want_ctr)
    ix.close()
