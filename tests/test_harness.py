"""Host-side checks of the seeded workload generators and diagnostics (no GPU)."""
import numpy as np

from oracle import oracle as O
from harness import diagnostics
from paper_2604_16402_amd import workloads as W


def test_generators_are_seeded_and_shaped():
    cfg = W.scaled(W.CONFIGS["c2"], 5000, n_queries=100)
    a, b = W.base_vectors(cfg), W.base_vectors(cfg)
    assert a.dtype == np.float32 and a.shape == (5000, 128) and np.array_equal(a, b)
    assert not np.array_equal(W.query_vectors(cfg), a[:100])
    attrs = W.attributes(cfg)
    assert attrs.dtype == np.int32 and attrs.min() >= 0 and attrs.max() < cfg.domain
    lo, hi = W.ranges(cfg, 0.1)
    assert ((hi - lo + 1) == cfg.domain // 10).all() and lo.min() >= 0 and hi.max() < cfg.domain
    c5 = W.scaled(W.CONFIGS["c5"], 5000, append_batch=50)
    assert W.append_vectors(c5, 0).shape == (50, 128) and not np.array_equal(W.append_vectors(c5, 0), W.append_vectors(c5, 1))
    c4 = W.scaled(W.CONFIGS["c4"], 20000, n_queries=200, buckets=8)
    x = W.base_vectors(c4)
    assert np.allclose(np.linalg.norm(x, axis=1), 1.0, atol=1e-5)
    z = W.attributes(c4)
    assert (z == 0).mean() > 0.05 and np.median(z) < c4.domain / 100       # heavy head, long tail
    lo, hi = W.ranges(c4, None)
    w = hi - lo + 1
    assert w.min() >= 1 and w.max() <= c4.domain and np.median(w) < c4.domain / 10
    assert [W.CONFIGS[k].n for k in ("c1", "c2", "c3", "c4", "c5")] == [10_000, 1_000_000, 1_000_000, 10_000_000, 1_000_000]


def test_strong_components_of_built_graphs():
    # Section 5.4: local edges alone leave one island per bucket; remote edges join them
    cfg = W.scaled(W.CONFIGS["c1"], 2400, buckets=6)
    X, a = W.base_vectors(cfg), W.attributes(cfg)
    ix = O.Index(X, a, cfg.buckets)
    occ = ix.slot2id != O.EMPTY
    ix.build_graph(12, 0, pool=24, threads=4)
    local_only = diagnostics.strong_components(ix.A, occ)
    ix.build_graph(12, 3, pool=24, threads=4)
    full = diagnostics.strong_components(ix.A, occ)
    assert local_only >= cfg.buckets and full < local_only and full <= 3
    ring = np.array([[1], [2], [0], [0xFFFFFFFF]], np.uint32)
    assert diagnostics.strong_components(ring, np.array([True, True, True, True])) == 2
    assert diagnostics.strong_components(ring, np.array([True, True, True, False])) == 1
    # nothing points to slot 3: one orphan while it is occupied
    assert diagnostics.orphans(ring, np.array([True, True, True, True])) == 1
    assert diagnostics.orphans(ring, np.array([True, True, True, False])) == 0
    assert diagnostics.in_degrees(ring, np.array([True, True, True, True])).tolist()[3] == 0
