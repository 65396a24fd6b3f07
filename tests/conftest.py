import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(scope="session")
def c1_small():
    """Config-1 shaped inputs (10k x 128, 16 buckets) with the harness graph, built once."""
    from harness import graphs as HG
    from paper_2604_16402_amd import workloads as W
    from oracle import oracle as O
    cfg = W.CONFIGS["c1"]
    X = W.base_vectors(cfg)
    a = W.attributes(cfg)
    q = W.query_vectors(cfg)
    lo, hi = W.ranges(cfg, 0.1)
    ix = O.Index(X, a, cfg.buckets)
    la, ra = HG.build_graph(X, ix.bucket_of_ids(), cfg.buckets, cfg.k_local, cfg.k_remote)
    ix.load_graph(la, ra)
    return dict(cfg=cfg, X=X, attrs=a, queries=q, lo=lo, hi=hi, local=la, remote=ra, oracle=ix)
