"""Parity at the benchmark's full size and launch configuration: 1M x 128, 64 buckets,
10,000 queries per selectivity, every query compared with the oracle (needs an MI355X)."""
import numpy as np
import pytest

from oracle import oracle as O
from paper_2604_16402_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def c2_full():
    import torch
    from paper_2604_16402_amd import binding, groundtruth as GT
    dev = torch.device("cuda:0")
    cfg = W.CONFIGS["c2"]
    X, a, q = W.base_vectors(cfg), W.attributes(cfg), W.query_vectors(cfg)
    ix = binding.Index(cfg.dim, cfg.metric, stream=torch.cuda.current_stream(dev).cuda_stream)
    Xd, ad = torch.from_numpy(X).to(dev), torch.from_numpy(a).to(dev)
    ix.build_buckets(Xd, ad, cfg.buckets)
    ora = O.Index(X, a, cfg.buckets)
    table, id2slot, slot2id = ix.get_layout()
    assert np.array_equal(table, ora.table) and np.array_equal(id2slot, ora.id2slot[:cfg.n])
    assert np.array_equal(slot2id, ora.slot2id)
    la, ra = W.build_graph(X, ora.bucket_of_ids(), cfg.buckets, cfg.k_local, cfg.k_remote, device="cuda:0", chunk=16384)
    ix.load_graph(torch.from_numpy(la.view(np.int32)).to(dev), torch.from_numpy(ra.view(np.int32)).to(dev))
    ora.load_graph(la, ra)
    return dict(cfg=cfg, X=X, attrs=a, q=q, ix=ix, ora=ora, dev=dev, Xd=Xd, ad=ad, GT=GT)


@pytest.mark.parametrize("sel,beam,seeds,width,vcap", [
    (0.1, 32, 512, 4, 1400),     # the launch configuration bench.py times
    (0.1, 64, 64, 1, 2800),      # library defaults
    (0.01, 64, 512, 1, 1400),
    (0.5, 128, 1024, 4, 4000),
])
def test_full_size_matches_oracle(c2_full, sel, beam, seeds, width, vcap):
    import torch
    c = c2_full
    cfg, ix, ora, dev = c["cfg"], c["ix"], c["ora"], c["dev"]
    lo, hi = W.ranges(cfg, sel)
    ix.set_param("visited_cap", vcap); ix.set_param("n_seeds", seeds); ix.set_param("search_width", width)
    ora.params.update(visited_cap=vcap, n_seeds=seeds, search_width=width)
    nq = len(c["q"])
    ids = torch.empty((nq, 10), dtype=torch.int32, device=dev)
    dist = torch.empty((nq, 10), dtype=torch.float32, device=dev)
    qd, lod, hid = torch.from_numpy(c["q"]).to(dev), torch.from_numpy(lo).to(dev), torch.from_numpy(hi).to(dev)
    ix.search_range(qd, lod, hid, 10, beam, ids, dist)
    torch.cuda.synchronize()
    want_ids, want_dist, want_ctr = ora.search(c["q"], lo, hi, 10, beam, threads=O.max_threads())
    got_ids = ids.cpu().numpy().view(np.uint32)
    assert np.array_equal(dist.cpu().numpy(), want_dist)
    assert np.array_equal(got_ids, want_ids)
    assert np.array_equal(ix.get_counters(nq), want_ctr)
    # definition-level properties on every row, and recall against exhaustive filtered k-NN
    a = c["attrs"]
    live = got_ids != 0xFFFFFFFF
    sel_a = a[np.where(live, got_ids, 0)]
    assert ((sel_a >= lo[:, None]) & (sel_a <= hi[:, None]) | ~live).all()
    assert (np.diff(want_dist, axis=1) >= 0).all()
    gt = c["GT"].exact_filtered_knn(c["Xd"], c["ad"], qd, lod, hid, 10)
    rec = c["GT"].recall(ids, gt)
    sample = np.arange(0, nq, 50)
    cpu_gt, _ = O.exact_filtered_knn(c["X"], a, c["q"][sample], lo[sample], hi[sample], 10)
    # the fp32 GPU ground truth agrees with the float64 exhaustive answer up to near-ties
    agree = np.mean([len(np.intersect1d(x, y)) / 10 for x, y in zip(gt.cpu().numpy()[sample], cpu_gt.astype(np.int64))])
    assert agree >= 0.998, agree
    if (sel, beam) == (0.1, 32):
        assert rec >= 0.95, rec
