"""The entry point that allocates nothing, against the allocating one (needs an MI355X).

Two calls in a row on the same index, the second with a smaller batch: ids, distances and
per-query counters must be bit-identical to grab_search_range's on the same inputs (which the
other GPU tests compare with the CPU oracle element by element)."""
import numpy as np
import pytest

from paper_2604_16402_amd import workloads as W

pytestmark = pytest.mark.gpu


def test_noalloc_search_equals_search_on_two_calls_in_a_row():
    import torch
    from oracle import oracle as O
    from paper_2604_16402_amd import binding
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    dev = torch.device("cuda:0")
    cfg = W.scaled(W.CONFIGS["c1"], 6000, n_queries=3000, buckets=8)
    X, attrs = W.base_vectors(cfg), W.attributes(cfg)
    ora = O.Index(X, attrs, cfg.buckets)
    ix = binding.Index(cfg.dim, cfg.metric, stream=torch.cuda.current_stream(dev).cuda_stream)
    ix.build_buckets(torch.from_numpy(X).to(dev), torch.from_numpy(attrs).to(dev), cfg.buckets)
    ix.build_graph(cfg.k_local, cfg.k_remote, 0)
    ix.set_param("search_width", 2)
    ix.set_param("n_seeds", 96)

    def both(nq, sel, stream, beam):
        q = torch.from_numpy(W.query_vectors(cfg, nq, stream=stream)).to(dev)
        lo, hi = W.ranges(cfg, sel, nq, stream=300 + stream)
        lod, hid = torch.from_numpy(lo).to(dev), torch.from_numpy(hi).to(dev)
        out = []
        for call in (ix.search_range, ix.search_range_noalloc):
            ids = torch.full((nq, cfg.k), -7, dtype=torch.int32, device=dev)
            dist = torch.full((nq, cfg.k), -7.0, dtype=torch.float32, device=dev)
            call(q, lod, hid, cfg.k, beam, ids, dist)
            torch.cuda.synchronize()
            out.append((ids.cpu().numpy().view(np.uint32), dist.cpu().numpy(), ix.get_counters(nq)))
        return out

    # first call: a batch large enough to take the bucket-ordered launch (2,048 queries and more)
    (ids_a, dist_a, ctr_a), (ids_n, dist_n, ctr_n) = both(3000, 0.1, 100, 64)
    assert np.array_equal(ids_n, ids_a) and np.array_equal(dist_n, dist_a) and np.array_equal(ctr_n, ctr_a)
    assert (ids_a != 0xFFFFFFFF).any()
    # second call: smaller batch, other ranges and queue size; the array still holds the first call's data
    (ids_a, dist_a, ctr_a), (ids_n, dist_n, ctr_n) = both(700, 0.3, 101, 40)
    assert np.array_equal(ids_n, ids_a) and np.array_equal(dist_n, dist_a) and np.array_equal(ctr_n, ctr_a)

    # limits and pointer kinds are refused before anything is launched
    q = torch.zeros((4, cfg.dim), dtype=torch.float32, device=dev)
    lo = torch.zeros(4, dtype=torch.int32, device=dev)
    ids = torch.zeros((4, cfg.k), dtype=torch.int32, device=dev)
    dist = torch.zeros((4, cfg.k), dtype=torch.float32, device=dev)
    with pytest.raises(binding.GrabError) as e:
        ix.search_range_noalloc(np.zeros((4, cfg.dim), np.float32), lo, lo, cfg.k, 64, ids, dist)
    assert e.value.status == binding.EINVAL and "device pointers" in str(e.value)
    big = 16385
    qb = torch.zeros((big, cfg.dim), dtype=torch.float32, device=dev)
    lob = torch.zeros(big, dtype=torch.int32, device=dev)
    idb = torch.zeros((big, cfg.k), dtype=torch.int32, device=dev)
    dib = torch.zeros((big, cfg.k), dtype=torch.float32, device=dev)
    with pytest.raises(binding.GrabError) as e:
        ix.search_range_noalloc(qb, lob, lob, cfg.k, 64, idb, dib)
    assert e.value.status == binding.EINVAL
    ix.close()
