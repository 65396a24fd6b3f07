"""HIP path against the CPU oracle, element by element, through the C ABI (needs an MI355X)."""
import numpy as np
import pytest

from oracle import oracle as O
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
