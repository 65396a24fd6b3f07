"""Float attributes through the C ABI against the oracle on its float order keys (needs an MI355X)."""
import numpy as np
import pytest

from oracle import oracle as O
from harness import graphs as HG
from paper_2604_16402_amd import workloads as W

pytestmark = pytest.mark.gpu


def _same_index(ix, ora):
    table, id2slot, slot2id = ix.get_layout()
    assert np.array_equal(table, ora.table)
    assert np.array_equal(id2slot, ora.id2slot[:ora.n]) and np.array_equal(slot2id, ora.slot2id)
    x, a = ix.get_rows()
    live = ora.slot2id != O.EMPTY
    assert np.array_equal(x[live], ora.X[live]) and np.array_equal(a[live], ora.attr[live])
    assert np.array_equal(ix.get_graph(), ora.A)


def test_float_attributes_match_oracle_through_build_search_and_append():
    import torch
    from paper_2604_16402_amd import binding as B
    n, dim, nb, kl, kr, n_cap = 6000, 128, 8, 16, 4, 9000
    cfg = W.Config("f1", n, dim, 16, 0.3, n, nb, kl, kr, 400, (0.1,), seed=77, append_rounds=2, append_batch=700)
    X = W.base_vectors(cfg)
    rng = np.random.default_rng(77)
    a = rng.random(n).astype(np.float32)                      # uniform in [0,1) as in Section 5.1
    a[:6] = [0.0, -0.0, 0.5, 0.5, 1.0, -0.25]
    ora = O.Index(X, O.float_order_key(a), nb, n_cap=n_cap)
    la, ra = HG.build_graph(X, ora.bucket_of_ids(), nb, kl, kr)
    ora.load_graph(la, ra)
    dev = torch.device("cuda:0")
    ix = B.Index(dim)
    # device inputs for the build, host inputs for the rest: both kinds of pointer are exercised
    ix.build_buckets_f32(torch.from_numpy(X).to(dev), torch.from_numpy(a).to(dev), nb, n_cap)
    ix.load_graph(la, ra)
    _same_index(ix, ora)
    # the stored images are the oracle's keys and turn back into the floats
    _, got_a = ix.get_rows()
    slot_of = ix.get_layout()[1]
    assert all(B.attr_value(int(got_a[slot_of[i]])) == a[i] for i in range(0, n, 97))

    q = W.query_vectors(cfg)
    lo = (rng.random(len(q)) * 0.9).astype(np.float32)
    hi = (lo + rng.random(len(q)).astype(np.float32) * 0.3).astype(np.float32)
    lo[:8] = [-np.inf, 0.0, -0.0, 0.5, np.nan, 0.2, 2.0, -1.0]
    hi[:8] = [np.inf, 0.0, 0.0, 0.5, 0.7, np.nan, 3.0, -0.2]

    def compare():
        ids, dist = ix.search_range_f32(q, lo, hi, 10, 64)
        ctr = ix.get_counters(len(q))
        klo, khi = O.float_range_keys(lo, hi)
        w_ids, w_dist, w_ctr = ora.search(q, klo, khi, 10, 64, threads=O.max_threads())
        assert np.array_equal(dist, w_dist) and np.array_equal(ids, w_ids) and np.array_equal(ctr, w_ctr)
        return ids

    ids = compare()
    # definition-level check with float comparisons on the caller's own values
    live = ids != 0xFFFFFFFF
    all_a = a
    with np.errstate(invalid="ignore"):
        ok = (all_a[np.where(live, ids, 0)] >= lo[:, None]) & (all_a[np.where(live, ids, 0)] <= hi[:, None])
    assert (ok | ~live).all()
    assert not live[4].any() and not live[5].any() and not live[6].any()     # NaN bounds, range above every value
    assert set(ids[1][live[1]]) == {0, 1} and set(ids[3][live[3]]) == {2, 3}  # [0,0] holds both zeros; [0.5,0.5]
    assert set(ids[7][live[7]]) == {5}                                       # the one negative attribute

    # appends with float attributes, then searches over the grown index
    all_a = a
    for r in range(2):
        nx = W.append_vectors(cfg, r)
        na = rng.random(len(nx)).astype(np.float32)
        if r == 1:
            na[:4] = [-3.0, 7.5, np.inf, -0.0]               # outside every bucket interval: edge buckets widen
        ix.append_batch_f32(nx, na)
        ora.append(nx, O.float_order_key(na), threads=O.max_threads())
        _same_index(ix, ora)
        all_a = np.concatenate([all_a, na])
    ids = compare()
    live = ids != 0xFFFFFFFF
    with np.errstate(invalid="ignore"):
        ok = (all_a[np.where(live, ids, 0)] >= lo[:, None]) & (all_a[np.where(live, ids, 0)] <= hi[:, None])
    assert (ok | ~live).all() and (ids[live] >= n).any()

    # a NaN attribute is refused and nothing changes
    bad = rng.random(10).astype(np.float32)
    bad[3] = np.nan
    with pytest.raises(B.GrabError):
        ix.append_batch_f32(W.append_vectors(cfg, 0)[:10], bad)
    _same_index(ix, ora)
    ix2 = B.Index(dim)
    with pytest.raises(B.GrabError):
        ix2.build_buckets_f32(X[:100], np.full(100, np.nan, np.float32), 2, 100)
    ix2.close()
    ix.close()
