"""Float attributes in the oracle: the order key against float comparison itself, and the search
on float keys against exhaustive filtering done with float comparisons (no GPU)."""
import numpy as np
import pytest

from oracle import oracle as O


def _specials():
    tiny = np.float32(1e-45)          # smallest subnormal
    return np.array([0.0, -0.0, tiny, -tiny, 1.17549435e-38, -1.17549435e-38, 1.0, -1.0, 0.5, 0.49999997,
                     np.nextafter(np.float32(1), np.float32(2)), 3.4028235e38, -3.4028235e38, np.inf, -np.inf,
                     1e-3, -1e-3, 255.5, -255.5], dtype=np.float32)


def test_key_orders_like_float_comparison():
    rng = np.random.default_rng(7)
    v = np.concatenate([_specials(), rng.standard_normal(300).astype(np.float32),
                        (rng.random(200) * 1e-40).astype(np.float32), rng.integers(-2**31, 2**31, 400).astype(np.int32).view(np.float32)])
    v = v[~np.isnan(v)]
    k = O.float_order_key(v).astype(np.int64)
    lt = v[:, None] < v[None, :]
    eq = v[:, None] == v[None, :]
    assert np.array_equal(lt, k[:, None] < k[None, :])
    assert np.array_equal(eq, k[:, None] == k[None, :])
    assert O.float_order_key(np.float32(-0.0)) == O.float_order_key(np.float32(0.0)) == 0
    with pytest.raises(ValueError):
        O.float_order_key(np.array([0.5, np.nan], np.float32))


def test_range_keys_select_what_float_comparison_selects():
    rng = np.random.default_rng(8)
    a = np.concatenate([_specials(), rng.random(500).astype(np.float32) * 2 - 1])
    lo = np.concatenate([rng.random(60).astype(np.float32) * 2 - 1, [-np.inf, 0.0, -0.0, np.nan, 0.3, np.inf]]).astype(np.float32)
    hi = np.concatenate([lo[:60] + rng.random(60).astype(np.float32) * 0.5 - 0.05, [np.inf, 0.0, 0.0, 0.7, np.nan, -np.inf]]).astype(np.float32)
    klo, khi = O.float_range_keys(lo, hi)
    ka = O.float_order_key(a)
    with np.errstate(invalid="ignore"):
        want = (a[None, :] >= lo[:, None]) & (a[None, :] <= hi[:, None])
    got = (ka[None, :] >= klo[:, None]) & (ka[None, :] <= khi[:, None])
    assert np.array_equal(want, got)
    assert not got[63].any() and not got[64].any()      # NaN bounds select nothing


def test_search_on_float_attributes_equals_exhaustive_float_filtering():
    rng = np.random.default_rng(9)
    n, d, B = 900, 32, 6
    X = rng.standard_normal((n, d)).astype(np.float32)
    a = rng.random(n).astype(np.float32)                 # uniform in [0,1) as in Section 5.1
    a[:5] = [0.0, -0.0, 0.25, 0.25, 1.0]
    ix = O.Index(X, O.float_order_key(a), B)
    ix.build_graph(8, 2, threads=2)
    q = rng.standard_normal((40, d)).astype(np.float32)
    lo = (rng.random(40) * 0.8).astype(np.float32)
    hi = (lo + 0.06).astype(np.float32)
    lo[0], hi[0] = -0.0, 0.0
    lo[1], hi[1] = 0.25, 0.25
    klo, khi = O.float_range_keys(lo, hi)
    # every object of the range is a seed, so the search is exhaustive over the range
    ix.params.update(n_seeds=256, visited_cap=2800)
    ids, dist, _ = ix.search(q, klo, khi, 10, 64)
    for i in range(len(q)):
        sel = np.flatnonzero((a >= lo[i]) & (a <= hi[i]))
        assert len(sel) <= 256
        dd = ((X[sel].astype(np.float64) - q[i].astype(np.float64)) ** 2).sum(1)
        order = sel[np.lexsort((sel, dd))][:10]
        got = ids[i][ids[i] != O.EMPTY]
        assert len(got) == min(10, len(sel))
        # same set up to ties at the cut (fp32 vs float64 distances)
        if len(sel) > 10:
            cut = np.sort(dd)[9]
            must = sel[dd < cut * (1 - 1e-5)]
            may = sel[dd <= cut * (1 + 1e-5)]
            assert set(must) <= set(got) <= set(may)
        else:
            assert set(got) == set(order)
    assert set(ids[0][ids[0] != O.EMPTY]) == {0, 1} and set(ids[1][ids[1] != O.EMPTY]) == {2, 3}
