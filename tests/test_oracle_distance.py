"""Pins for the oracle's fp32 distance (Algorithm 2, ComputeDistance; Table 2: Euclidean)."""
import numpy as np
import pytest

from oracle import oracle as O


@pytest.mark.parametrize("dim", [32, 96, 128, 960])
@pytest.mark.parametrize("metric", [O.L2SQ, O.IP])
def test_matches_float64_definition(dim, metric):
    rng = np.random.default_rng(7 + dim + metric)
    for _ in range(50):
        q = rng.standard_normal(dim).astype(np.float32)
        v = rng.standard_normal(dim).astype(np.float32)
        q64, v64 = q.astype(np.float64), v.astype(np.float64)
        want = ((q64 - v64) ** 2).sum() if metric == O.L2SQ else -(q64 * v64).sum()
        scale = (q64 ** 2).sum() + (v64 ** 2).sum() if metric == O.L2SQ else np.linalg.norm(q64) * np.linalg.norm(v64)
        assert abs(float(O.distance(q, v, metric)) - want) <= 1e-5 * scale


def test_exact_on_small_integers():
    # every product and partial sum is a small integer, so any summation order is exact:
    # a dropped element, a wrong index or a transposed operand changes the value
    rng = np.random.default_rng(3)
    for dim in (32, 128, 960):
        q = rng.integers(-8, 9, dim).astype(np.float32)
        v = rng.integers(-8, 9, dim).astype(np.float32)
        assert float(O.distance(q, v, O.L2SQ)) == float(((q - v) ** 2).sum(dtype=np.float64))
        assert float(O.distance(q, v, O.IP)) == -float((q * v).sum(dtype=np.float64))


def test_every_element_is_used_once():
    dim = 128
    q = np.zeros(dim, np.float32)
    for j in range(dim):
        v = np.zeros(dim, np.float32)
        v[j] = 3.0
        assert float(O.distance(q, v, O.L2SQ)) == 9.0
        w = np.zeros(dim, np.float32)
        w[j] = 2.0
        assert float(O.distance(w, v, O.IP)) == -6.0
        assert float(O.distance(w, np.roll(v, 1), O.IP)) == 0.0


def test_closed_forms():
    dim = 96
    e0 = np.zeros(dim, np.float32); e0[0] = 1
    e1 = np.zeros(dim, np.float32); e1[1] = 1
    z = np.zeros(dim, np.float32)
    assert float(O.distance(e0, e0, O.L2SQ)) == 0.0
    assert float(O.distance(e0, e1, O.L2SQ)) == 2.0
    assert float(O.distance(e0, z, O.L2SQ)) == 1.0
    assert float(O.distance(e0, e0, O.IP)) == -1.0
    assert float(O.distance(e0, e1, O.IP)) == 0.0
    assert float(O.distance(e0, -e0, O.IP)) == 1.0


def test_symmetry_and_polarisation():
    rng = np.random.default_rng(11)
    q = rng.standard_normal(128).astype(np.float32)
    v = rng.standard_normal(128).astype(np.float32)
    assert O.distance(q, v, O.L2SQ) == O.distance(v, q, O.L2SQ)
    assert O.distance(q, v, O.IP) == O.distance(v, q, O.IP)
    z = np.zeros(128, np.float32)
    lhs = float(O.distance(q, v, O.L2SQ))
    rhs = float(O.distance(q, z, O.L2SQ)) + float(O.distance(v, z, O.L2SQ)) + 2 * float(O.distance(q, v, O.IP))
    assert abs(lhs - rhs) <= 1e-4 * lhs
