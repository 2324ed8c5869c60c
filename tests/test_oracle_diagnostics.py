"""Pins for the oracle's consensus-distance diagnostic (the quantity of Eq. 2,
Eq. 5 and Fig. 2) and the weighted average (convex combinations of models)."""
import numpy as np
import pytest

import oracle


def _pop(N, P, seed=0, scale=0.02):
    return (np.random.default_rng(seed).standard_normal((N, P)) * scale).astype(np.float32)


def test_sqdist_matches_numpy_definition():
    for N, P in [(1, 10), (2, 1001), (5, 4099), (20, 777)]:
        pop = _pop(N, P, seed=N)
        x = pop.astype(np.float64)
        want = ((x - x.mean(axis=0)) ** 2).sum(axis=1)
        got = oracle.consensus_sqdist(pop)
        assert np.allclose(got, want, rtol=1e-12, atol=0)
    assert oracle.consensus_sqdist(_pop(1, 50))[0] == 0.0            # one model is its own consensus


def test_sqdist_closed_forms():
    a = np.array([[1.0, 2.0, 3.0], [3.0, 2.0, -1.0]], dtype=np.float32)
    # two models: each is at half the distance between them: ||a0 - a1||^2 / 4 = (4 + 0 + 16) / 4
    assert list(oracle.consensus_sqdist(a)) == [5.0, 5.0]
    same = np.repeat(_pop(1, 100), 4, axis=0)
    assert np.all(oracle.consensus_sqdist(same) == 0.0)              # identical rows: zero
    # slices add up, empty slice is zero
    pop = _pop(6, 1000, seed=9)
    whole = oracle.consensus_sqdist(pop)
    parts = oracle.consensus_sqdist(pop, 0, 250) + oracle.consensus_sqdist(pop, 250, 1000)
    assert np.allclose(whole, parts, rtol=1e-13)
    assert np.all(oracle.consensus_sqdist(pop, 400, 400) == 0.0)
    with pytest.raises(ValueError):
        oracle.consensus_sqdist(pop, 10, 5)
    with pytest.raises(ValueError):
        oracle.consensus_sqdist(pop, 0, 1001)


def test_eq2_ema_contracts_and_eq5_shuffle_preserves():
    pop = _pop(8, 30000, seed=2, scale=1.0)
    d0 = oracle.consensus_sqdist(pop)
    e = pop.copy()
    oracle.ema(e, 0.9)
    al = float(np.float32(0.9))
    assert np.allclose(oracle.consensus_sqdist(e), al * al * d0, rtol=1e-5)      # Eq. 2, row by row
    s = pop.copy()
    oracle.shuffle(s, None, [(0, 30000, 0.3)], 1, 0)
    d1 = oracle.consensus_sqdist(s)
    assert abs(d1.sum() - d0.sum()) <= 1e-12 * d0.sum()                          # Eq. 5: the total is kept
    assert not np.allclose(d1, d0, rtol=1e-6)                                    # the split over models is not


def test_weighted_average_pins():
    pop = _pop(5, 3001, seed=4, scale=1.0)
    w = np.array([0.1, 0.2, 0.3, 0.15, 0.25])
    got = oracle.weighted_average(pop, w)
    want = (w[:, None] * pop.astype(np.float64)).sum(axis=0).astype(np.float32)
    assert np.allclose(got, want, rtol=0, atol=1e-12) and np.mean(got == want) > 0.999
    for n in range(5):                                                           # one-hot weights copy a row
        assert np.array_equal(oracle.weighted_average(pop, np.eye(5)[n]), pop[n])
    avg = oracle.average(pop)
    uni = oracle.weighted_average(pop, np.full(5, 0.2))
    assert np.allclose(uni, avg, rtol=2e-7, atol=1e-12)                          # 0.2 is not exactly 1/5
    pw2 = _pop(4, 500, seed=5)
    assert np.array_equal(oracle.weighted_average(pw2, np.full(4, 0.25)), oracle.average(pw2))   # 1/4 is exact
    # the path between two models is a straight line: midpoint of endpoints
    a = oracle.weighted_average(pop[:2].copy(), [0.5, 0.5])
    assert np.allclose(a, 0.5 * (pop[0].astype(np.float64) + pop[1]), atol=1e-12)
    with pytest.raises(ValueError):
        oracle.weighted_average(pop, [0.2] * 4)
    with pytest.raises(ValueError):
        oracle.weighted_average(pop, [0.2, 0.2, float("nan"), 0.2, 0.2])
