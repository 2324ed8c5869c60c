"""Pins for the oracle's uniform average (Alg. 1 output), PAPA EMA (Eq. 1) and
the layer-wise probability schedule (Eq. 6)."""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle


def _pop(N, P, seed=0, scale=0.02):
    return (np.random.default_rng(seed).standard_normal((N, P)) * scale).astype(np.float32)


def test_average_reduces_to_library_mean():
    for N, P in [(1, 100), (4, 4097), (20, 1000), (32, 77)]:
        pop = _pop(N, P, seed=N)
        want = pop.mean(axis=0, dtype=np.float64).astype(np.float32)
        got = oracle.average(pop)
        # numpy may sum pairwise: identical up to the last fp64 bit before rounding to fp32
        assert np.allclose(got, want, rtol=0, atol=1e-12)
        assert np.mean(got == want) > 0.999


def test_average_exact_cases():
    pop = np.full((7, 50), 0.1, dtype=np.float32)
    assert np.array_equal(oracle.average(pop), pop[0])              # constant rows: exact
    one = _pop(1, 300)
    assert np.array_equal(oracle.average(one), one[0])              # N = 1: a copy
    pop = np.array([[1.0, 2.0, -4.0], [3.0, 2.0, 4.0]], dtype=np.float32)
    assert list(oracle.average(pop)) == [2.0, 2.0, 0.0]
    # exact rational check against rounding once from the true quotient
    pop = _pop(3, 200, seed=5, scale=1.0)
    got = oracle.average(pop)
    for g in range(200):
        q = sum(Fraction(float(pop[n, g])) for n in range(3)) / 3
        assert got[g] == np.float32(float(q))


def test_ema_definition_and_limits():
    pop = _pop(5, 3000, seed=3)
    for alpha in (0.99, 0.5, 0.123):
        a = pop.copy()
        oracle.ema(a, alpha)
        x = pop.astype(np.float64)
        al = float(np.float32(alpha))
        want = (al * x + (1.0 - al) * x.mean(axis=0, keepdims=True)).astype(np.float32)
        assert np.allclose(a, want, rtol=0, atol=1e-10)
    a = pop.copy()
    oracle.ema(a, 1.0)
    assert np.array_equal(a, pop)                                    # alpha = 1: identity
    a = pop.copy()
    oracle.ema(a, 0.0)
    avg = oracle.average(pop)
    assert all(np.array_equal(a[n], avg) for n in range(5))          # alpha = 0: every row = consensus


def test_ema_uses_pre_update_mean_in_every_row():
    pop = np.array([[0.0], [10.0]], dtype=np.float32)
    oracle.ema(pop, 0.5)
    assert list(pop[:, 0]) == [2.5, 7.5]       # mean 5 for both rows, not re-computed after row 0


def test_ema_contracts_consensus_distance_by_alpha_squared():
    # Eq. 2: sum_n ||theta~_n - mean||^2 = alpha^2 sum_n ||theta_n - mean||^2, mean unchanged.
    pop = _pop(10, 50000, seed=4, scale=1.0)
    alpha = 0.9
    a = pop.copy()
    oracle.ema(a, alpha)
    x, y = pop.astype(np.float64), a.astype(np.float64)
    d0 = ((x - x.mean(0)) ** 2).sum()
    d1 = ((y - y.mean(0)) ** 2).sum()
    al = float(np.float32(alpha))
    assert abs(d1 / d0 - al * al) < 1e-6
    assert np.abs(x.mean(0) - y.mean(0)).max() < 1e-7


def test_shuffle_matches_ema_in_expectation():
    # Text below Eq. 4: WASH equals the EMA in expectation when p = 1 - alpha.
    N, P, alpha, R = 3, 32, 0.75, 8000
    pop = _pop(N, P, seed=6, scale=1.0)
    acc = np.zeros((N, P))
    for step in range(R):
        a = pop.copy()
        oracle.shuffle(a, None, [(0, P, 1 - alpha)], 99, step)
        acc += a
    e = pop.copy()
    oracle.ema(e, alpha)
    tol = 5.0 * np.abs(pop).max() * np.sqrt((1 - alpha) / R)
    assert np.abs(acc / R - e).max() < tol


def test_layer_probs_eq6():
    p, L = 0.05, 11
    pl = oracle.layer_probs(p, L, 0)
    assert pl[0] == p and pl[-1] == 0.0
    assert np.allclose(pl, [p * (1 - l / (L - 1)) for l in range(L)], rtol=0, atol=1e-18)
    assert abs(pl.mean() - p / 2) < 1e-15                       # halves the volume
    assert np.allclose(oracle.layer_probs(p, L, 1), p)
    inc = oracle.layer_probs(p, L, 2)
    assert inc[0] == 0.0 and inc[-1] == p and np.allclose(inc, pl[::-1], atol=1e-15)
    assert list(oracle.layer_probs(0.3, 1, 0)) == [0.3]         # L = 1: the base probability
    for bad in ((-0.1, 3, 0), (1.1, 3, 0), (0.1, 0, 0), (0.1, 3, 3)):
        with pytest.raises(ValueError):
            oracle.layer_probs(*bad)


def test_table1_communication_ratios(golden_dir):
    # (mean of Eq. 6 probabilities) / (1/T) reproduces the ratios printed in Table 1
    with open(os.path.join(golden_dir, "table1_comm_volume.txt")) as f:
        rows = [l.split() for l in f if l.strip() and not l.startswith("#")]
    assert len(rows) == 5
    for name, p, T, variant, num, den in rows:
        p, T = float(p), int(T)
        mean_p = oracle.layer_probs(p, 1001, 0).mean() * (2 if variant == "wash_opt" else 1)
        ratio = mean_p / (1.0 / T)
        assert abs(ratio - int(num) / int(den)) < 1e-12, (name, variant)
