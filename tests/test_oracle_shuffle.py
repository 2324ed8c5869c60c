"""Pins for the oracle's shuffle step: what Sec. 3 of the paper and the
definition of the stream fix, checked without any GPU."""
import itertools
import math

import numpy as np
import pytest

import oracle
from oracle import philox_bigint as pb
from workloads import distinct_population

CHI2_999 = {1: 10.83, 5: 20.52, 23: 49.73, 119: 177.0}  # 0.999 quantiles (df = N! - 1)


def _bits(a):
    return a.view(np.uint32)


def _python_shuffle(pop, mom, segs, seed, step):
    """Brute-force second implementation on tiny inputs: pure Python, big-int
    Philox, Eq. 3 applied coordinate by coordinate."""
    N, P = pop.shape
    out, outm = pop.copy(), None if mom is None else mom.copy()
    count = 0
    for off, length, p in segs:
        T = int(math.floor(p * 2 ** 32 + 0.5))
        for g in range(off, off + length):
            if pb.mask_word(seed, step, g) < T:
                count += 1
                pi = pb.permutation(seed, step, g, N)
                for n in range(N):
                    out[n, g] = pop[pi[n], g]          # theta_hat_n = theta_{pi(n)}
                    if mom is not None:
                        outm[n, g] = mom[pi[n], g]
    return out, outm, count


@pytest.mark.parametrize("N,P,p", [(1, 50, 1.0), (2, 333, 0.5), (5, 401, 0.3), (20, 97, 1.0), (32, 64, 0.7)])
def test_brute_force_tiny(N, P, p):
    pop = distinct_population(N, P)
    mom = distinct_population(N, P, base=0x40000000)
    segs = [(0, P // 3, p), (P // 3, P - P // 3 - 5, p / 2)]     # last 5 coordinates uncovered
    ref, refm, cnt = _python_shuffle(pop, mom, segs, seed=11, step=3)
    a, m = pop.copy(), mom.copy()
    got = oracle.shuffle(a, m, segs, 11, 3)
    assert got == cnt
    assert np.array_equal(_bits(a), _bits(ref)) and np.array_equal(_bits(m), _bits(refm))
    assert np.array_equal(_bits(a[:, P - 5:]), _bits(pop[:, P - 5:]))


def test_p0_identity_and_p1_all_selected():
    pop = distinct_population(6, 5000)
    a = pop.copy()
    assert oracle.shuffle(a, None, [(0, 5000, 0.0)], 1, 1) == 0
    assert np.array_equal(_bits(a), _bits(pop))
    assert oracle.shuffle(a, None, [(0, 5000, 1.0)], 1, 1) == 5000
    assert oracle.shuffle(a, None, [], 1, 1) == 0


def test_multiset_mean_and_consensus_distance_preserved():
    # Eq. 5: each coordinate's N values are permuted as a whole, so the multiset per
    # coordinate, the mean and the consensus distance are unchanged.
    rng = np.random.default_rng(0)
    pop = (rng.standard_normal((7, 20000)) * 0.02).astype(np.float32)
    a = pop.copy()
    cnt = oracle.shuffle(a, None, [(0, 20000, 0.2)], 3, 0)
    assert cnt > 0 and not np.array_equal(a, pop)
    assert np.array_equal(np.sort(_bits(a), axis=0), np.sort(_bits(pop), axis=0))

    def dist(x):
        x = np.sort(x.astype(np.float64), axis=0)          # order-free summation per coordinate
        return ((x - x.mean(axis=0)) ** 2).sum(axis=0)

    assert np.array_equal(dist(a), dist(pop))
    assert np.array_equal(np.sort(a.astype(np.float64), axis=0).sum(axis=0),
                          np.sort(pop.astype(np.float64), axis=0).sum(axis=0))


def test_mask_shared_by_all_models_and_gather_convention():
    # A selected coordinate moves in every row at once (one Bernoulli per coordinate), and
    # row n receives the old value of row pi(n).
    N, P = 5, 3000
    pop = np.repeat(np.arange(N, dtype=np.float32)[:, None], P, axis=1).copy()
    a = pop.copy()
    segs = [(0, P, 0.25)]
    oracle.shuffle(a, None, segs, 77, 5)
    T = oracle.threshold(0.25)
    for g in range(P):
        sel = oracle.mask_word(77, 5, g) < T
        if sel:
            assert list(a[:, g].astype(int)) == list(oracle.permutation(77, 5, g, N))
        else:
            assert list(a[:, g].astype(int)) == list(range(N))


@pytest.mark.parametrize("N", [2, 3, 4, 5])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_uniform_over_all_permutations(N, seed):
    # p = 1: every coordinate is permuted; chi-square over the N! cells.
    P = 1_200_000
    pop = np.repeat(np.arange(N, dtype=np.float32)[:, None], P, axis=1).copy()
    assert oracle.shuffle(pop, None, [(0, P, 1.0)], seed, 0, threads=4) == P
    code = np.zeros(P, dtype=np.int64)
    for n in range(N):
        code = code * N + pop[n].astype(np.int64)
    cells = {}
    for perm in itertools.permutations(range(N)):
        c = 0
        for v in perm:
            c = c * N + v
        cells[c] = 0
    vals, counts = np.unique(code, return_counts=True)
    assert set(vals.tolist()) <= set(cells)         # only valid permutations occur
    for v, c in zip(vals.tolist(), counts.tolist()):
        cells[v] = c
    expected = P / math.factorial(N)
    chi2 = sum((c - expected) ** 2 / expected for c in cells.values())
    assert chi2 < CHI2_999[math.factorial(N) - 1]


def test_permutation_independent_of_mask():
    # Conditional on selection at p = 0.1 the permutation histogram is still uniform.
    N, P = 3, 3_000_000
    pop = np.repeat(np.arange(N, dtype=np.float32)[:, None], P, axis=1).copy()
    cnt = oracle.shuffle(pop, None, [(0, P, 0.1)], 9, 4, threads=4)
    T = oracle.threshold(0.1)
    code = (pop[0] * 9 + pop[1] * 3 + pop[2]).astype(np.int64)
    ident = 0 * 9 + 1 * 3 + 2
    # unselected coordinates show the identity; among selected ones the identity has prob 1/6
    counts = {c: int((code == c).sum()) for c in np.unique(code)}
    non_ident = sum(v for k, v in counts.items() if k != ident)
    # selected = non_ident + selected-with-identity; estimate uniformity on the 5 other cells
    exp = cnt / 6.0
    chi2 = sum((v - exp) ** 2 / exp for k, v in counts.items() if k != ident)
    chi2 += ((cnt - non_ident) - exp) ** 2 / exp
    assert len(counts) == 6 and chi2 < CHI2_999[5]
    assert abs(cnt - 0.1 * P) < 5 * math.sqrt(P * 0.1 * 0.9)
    assert T == 429496730


def test_position_marginals_N20():
    # P(pi(n) = m) = 1/N for every pair: fixed points allowed (not derangements).
    N, P = 20, 400_000
    pop = np.repeat(np.arange(N, dtype=np.float32)[:, None], P, axis=1).copy()
    oracle.shuffle(pop, None, [(0, P, 1.0)], 5, 1, threads=4)
    src = pop.astype(np.int64)
    table = np.zeros((N, N))
    for n in range(N):
        table[n] = np.bincount(src[n], minlength=N)
    exp = P / N
    sigma = math.sqrt(P * (1 / N) * (1 - 1 / N))
    assert np.abs(table - exp).max() < 5.5 * sigma
    assert abs(np.trace(table) / P - 1.0) < 0.02       # expected number of fixed points is 1


def test_expectation_matches_eq4():
    # Eq. 4: E[theta_hat_n] = (1 - p) theta_n + p * mean, Monte-Carlo over steps.
    N, P, p, R = 4, 64, 0.3, 6000
    rng = np.random.default_rng(1)
    pop = rng.standard_normal((N, P)).astype(np.float32)
    acc = np.zeros((N, P))
    for step in range(R):
        a = pop.copy()
        oracle.shuffle(a, None, [(0, P, p)], 2024, step)
        acc += a
    emp = acc / R
    want = (1 - p) * pop + p * pop.mean(axis=0, keepdims=True)
    # per-entry standard error <= max|theta| * sqrt(p/R)
    tol = 5.0 * np.abs(pop).max() * math.sqrt(p / R)
    assert np.abs(emp - want).max() < tol
    # the derangement reading would give (1-p) theta_n + p (N mean - theta_n)/(N-1): must be far
    wrong = (1 - p) * pop + p * (N * pop.mean(axis=0, keepdims=True) - pop) / (N - 1)
    assert np.abs(emp - wrong).max() > 2 * tol


def test_selected_fraction_binomial():
    for p, P in [(0.01, 1 << 20), (0.001, 4_000_000), (0.005, 2_000_000)]:
        pop = np.zeros((2, P), dtype=np.float32)
        cnt = oracle.shuffle(pop, None, [(0, P, p)], 0, 0, threads=4)
        assert abs(cnt - p * P) < 5 * math.sqrt(P * p * (1 - p))


def test_momentum_travels_with_its_weight():
    rng = np.random.default_rng(2)
    pop = rng.standard_normal((10, 30000)).astype(np.float32)
    mom = pop.copy()
    a = pop.copy()
    oracle.shuffle(a, mom, [(0, 30000, 0.05)], 8, 2)
    assert np.array_equal(_bits(a), _bits(mom))
    # and passing momentum does not change what happens to the parameters
    b = pop.copy()
    oracle.shuffle(b, None, [(0, 30000, 0.05)], 8, 2)
    assert np.array_equal(_bits(a), _bits(b))


def test_segmentation_window_and_threads_do_not_change_bits():
    N, P = 6, 100_003
    pop = distinct_population(N, P)
    one = pop.copy()
    c1 = oracle.shuffle(one, None, [(0, P, 0.07)], 3, 9)
    cut = pop.copy()
    c2 = oracle.shuffle(cut, None, [(0, 10, 0.07), (10, 4085, 0.07), (4095, 3, 0.07), (4098, P - 4098, 0.07)], 3, 9)
    mt = pop.copy()
    c3 = oracle.shuffle(mt, None, [(0, P, 0.07)], 3, 9, threads=5)
    assert c1 == c2 == c3
    assert np.array_equal(_bits(one), _bits(cut)) and np.array_equal(_bits(one), _bits(mt))
    # a window of columns shuffled on its own gives the same columns
    g0, W = 4090, 20000
    win = np.ascontiguousarray(pop[:, g0:g0 + W])
    oracle.shuffle_window(win, None, P, g0, [(0, P, 0.07)], 3, 9)
    assert np.array_equal(_bits(win), _bits(one[:, g0:g0 + W]))


def test_step_and_seed_address_the_stream():
    N, P, p = 3, 200_000, 0.05
    pop = distinct_population(N, P)
    outs = {}
    for seed, step in [(0, 0), (0, 1), (1, 0), (1 << 32, 0)]:
        a = pop.copy()
        oracle.shuffle(a, None, [(0, P, p)], seed, step)
        outs[(seed, step)] = a
    a = pop.copy()
    oracle.shuffle(a, None, [(0, P, p)], 0, 0)
    assert np.array_equal(_bits(a), _bits(outs[(0, 0)]))          # stateless: same call, same bits
    T = oracle.threshold(p)
    masks = {k: np.array([oracle.mask_word(k[0], k[1], g) < T for g in range(0, P, 7)]) for k in outs}
    keys = list(outs)
    for i in range(len(keys)):
        for j in range(i + 1, len(keys)):
            ham = np.mean(masks[keys[i]] != masks[keys[j]])
            assert abs(ham - 2 * p * (1 - p)) < 0.01              # independent masks


def test_special_values_move_bit_for_bit():
    N, P = 4, 1000
    bits = np.random.default_rng(3).integers(0, 2 ** 32, size=(N, P), dtype=np.uint64).astype(np.uint32)
    bits[0, :4] = [0x7FC00001, 0xFFC12345, 0x80000000, 0x7F800000]   # NaN payloads, -0.0, inf
    pop = bits.view(np.float32).copy()
    a = pop.copy()
    oracle.shuffle(a, None, [(0, P, 1.0)], 0, 0)
    assert np.array_equal(np.sort(_bits(a), axis=0), np.sort(_bits(pop), axis=0))


def test_invalid_arguments_are_rejected():
    pop = np.zeros((2, 10), dtype=np.float32)
    for segs in ([(0, 11, 0.1)], [(5, 6, 0.1)], [(0, 5, 1.5)], [(0, 5, -0.1)], [(0, 5, float("nan"))],
                 [(4, 3, 0.1), (0, 2, 0.1)], [(0, 5, 0.1), (4, 2, 0.1)]):
        with pytest.raises(ValueError):
            oracle.shuffle(pop, None, segs, 0, 0)
    with pytest.raises(ValueError):
        oracle.shuffle(pop, None, [(0, 5, 0.1)], 0, 1 << 32)
    with pytest.raises(ValueError):
        oracle.shuffle(np.zeros((33, 4), dtype=np.float32), None, [(0, 4, 0.1)], 0, 0)
