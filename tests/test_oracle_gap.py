"""Pins for the oracle's second mask stream ("gap": geometric gap sampling).
The law it must realise is the one of Eq. 3: every coordinate selected
independently with probability p, permutation as in stream v1."""
import math
import struct

import numpy as np
import pytest

import oracle
from oracle import philox_bigint as pb
from workloads import distinct_population

PIECE = 1024


def _bits(a):
    return a.view(np.uint32)


# ---- second implementation, pure Python (Python floats are IEEE doubles) ------------------------

def _py_log2(x):
    bits = struct.unpack("<Q", struct.pack("<d", x))[0]
    e = ((bits >> 52) & 0x7FF) - 1023
    m = struct.unpack("<d", struct.pack("<Q", (bits & 0xFFFFFFFFFFFFF) | 0x3FF0000000000000))[0]
    if m > 1.4142135623730951:
        m, e = m * 0.5, e + 1
    s = (m - 1.0) / (m + 1.0)
    z = s * s
    poly = 1.0 / 21.0
    for k in (19, 17, 15, 13, 11, 9, 7, 5, 3, 1):
        poly = poly * z + 1.0 / k
    t = s * poly
    return float(e) + (t + t) * 1.4426950408889634


def _py_gap(U, inv):
    q = (_py_log2(float(U + 1)) - 53.0) * inv
    if not q < 2047.0:
        q = 2047.0
    if q < 0.0:
        q = 0.0
    return 1 + int(math.floor(q))


def _py_uniform(seed, step, s, d):
    out = pb.philox4x32_10((s & 0xFFFFFFFF, s >> 32, step, 0x80000000 + (d >> 1)), (seed & 0xFFFFFFFF, seed >> 32))
    return ((out[2 * (d & 1)] << 32) | out[2 * (d & 1) + 1]) >> 11


def _py_mask(P, segs, seed, step):
    merged = []
    for off, ln, p in segs:
        if ln == 0:
            continue
        if merged and merged[-1][1] == off and merged[-1][2] == p:
            merged[-1][1] = off + ln
        else:
            merged.append([off, off + ln, p])
    sel = []
    for a, b, p in merged:
        if p == 0.0 or 1.0 - p == 1.0:
            continue
        inv = 0.0 if p >= 1.0 else 1.0 / _py_log2(1.0 - p)
        s = a
        while s < b:
            e = min((s // PIECE + 1) * PIECE, b)
            pos, d = s - 1, 0
            while True:
                pos += _py_gap(_py_uniform(seed, step, s, d), inv)
                if pos >= e:
                    break
                sel.append(pos)
                d += 1
            s = e
    return sel


# ---- the pieces -----------------------------------------------------------------------------

def test_log2_accuracy_and_python_twin():
    rng = np.random.default_rng(0)
    xs = list(np.exp(rng.uniform(-40, 40, 4000))) + [float(u) for u in rng.integers(1, 2 ** 53, 4000)]
    xs += [1.0, 2.0, 0.5, 2.0 ** 53, 2.0 ** -40, 1.4142135623730951, 1.4142135623730954, 1 - 1e-9, 1 - 2.0 ** -53]
    for x in xs:
        v = oracle.log2(x)
        assert v == _py_log2(x)                                   # same IEEE sequence, same bits
        assert abs(v - math.log2(x)) <= 4e-16 * max(1.0, abs(math.log2(x)))
    for k in range(-60, 60):
        assert oracle.log2(2.0 ** k) == float(k)                   # exact at powers of two


def test_gap_scale_and_gap_function():
    assert oracle.gap_scale(1.0) == 0.0
    assert oracle.gap_scale(0.5) == -1.0
    for p in (1e-4, 1e-3, 0.05, 0.9):
        assert abs(oracle.gap_scale(p) - 1.0 / math.log2(1.0 - p)) < 1e-12 * abs(oracle.gap_scale(p))
    # p = 1/2: gap = 1 + floor(-log2 u): u in (1/2, 1] -> 1, (1/4, 1/2] -> 2, ...
    assert oracle.gap(2 ** 53 - 1, -1.0) == 1
    assert oracle.gap(2 ** 52 + 2 ** 12, -1.0) == 1    # u just above 1/2 (beyond the rounding of log2 near 52)
    assert oracle.gap(2 ** 52 - 1, -1.0) == 2      # u = 1/2
    assert oracle.gap(2 ** 51 - 1, -1.0) == 3      # u = 1/4
    assert oracle.gap(0, -1.0) == 54               # u = 2^-53
    assert oracle.gap(12345, 0.0) == 1             # p = 1
    assert oracle.gap(0, oracle.gap_scale(1e-6)) == 2048    # capped
    rng = np.random.default_rng(1)
    for U in rng.integers(0, 2 ** 53, 3000):
        for p in (0.3, 0.01, 1e-4):
            inv = oracle.gap_scale(p)
            assert oracle.gap(int(U), inv) == _py_gap(int(U), inv)


@pytest.mark.parametrize("p", [0.3, 0.05, 0.002])
def test_gap_is_geometric(p):
    # regular grid over the 53-bit uniform: the histogram of the gap must be p (1-p)^(k-1)
    n = 1 << 18
    inv = oracle.gap_scale(p)
    gaps = np.array([oracle.gap(int(((2 * i + 1) << 53) // (2 * n)), inv) for i in range(n)])
    kmax = min(int(gaps.max()), 2047)
    hist = np.bincount(gaps, minlength=kmax + 1)[1:kmax + 1] / n
    k = np.arange(1, kmax + 1)
    want = p * (1 - p) ** (k - 1)
    assert np.abs(hist - want).max() < 2.0 / n + 1e-9
    if (1 - p) ** 2047 < 1e-12:                     # the cap at 2048 does not bite
        assert abs(gaps.mean() - 1 / p) < 0.01 / p
    else:                                           # P(gap > 2047) = (1-p)^2047
        assert abs(np.mean(gaps == 2048) - (1 - p) ** 2047) < 2.0 / n


def test_uniform_addressing():
    for seed, step, s, d in [(0, 0, 0, 0), (5, 7, 1024 * 999, 3), (1 << 40, 4294967295, (1 << 33) + 5, 1000)]:
        assert oracle.gap_uniform(seed, step, s, d) == _py_uniform(seed, step, s, d)
    # draws 0 and 1 share one Philox call, draw 2 needs the next counter
    a = pb.philox4x32_10((77, 0, 3, 0x80000000), (9, 0))
    b = pb.philox4x32_10((77, 0, 3, 0x80000001), (9, 0))
    assert oracle.gap_uniform(9, 3, 77, 0) == ((a[0] << 32) | a[1]) >> 11
    assert oracle.gap_uniform(9, 3, 77, 1) == ((a[2] << 32) | a[3]) >> 11
    assert oracle.gap_uniform(9, 3, 77, 2) == ((b[0] << 32) | b[1]) >> 11


def test_mask_matches_python_twin():
    P = 7000
    segs = [(0, 100, 0.5), (100, 900, 0.5), (1000, 0, 0.9), (1000, 24, 0.5), (1030, 3000, 0.02),
            (4030, 66, 1.0), (4096, 1000, 0.0), (5096, 1900, 0.3)]
    for seed, step in [(0, 0), (123456789012345, 77)]:
        mask = oracle.gap_mask(P, segs, seed, step)
        assert list(np.flatnonzero(mask)) == _py_mask(P, segs, seed, step)
        assert mask[4030:4096].all() and not mask[4096:5096].any() and not mask[1024:1030].any()


# ---- the law of the mask ----------------------------------------------------------------------

@pytest.mark.parametrize("p", [1e-4, 1e-3, 0.005, 0.05, 0.3, 0.9])
def test_mask_is_iid_bernoulli(p):
    P = 1 << 24
    m = oracle.gap_mask(P, [(0, P, p)], seed=11, step=int(p * 1e6)).astype(np.int64)
    n1 = int(m.sum())
    assert abs(n1 - p * P) < 5 * math.sqrt(P * p * (1 - p))
    # every position inside a piece is selected with probability p (no edge effect at restarts)
    by_pos = m.reshape(-1, PIECE).sum(axis=0)
    npieces = P // PIECE
    sig = math.sqrt(npieces * p * (1 - p))
    assert np.abs(by_pos - npieces * p).max() < 5.5 * sig
    assert abs(by_pos[0] - npieces * p) < 5 * sig and abs(by_pos[-1] - npieces * p) < 5 * sig
    # neighbours are independent, inside a piece and across a restart
    for lag in (1, 2, 7):
        both = int((m[:-lag] * m[lag:]).sum())
        exp = (P - lag) * p * p
        assert abs(both - exp) < 5.5 * math.sqrt(exp * (1 + 2 * p)) + 5
    across = int((m[PIECE - 1:-1:PIECE] * m[PIECE::PIECE]).sum())
    exp = (npieces - 1) * p * p
    assert abs(across - exp) < 5.5 * math.sqrt(exp) + 5
    # counts in blocks of 32 follow Binomial(32, p)
    blocks = m.reshape(-1, 32).sum(axis=1)
    hist = np.bincount(blocks, minlength=33).astype(float)
    pmf = np.array([math.comb(32, k) * p ** k * (1 - p) ** (32 - k) for k in range(33)]) * len(blocks)
    keep = pmf > 10
    chi2 = (((hist - pmf) ** 2 / np.maximum(pmf, 1e-300))[keep]).sum() + (hist[~keep].sum() - pmf[~keep].sum()) ** 2 / max(pmf[~keep].sum(), 1.0)
    assert chi2 < 30 + 4 * keep.sum()


def test_bit_patterns_of_8_neighbours():
    p, P = 0.3, 1 << 23
    m = oracle.gap_mask(P, [(0, P, p)], seed=3, step=0)
    codes = np.packbits(m.reshape(-1, 8), axis=1, bitorder="little").ravel()
    hist = np.bincount(codes, minlength=256).astype(float)
    ones = np.array([bin(c).count("1") for c in range(256)])
    exp = (p ** ones) * ((1 - p) ** (8 - ones)) * len(codes)
    chi2 = ((hist - exp) ** 2 / exp).sum()
    assert chi2 < 340                              # 0.999 quantile of chi-square with 255 df is 330.5


# ---- the whole shuffle ------------------------------------------------------------------------

def test_shuffle_follows_the_mask_and_the_same_permutations():
    N, P = 5, 9000
    segs = [(0, 5000, 0.2), (5000, 3990, 0.05)]
    mask = oracle.gap_mask(P, segs, 21, 6)
    pop = np.repeat(np.arange(N, dtype=np.float32)[:, None], P, axis=1).copy()
    cnt = oracle.shuffle(pop, None, segs, 21, 6, stream="gap")
    assert cnt == int(mask.sum()) and not mask[8990:].any()
    for g in range(P):
        want = list(oracle.permutation(21, 6, g, N)) if mask[g] else list(range(N))
        assert list(pop[:, g].astype(int)) == want


def test_p1_equals_stream_v1_and_p0_is_identity():
    pop = distinct_population(6, 5000)
    a, b = pop.copy(), pop.copy()
    assert oracle.shuffle(a, None, [(0, 5000, 1.0)], 4, 2, stream="gap") == 5000
    assert oracle.shuffle(b, None, [(0, 5000, 1.0)], 4, 2, stream="v1") == 5000
    assert np.array_equal(_bits(a), _bits(b))
    c = pop.copy()
    assert oracle.shuffle(c, None, [(0, 5000, 0.0)], 4, 2, stream="gap") == 0
    assert np.array_equal(_bits(c), _bits(pop))


def test_probabilities_below_double_resolution_select_nothing():
    """Bernoulli(p) of Eq. 3 for p so small that 1 - p rounds to 1: log2(1 - p) is 0 there and a naive
    inversion would select EVERY coordinate; the law asks for (almost surely) none."""
    P = 1 << 16
    pop = distinct_population(4, P)
    for p in (5e-324, 1e-300, 1e-17, 2.0 ** -54):
        assert 1.0 - p == 1.0
        for seed in (0, 7):
            assert not oracle.gap_mask(P, [(0, P, p)], seed, 3).any()
            a = pop.copy()
            assert oracle.shuffle(a, None, [(0, P, p)], seed, 3, stream="gap") == 0
            assert np.array_equal(_bits(a), _bits(pop))
    # the smallest probabilities that still have a logarithm: the walk runs, and selects with probability
    # about p per coordinate (P * p < 1e-11 here, so nothing is selected either)
    for p in (2.0 ** -53, 1.2e-16, 1e-15):
        assert 1.0 - p != 1.0 and math.isfinite(oracle.gap_scale(p))
        assert not oracle.gap_mask(P, [(0, P, p)], 1, 0).any()
    # a tiny-p segment between two ordinary ones leaves their streams alone (pieces restart at segment starts)
    segs = [(0, 3000, 0.05), (3000, 2000, 1e-300), (5000, 3000, 0.05)]
    m = oracle.gap_mask(8000, segs, 5, 1)
    assert not m[3000:5000].any() and m[:3000].any() and m[5000:].any()
    assert np.array_equal(m[:3000], oracle.gap_mask(8000, [(0, 3000, 0.05)], 5, 1)[:3000])
    assert np.array_equal(m[5000:], oracle.gap_mask(8000, [(5000, 3000, 0.05)], 5, 1)[5000:])
    # the distance is defined for any scale, also the degenerate ones (no undefined conversion)
    inf = float("inf")
    assert oracle.gap(12345, -inf) == 2048 and oracle.gap(2 ** 53 - 1, -inf) == 2048
    assert oracle.gap(12345, inf) == 1 and oracle.gap(12345, float("nan")) == 2048


def test_log2_against_libm_dense_sample():
    """The stream's log2 against the C library's on a dense sample, as a RELATIVE error (also just
    below 1, where the result is tiny and log2(1 - p) of a small p lives): a wrong series coefficient
    or constant cannot hide behind an absolute tolerance."""
    rng = np.random.default_rng(11)
    xs = np.concatenate([rng.uniform(0.5, 2.0, 20000),
                         1.0 - rng.uniform(0.5, 1.0, 20000) * 2.0 ** -rng.integers(1, 50, 20000).astype(np.float64),
                         rng.integers(1, 2 ** 53, 20000).astype(np.float64)])
    for x in xs:
        ref = math.log2(float(x))
        assert abs(oracle.log2(float(x)) - ref) <= 4.5e-16 * abs(ref), x


def test_invariants_momentum_threads_windows_segmentation():
    N, P = 7, 100_003
    rng = np.random.default_rng(5)
    pop = (rng.standard_normal((N, P)) * 0.02).astype(np.float32)
    one, mom = pop.copy(), pop.copy()
    c1 = oracle.shuffle(one, mom, [(0, P, 0.07)], 3, 9, stream="gap")
    assert c1 > 0 and np.array_equal(_bits(one), _bits(mom))                  # momentum travels with its weight
    assert np.array_equal(np.sort(_bits(one), axis=0), np.sort(_bits(pop), axis=0))   # Eq. 5: multiset kept
    cut = pop.copy()                                                           # touching segments of equal p merge
    c2 = oracle.shuffle(cut, None, [(0, 10, 0.07), (10, 4085, 0.07), (4095, 0, 0.5), (4095, 3, 0.07),
                                    (4098, P - 4098, 0.07)], 3, 9, stream="gap")
    mt = pop.copy()
    c3 = oracle.shuffle(mt, None, [(0, P, 0.07)], 3, 9, threads=5, stream="gap")
    assert c1 == c2 == c3
    assert np.array_equal(_bits(one), _bits(cut)) and np.array_equal(_bits(one), _bits(mt))
    g0, W = 4096, 20480
    win = np.ascontiguousarray(pop[:, g0:g0 + W])
    oracle.shuffle_window(win, None, P, g0, [(0, P, 0.07)], 3, 9, stream="gap")
    assert np.array_equal(_bits(win), _bits(one[:, g0:g0 + W]))
    with pytest.raises(ValueError):                                            # windows must sit on the piece grid
        oracle.shuffle_window(win, None, P, 4000, [(0, P, 0.07)], 3, 9, stream="gap")
    # a different step or seed gives an independent mask
    m0 = oracle.gap_mask(P, [(0, P, 0.07)], 3, 9)
    for seed, step in [(3, 10), (4, 9)]:
        m1 = oracle.gap_mask(P, [(0, P, 0.07)], seed, step)
        assert abs(np.mean(m0 != m1) - 2 * 0.07 * 0.93) < 0.01


def test_expectation_matches_eq4_gap_stream():
    N, P, p, R = 4, 64, 0.3, 6000
    rng = np.random.default_rng(1)
    pop = rng.standard_normal((N, P)).astype(np.float32)
    acc = np.zeros((N, P))
    for step in range(R):
        a = pop.copy()
        oracle.shuffle(a, None, [(0, P, p)], 2024, step, stream="gap")
        acc += a
    want = (1 - p) * pop + p * pop.mean(axis=0, keepdims=True)
    tol = 5.0 * np.abs(pop).max() * math.sqrt(p / R)
    assert np.abs(acc / R - want).max() < tol
