"""Do the pins bite?  Each case plants one plausible mistake in a COPY of the oracle's C source
(a swapped constant, a wrong index, a dropped term, a transposed operand), builds it with gcc and
runs a condensed set of the pins against it: at least one must fail.  The unmodified source must
pass the same set.  Everything here runs on the CPU."""
import itertools
import math
import os
import subprocess

import numpy as np
import pytest

import oracle
from oracle import philox_bigint as pb
from test_oracle_gap import _py_mask

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(os.path.dirname(HERE), "oracle", "wash_ref.c")


# ---- the condensed pins (each raises AssertionError on a wrong oracle) -------------------------

def _pin_philox():
    assert oracle.philox([0] * 4, [0] * 2) == (0x6627E8D5, 0xE169C58D, 0xBC57AC4C, 0x9B00DBD8)
    assert oracle.philox([0x243F6A88, 0x85A308D3, 0x13198A2E, 0x03707344], [0xA4093822, 0x299F31D0]) == \
        (0xD16CFE09, 0x94FDCCEB, 0x5001E420, 0x24126EA1)


def _pin_stream_addressing():
    for seed, step, g in [(1, 2, 3), (0xDEADBEEFCAFEF00D, 77, (1 << 34) + 6)]:
        assert oracle.mask_word(seed, step, g) == pb.mask_word(seed, step, g)
        for N in (2, 5, 9, 20):
            assert list(oracle.permutation(seed, step, g, N)) == pb.permutation(seed, step, g, N)


def _pin_threshold():
    assert [oracle.threshold(p) for p in (0.0, 1.0, 0.5, 1e-4, 1e-3)] == [0, 1 << 32, 1 << 31, 429497, 4294967]


def _pin_fisher_yates():
    def word(j, m):
        return -((-j << 32) // m)
    for N in (3, 4, 5):
        seen = set()
        for js in itertools.product(*[range(i + 1) for i in range(N - 1, 0, -1)]):
            words = [word(j, i + 1) for j, i in zip(js, range(N - 1, 0, -1))]
            seen.add(tuple(int(v) for v in oracle.fisher_yates(words, N)))
        assert len(seen) == math.factorial(N)
    assert list(oracle.fisher_yates([word(0, 4), word(2, 3), word(0, 2)], 4)) == [1, 3, 2, 0]


def _pin_shuffle_semantics():
    N, P = 5, 3000
    pop = np.repeat(np.arange(N, dtype=np.float32)[:, None], P, axis=1).copy()
    mom = pop * 10
    segs = [(0, P, 0.25)]
    cnt = oracle.shuffle(pop, mom, segs, 77, 5)
    T = oracle.threshold(0.25)
    nsel = 0
    for g in range(P):
        sel = pb.mask_word(77, 5, g) < T
        nsel += sel
        want = pb.permutation(77, 5, g, N) if sel else list(range(N))
        assert list(pop[:, g].astype(int)) == want              # gather: row n receives row pi(n)
        assert list((mom[:, g] / 10).astype(int)) == want       # momentum travels with its weight
    assert cnt == nsel
    assert abs(cnt - 0.25 * P) < 5 * math.sqrt(P * 0.25 * 0.75)


def _pin_uniform_and_eq4():
    N, P = 3, 300_000
    pop = np.repeat(np.arange(N, dtype=np.float32)[:, None], P, axis=1).copy()
    oracle.shuffle(pop, None, [(0, P, 1.0)], 3, 0)
    code = (pop[0] * 9 + pop[1] * 3 + pop[2]).astype(np.int64)
    counts = np.bincount(code, minlength=27)
    valid = [a * 9 + b * 3 + c for a, b, c in itertools.permutations(range(3))]
    assert counts.sum() == counts[valid].sum()
    chi2 = (((counts[valid] - P / 6) ** 2) / (P / 6)).sum()
    assert chi2 < 20.52
    N, P, p, R = 4, 32, 0.3, 3000
    x = np.random.default_rng(1).standard_normal((N, P)).astype(np.float32)
    acc = np.zeros((N, P))
    for step in range(R):
        a = x.copy()
        oracle.shuffle(a, None, [(0, P, p)], 5, step)
        acc += a
    want = (1 - p) * x + p * x.mean(axis=0, keepdims=True)
    assert np.abs(acc / R - want).max() < 5.0 * np.abs(x).max() * math.sqrt(p / R)


def _pin_average_ema_eq6():
    pop = (np.random.default_rng(2).standard_normal((5, 2000))).astype(np.float32)
    x = pop.astype(np.float64)
    assert np.allclose(oracle.average(pop), x.mean(axis=0), rtol=0, atol=1e-6)
    assert np.array_equal(oracle.average(pop[:1].copy()), pop[0])
    e = pop.copy()
    oracle.ema(e, 0.75)
    assert np.allclose(e, 0.75 * x + 0.25 * x.mean(axis=0, keepdims=True), rtol=0, atol=1e-6)
    two = np.array([[0.0], [10.0]], dtype=np.float32)
    oracle.ema(two, 0.5)
    assert list(two[:, 0]) == [2.5, 7.5]
    pl = oracle.layer_probs(0.05, 11, 0)
    assert pl[0] == 0.05 and pl[-1] == 0.0 and abs(pl.mean() - 0.025) < 1e-15
    d = oracle.consensus_sqdist(pop)
    assert np.allclose(d, ((x - x.mean(axis=0)) ** 2).sum(axis=1), rtol=1e-12)
    w = np.array([0.1, 0.2, 0.3, 0.15, 0.25])
    assert np.allclose(oracle.weighted_average(pop, w), (w[:, None] * x).sum(axis=0), rtol=0, atol=1e-6)


def _pin_gap_stream():
    for x in (3.0, 0.75, 1e-3, 12345.678, 2.0 ** 52 + 12345, 1.9999, 7.99, 1.42, 0.70710678):
        assert abs(oracle.log2(x) - math.log2(x)) <= 4e-16 * max(1.0, abs(math.log2(x)))
    assert oracle.gap(2 ** 52 - 1, -1.0) == 2 and oracle.gap(2 ** 53 - 1, -1.0) == 1 and oracle.gap(7, 0.0) == 1
    a = pb.philox4x32_10((77, 0, 3, 0x80000000), (9, 0))
    assert oracle.gap_uniform(9, 3, 77, 1) == ((a[2] << 32) | a[3]) >> 11
    p, n = 0.05, 1 << 15
    inv = oracle.gap_scale(p)
    gaps = np.array([oracle.gap(int(((2 * i + 1) << 53) // (2 * n)), inv) for i in range(n)])
    hist = np.bincount(gaps, minlength=60)[1:60] / n
    assert np.abs(hist - p * (1 - p) ** np.arange(59)).max() < 3.0 / n
    P = 1 << 20
    m = oracle.gap_mask(P, [(0, 1000, 0.05), (1000, P - 1000, 0.05)], 11, 4).astype(np.int64)
    assert abs(m.sum() - 0.05 * P) < 5 * math.sqrt(P * 0.05 * 0.95)
    by_pos = m.reshape(-1, 1024).sum(axis=0)
    assert np.abs(by_pos - 1024 * 0.05).max() < 5.5 * math.sqrt(1024 * 0.05 * 0.95)
    both = int((m[:-1] * m[1:]).sum())
    assert abs(both - P * 0.0025) < 6 * math.sqrt(P * 0.0025)
    one = oracle.gap_mask(P, [(0, P, 0.05)], 11, 4)
    assert np.array_equal(one, m.astype(np.uint8))               # touching equal-p segments merge
    segs = [(0, 100, 0.5), (100, 900, 0.5), (1000, 24, 0.5), (1030, 3000, 0.02), (4030, 66, 1.0), (5096, 1900, 0.3)]
    assert list(np.flatnonzero(oracle.gap_mask(7000, segs, 5, 9))) == _py_mask(7000, segs, 5, 9)   # Python twin
    assert not oracle.gap_mask(4096, [(0, 4096, 1e-17)], 3, 1).any()    # 1 - p rounds to 1: Bernoulli(p) selects nothing
    a1 = np.repeat(np.arange(4, dtype=np.float32)[:, None], 2000, axis=1).copy()
    b1 = a1.copy()
    oracle.shuffle(a1, None, [(0, 2000, 1.0)], 4, 2, stream="gap")
    oracle.shuffle(b1, None, [(0, 2000, 1.0)], 4, 2, stream="v1")
    assert np.array_equal(a1, b1)


PINS = [_pin_philox, _pin_stream_addressing, _pin_threshold, _pin_fisher_yates, _pin_shuffle_semantics,
        _pin_uniform_and_eq4, _pin_average_ema_eq6, _pin_gap_stream]


def _first_failure():
    for pin in PINS:
        try:
            pin()
        except (AssertionError, ValueError) as exc:
            return pin.__name__, exc
    return None


# ---- planted mistakes: (name, text to find, replacement) ---------------------------------------

MUTATIONS = [
    ("philox multipliers swapped", "(uint64_t)0xD2511F53u * (uint64_t)c0", "(uint64_t)0xCD9E8D57u * (uint64_t)c0"),
    ("philox weyl constant off by one", "k1 += 0xBB67AE85u;", "k1 += 0xBB67AE86u;"),
    ("philox nine rounds", "round < 10; ++round", "round < 9; ++round"),
    ("philox wrong high half", "uint32_t n0 = hi1 ^ c1 ^ k0;", "uint32_t n0 = hi0 ^ c1 ^ k0;"),
    ("philox key not mixed in", "uint32_t n2 = hi0 ^ c3 ^ k1;", "uint32_t n2 = hi0 ^ c3;"),
    ("mask word index shifted", "return out[g & 3u];", "return out[(g + 1u) & 3u];"),
    ("mask quad not shared by 4 coordinates", "uint64_t quad = g >> 2;", "uint64_t quad = g;"),
    ("perm words collide with mask counter", "(uint32_t)step, 1u + (t >> 2) };", "(uint32_t)step, (t >> 2) };"),
    ("perm words ignore the step", "{ (uint32_t)g, (uint32_t)(g >> 32), (uint32_t)step, 1u + (t >> 2) }",
     "{ (uint32_t)g, (uint32_t)(g >> 32), 0u, 1u + (t >> 2) }"),
    ("fisher-yates ascending", "uint32_t i = N - 1u - t;", "uint32_t i = t + 1u;"),
    ("fisher-yates without fixed points (j < i)", "(uint64_t)w[t] * (uint64_t)(i + 1u)) >> 32", "(uint64_t)w[t] * (uint64_t)i) >> 32"),
    ("threshold truncated instead of rounded", "floor(p * 4294967296.0 + 0.5)", "floor(p * 4294967296.0)"),
    ("scatter instead of gather", "vals[(uint64_t)n * row_stride + col] = old[perm[n]];",
     "vals[(uint64_t)perm[n] * row_stride + col] = old[n];"),
    ("momentum not permuted", "moms[(uint64_t)n * row_stride + col] = old[perm[n]];", "moms[(uint64_t)n * row_stride + col] = old[n];"),
    ("bernoulli inverted", "if (!((uint64_t)u < T)) continue;", "if ((uint64_t)u < T) continue;"),
    ("average divides by N-1", "out[g] = (float)(sum / (double)N);", "out[g] = (float)(sum / (double)(N - 1u + (N == 1u)));"),
    ("ema weights swapped", "(float)(a * x + (1.0 - a) * mean)", "(float)((1.0 - a) * x + a * mean)"),
    ("ema mean drifts with the update", "double x = (double)params[(uint64_t)n * P + g];\n            params[(uint64_t)n * P + g] = (float)(a * x + (1.0 - a) * mean);",
     "double x = (double)params[(uint64_t)n * P + g];\n            params[(uint64_t)n * P + g] = (float)(a * x + (1.0 - a) * mean);\n            mean += ((double)params[(uint64_t)n * P + g] - x) / (double)N;"),
    ("eq.6 divides by L", "(double)l / (double)(L - 1u)", "(double)l / (double)L"),
    ("consensus distance without the mean", "double d = (double)params[(uint64_t)n * P + g] - mean;", "double d = (double)params[(uint64_t)n * P + g];"),
    ("weighted average ignores the weights", "sum += w[n] * (double)params[(uint64_t)n * P + g];", "sum += (double)params[(uint64_t)n * P + g] / (double)N;"),
    ("gap: series term dropped", "poly = poly * z + 1.0 / 3.0;", "poly = poly * z;"),
    ("gap: sqrt(2) reduction skipped", "if (m > 1.4142135623730951) { m = m * 0.5; e += 1; }", ""),
    ("gap: distance starts at 0", "return 1u + (uint32_t)floor(q);", "return (uint32_t)floor(q) + (q < 1.0 ? 1u : 0u);"),
    ("gap: 52-bit uniform", "return w >> 11;", "return w >> 12;"),
    ("gap: second draw reuses the first words", "out[2u * (d & 1u)] << 32) | (uint64_t)out[2u * (d & 1u) + 1u]", "out[0] << 32) | (uint64_t)out[1]"),
    ("gap: log of p instead of 1-p", "return 1.0 / wash_ref_log2(1.0 - p);", "return 1.0 / wash_ref_log2(p);"),
    ("gap: no restart at 1024", "uint64_t e = (s / WASH_REF_PIECE + 1u) * WASH_REF_PIECE;", "uint64_t e = (s / 4096u + 1u) * 4096u;"),
    ("gap: probabilities below double resolution select everything", "if (p == 0.0 || 1.0 - p == 1.0) continue;", "if (p == 0.0) continue;"),
    ("gap: touching equal-p segments not merged", "(segs[k].offset == b && segs[k].p == p)", "(0)"),
]


def _build(text, path):
    src = path + ".c"
    with open(src, "w") as f:
        f.write(text)
    subprocess.run(["gcc", "-std=c11", "-O1", "-ffp-contract=off", "-fPIC", "-shared", "-pthread", src, "-o", path, "-lm"],
                   check=True)


def test_unmodified_oracle_passes_the_condensed_pins(tmp_path):
    path = str(tmp_path / "libref_copy.so")
    _build(open(SRC).read(), path)
    try:
        oracle.use_library(path)
        assert _first_failure() is None
    finally:
        oracle.use_library(None)


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_noticed(tmp_path, name, old, new):
    text = open(SRC).read()
    assert text.count(old) >= 1, f"mutation '{name}' no longer applies to the source"
    path = str(tmp_path / "libref_mut.so")
    _build(text.replace(old, new), path)
    try:
        oracle.use_library(path)
        failure = _first_failure()
    finally:
        oracle.use_library(None)
    assert failure is not None, f"no pin noticed: {name}"
