"""Pins for the oracle's Philox4x32-10 and the stream built on it."""
import os
import random

import numpy as np

import oracle
from oracle import philox_bigint as pb


def _kat_lines(golden_dir):
    with open(os.path.join(golden_dir, "philox4x32_10_kat.txt")) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                v = [int(x, 16) for x in line.split()]
                yield v[0:4], v[4:6], tuple(v[6:10])


def test_known_answers_c(golden_dir):
    n = 0
    for ctr, key, out in _kat_lines(golden_dir):
        assert oracle.philox(ctr, key) == out
        n += 1
    assert n == 3


def test_known_answers_bigint(golden_dir):
    for ctr, key, out in _kat_lines(golden_dir):
        assert pb.philox4x32_10(ctr, key) == out


def test_two_implementations_agree():
    rnd = random.Random(20240517)
    for _ in range(20000):
        ctr = [rnd.getrandbits(32) for _ in range(4)]
        key = [rnd.getrandbits(32) for _ in range(2)]
        assert oracle.philox(ctr, key) == pb.philox4x32_10(ctr, key)


def test_bijective_on_a_small_cube():
    # For a fixed key Philox is a permutation of the counter space: distinct
    # counters must give distinct 128-bit outputs.
    seen = set()
    for a in range(16):
        for b in range(16):
            for c in range(16):
                seen.add(oracle.philox([a, b, c, 0], [7, 9]))
                seen.add(oracle.philox([a, b, c, 1], [7, 9]))
    assert len(seen) == 2 * 16 ** 3


def test_mask_word_addressing():
    # word (g mod 4) of the call at counter (g/4, step, 0); 64-bit g and seed split low/high
    for seed, step, g in [(0, 0, 0), (1, 2, 3), (0xDEADBEEFCAFEF00D, 4294967295, (1 << 34) + 5),
                          (12345, 99, 11173961)]:
        q = g >> 2
        ref = pb.philox4x32_10((q & 0xFFFFFFFF, q >> 32, step, 0), (seed & 0xFFFFFFFF, seed >> 32))[g & 3]
        assert oracle.mask_word(seed, step, g) == ref == pb.mask_word(seed, step, g)


def test_perm_words_addressing_and_separation():
    seed, step, g, N = 42, 7, 1000003, 20
    w = oracle.perm_words(seed, step, g, N)
    assert len(w) == N - 1
    for t in range(N - 1):
        ref = pb.philox4x32_10((g, 0, step, 1 + t // 4), (seed, 0))[t % 4]
        assert int(w[t]) == ref
    # the mask call (last counter word 0) never coincides with a perm call (>= 1)
    assert pb.philox4x32_10((g, 0, step, 0), (seed, 0)) != pb.philox4x32_10((g, 0, step, 1), (seed, 0))


def test_permutation_matches_bigint():
    rnd = random.Random(5)
    for _ in range(300):
        N = rnd.randint(1, 32)
        seed, step, g = rnd.getrandbits(64), rnd.getrandbits(32), rnd.getrandbits(40)
        assert list(oracle.permutation(seed, step, g, N)) == pb.permutation(seed, step, g, N)


def test_threshold_values():
    assert oracle.threshold(0.0) == 0
    assert oracle.threshold(1.0) == 1 << 32
    assert oracle.threshold(0.5) == 1 << 31
    assert oracle.threshold(1e-4) == 429497          # 429496.7296 rounds up
    assert oracle.threshold(0.001) == 4294967        # 4294967.296 rounds down
    assert oracle.threshold(2.0 ** -33) == 1         # exactly half: floor(x + 0.5)
    for p in np.linspace(0, 1, 1001):
        assert abs(oracle.threshold(p) - p * 2 ** 32) <= 0.5
