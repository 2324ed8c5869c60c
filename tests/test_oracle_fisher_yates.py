"""Pins for the oracle's Fisher-Yates step and range reduction."""
import itertools
import math

import numpy as np

import oracle


def _word_for(j, m):
    """Smallest 32-bit word w with (w * m) >> 32 == j."""
    return -((-j << 32) // m)  # ceil(j * 2^32 / m)


def test_mulhi_buckets_closed_form():
    # #{w : (w*m)>>32 == j} = ceil(2^32 (j+1)/m) - ceil(2^32 j/m): sizes differ by at most 1,
    # so each index in [0, m) has probability 1/m up to 2^-32.
    for m in range(1, 33):
        edges = [_word_for(j, m) for j in range(m + 1)]
        assert edges[0] == 0 and edges[-1] == 1 << 32
        sizes = [edges[j + 1] - edges[j] for j in range(m)]
        assert max(sizes) - min(sizes) <= 1
        for j in range(m):
            for w in (edges[j], edges[j + 1] - 1):
                assert (w * m) >> 32 == j


def test_exhaustive_bijection():
    # Feeding every index tuple (j_{N-1}, ..., j_1), j_i in [0, i], yields each of the N!
    # permutations exactly once.
    for N in range(1, 8):
        seen = set()
        ranges = [range(i + 1) for i in range(N - 1, 0, -1)]
        for js in itertools.product(*ranges):
            words = [_word_for(j, i + 1) for j, i in zip(js, range(N - 1, 0, -1))]
            perm = tuple(int(v) for v in oracle.fisher_yates(words, N))
            assert sorted(perm) == list(range(N))
            seen.add(perm)
        assert len(seen) == math.factorial(N)


def test_descending_order_and_swap_semantics():
    # N = 4, words choosing j_3 = 0, j_2 = 2, j_1 = 0:
    # [0,1,2,3] -swap(3,0)-> [3,1,2,0] -swap(2,2)-> same -swap(1,0)-> [1,3,2,0]
    words = [_word_for(0, 4), _word_for(2, 3), _word_for(0, 2)]
    assert list(oracle.fisher_yates(words, 4)) == [1, 3, 2, 0]
    # all-zero words: every step swaps slot i with slot 0 -> a left rotation
    assert list(oracle.fisher_yates([0] * 4, 5)) == [1, 2, 3, 4, 0]
    # maximal words pick j = i: identity
    assert list(oracle.fisher_yates([0xFFFFFFFF] * 7, 8)) == list(range(8))
    assert list(oracle.fisher_yates([], 1)) == [0]
