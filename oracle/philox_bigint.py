"""Second, independent Philox4x32-10 for cross-checking the C oracle.

TEST INFRASTRUCTURE.  Written from the published definition (Salmon, Moraes,
Dror, Shaw, SC'11) with Python's unbounded integers, sharing nothing with
wash_ref.c: the round is expressed on the full 64-bit products and the key
schedule as an explicit list, so a slip in either implementation (a swapped
multiplier, a wrong word order, a missing key bump) makes the two disagree.
"""

M_A = 0xD2511F53  # multiplies counter word 0
M_B = 0xCD9E8D57  # multiplies counter word 2
W_A = 0x9E3779B9  # Weyl increment of key word 0
W_B = 0xBB67AE85  # Weyl increment of key word 1
MASK = (1 << 32) - 1


def philox4x32_10(ctr, key):
    """ctr: 4 ints, key: 2 ints (each < 2**32) -> tuple of 4 ints."""
    x = [int(v) & MASK for v in ctr]
    keys = [((int(key[0]) + r * W_A) & MASK, (int(key[1]) + r * W_B) & MASK) for r in range(10)]
    for ka, kb in keys:
        pa = M_A * x[0]
        pb = M_B * x[2]
        x = [((pb >> 32) ^ x[1] ^ ka) & MASK, pb & MASK, ((pa >> 32) ^ x[3] ^ kb) & MASK, pa & MASK]
    return tuple(x)


def mask_word(seed, step, g):
    quad = g >> 2
    out = philox4x32_10((quad & MASK, quad >> 32, step & MASK, 0), (seed & MASK, (seed >> 32) & MASK))
    return out[g & 3]


def permutation(seed, step, g, N):
    """Stream v1 permutation of coordinate g, in pure Python."""
    key = (seed & MASK, (seed >> 32) & MASK)
    perm = list(range(N))
    for t in range(N - 1):
        out = philox4x32_10((g & MASK, g >> 32, step & MASK, 1 + t // 4), key)
        i = N - 1 - t
        j = (out[t % 4] * (i + 1)) >> 32
        perm[i], perm[j] = perm[j], perm[i]
    return perm
