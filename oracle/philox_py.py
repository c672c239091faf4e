"""Philox4x32-10 in unbounded Python integers (test infrastructure).

Written from the published description of the generator (Salmon, Moraes, Dror,
Shaw, "Parallel random numbers: as easy as 1, 2, 3", SC'11): a 4-word counter, a
2-word key, ten rounds; each round multiplies counter words 0 and 2 by fixed
odd constants, keeps the low halves and folds the high halves into the other
two words together with the round key; the key advances by a Weyl constant
between rounds.  Used to cross-check the C++ oracle's generator and to
brute-force tiny cases of Algorithm 1 without touching the C++ code.
"""
import math

MASK = 0xFFFFFFFF
MUL_A = 0xD2511F53
MUL_B = 0xCD9E8D57
WEYL_A = 0x9E3779B9
WEYL_B = 0xBB67AE85


def philox4x32(ctr, key, rounds=10):
    c0, c1, c2, c3 = (int(v) & MASK for v in ctr)
    k0, k1 = (int(v) & MASK for v in key)
    for r in range(rounds):
        pa = MUL_A * c0
        pb = MUL_B * c2
        c0, c1, c2, c3 = ((pb >> 32) ^ c1 ^ k0) & MASK, pb & MASK, ((pa >> 32) ^ c3 ^ k1) & MASK, pa & MASK
        k0 = (k0 + WEYL_A) & MASK
        k1 = (k1 + WEYL_B) & MASK
    return [c0, c1, c2, c3]


def shared_word(seed, row, k, i):
    """The 32-bit word of element (row, draft k, index i).

    Its upper 16 bits come from the block with counter (lo32(row), i >> 2, hi32(row), k >> 1),
    its lower 16 bits from the block whose fourth counter word also has bit 31 set; both read output word
    i & 3, the lower half-word for even k and the upper one for odd k."""
    key = [seed & MASK, (seed >> 32) & MASK]
    row_words = [row & MASK, (row >> 32) & MASK]
    hi_block = philox4x32([row_words[0], i >> 2, row_words[1], k >> 1], key)
    lo_block = philox4x32([row_words[0], i >> 2, row_words[1], (k >> 1) | 0x80000000], key)
    shift = 16 if (k & 1) else 0
    return (((hi_block[i & 3] >> shift) & 0xFFFF) << 16) | ((lo_block[i & 3] >> shift) & 0xFFFF)


def aux_word(seed, row, i, which):
    """Auxiliary word of (row, i): output word i & 3 of the block with counter
    (lo32(row), i >> 2, hi32(row), 0x40000000 | which)."""
    key = [seed & MASK, (seed >> 32) & MASK]
    return philox4x32([row & MASK, i >> 2, (row >> 32) & MASK, 0x40000000 | which], key)[i & 3]


def uniform(x):
    """Open-interval uniform from a 32-bit word: the midpoint of its 2^-32 cell."""
    return (x + 0.5) / 4294967296.0


def race_time(x):
    """Exp(1) race time S = -ln U (Section 3)."""
    return -math.log(uniform(x))
