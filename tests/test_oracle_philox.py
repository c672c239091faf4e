"""Pins for the oracle's random stream (CPU only)."""
import math
import os

import numpy as np

import oracle
from oracle import philox_py

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def _kat():
    rows = []
    with open(GOLDEN) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            w = [int(t, 16) for t in line.split()]
            rows.append((w[0:4], w[4:6], w[6:10]))
    return rows


def test_known_answer_vectors_cpp_and_python():
    kat = _kat()
    assert len(kat) == 3
    for ctr, key, want in kat:
        assert [int(v) for v in oracle.philox4x32_10(ctr, key)] == want
        assert philox_py.philox4x32(ctr, key) == want


def test_cpp_matches_python_on_random_inputs():
    rng = np.random.default_rng(7)
    words = rng.integers(0, 2 ** 32, size=(20000, 6), dtype=np.uint64)
    for row in words:
        ctr, key = [int(v) for v in row[:4]], [int(v) for v in row[4:]]
        assert [int(v) for v in oracle.philox4x32_10(ctr, key)] == philox_py.philox4x32(ctr, key)


def test_element_keying_layout():
    # four consecutive indices and two consecutive drafts share a block; the upper and lower
    # half-words come from two blocks that differ in bit 31 of the second counter word
    seed, row = 0x0123456789ABCDEF, (5 << 32) | 77
    key = [seed & 0xFFFFFFFF, seed >> 32]
    for k in (0, 1, 2, 3, 7, 65534, 65535):
        for i in (0, 1, 2, 3, 4, 1023, 128255):
            hi = philox_py.philox4x32([row & 0xFFFFFFFF, i >> 2, row >> 32, k >> 1], key)[i & 3]
            lo = philox_py.philox4x32([row & 0xFFFFFFFF, i >> 2, row >> 32, (k >> 1) + 2 ** 31], key)[i & 3]
            if k % 2:
                hi, lo = hi >> 16, lo >> 16
            want = ((hi & 0xFFFF) << 16) | (lo & 0xFFFF)
            assert oracle.shared_word(seed, row, k, i) == want
            assert philox_py.shared_word(seed, row, k, i) == want


def test_words_of_distinct_elements_do_not_repeat():
    # every (k, i) gets its own 32 bits: neighbours in k and in i are distinct words
    seed, row = 99, 3
    words = {(k, i): oracle.shared_word(seed, row, k, i) for k in range(6) for i in range(64)}
    assert len(set(words.values())) == len(words)
    # and they do not depend on the neighbour: the same word from the Python generator
    assert all(philox_py.shared_word(seed, row, k, i) == w for (k, i), w in words.items())


def test_race_time_mapping():
    # S = -ln((x + 1/2) / 2^32): endpoints and a mid value, against mpmath-free closed forms
    assert oracle.race_time(0xFFFFFFFF) == -math.log1p(-(2.0 ** -33))
    assert abs(oracle.race_time(0) - 33 * math.log(2.0)) < 1e-14
    assert abs(oracle.race_time(0x7FFFFFFF) - (-math.log(0.5 - 2.0 ** -33))) < 1e-15
    for x in (1, 12345, 0x80000000, 0xFFFFFFFE):
        assert abs(oracle.race_time(x) - philox_py.race_time(x)) <= 1e-15 * philox_py.race_time(x) + 1e-300


def test_uniformity_of_stream():
    # chi-square of the top byte and of the byte that straddles the two half-words, over 2^16
    # words drawn the way the sampler draws them
    n = 1 << 16
    top = np.zeros(256, dtype=np.int64)
    mid = np.zeros(256, dtype=np.int64)
    for e in range(n):
        w = oracle.shared_word(42, 9, e & 3, e >> 2)
        top[w >> 24] += 1
        mid[(w >> 12) & 0xFF] += 1
    from scipy import stats
    for counts in (top, mid):
        expected = n / 256
        chi2 = float(((counts - expected) ** 2 / expected).sum())
        assert stats.chi2.sf(chi2, 255) > 1e-4
