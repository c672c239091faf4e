"""Pins for the oracle's second way of drawing Algorithm 1's race times (CPU only).

Step 1 of Algorithm 1 asks for K N independent uniforms, i.e. independent Exp(1) race times; the
"min-first" construction draws the K times of one index through their minimum (Exp(K), at a
uniformly random draft, the others exceeding it by independent Exp(1) amounts).  What fixes it: the
K times must again be independent Exp(1) variables (marginals, joint law of pairs, law of the
minimum and of its position); everything the paper proves about the sampler then holds unchanged
(Proposition 1's marginals, its extension to distinct proposals, Theorem 1's bound); for K = 1 it is
the two-party Gumbel-max coupling on the index's first auxiliary word; a pure-Python transcription
agrees on tiny inputs; the target's sample still ignores the drafts.
"""
import numpy as np
import pytest
from scipy import stats

import oracle
from oracle import gls_py, lml, philox_py


def _dirichlet(rng, V, alpha=1.0):
    return rng.dirichlet(np.full(V, alpha))


def _bcast(vec, B):
    return np.broadcast_to(np.asarray(vec, np.float32), (B, len(vec)))


def test_auxiliary_words_follow_the_documented_counter_layout():
    seed = 0x0123456789ABCDEF
    for row, i in ((0, 0), (5, 3), ((1 << 40) + 9, 1234567), (2**64 - 1, 2**31 + 5)):
        for which in (0, 1):
            block = philox_py.philox4x32([row & 0xFFFFFFFF, i >> 2, row >> 32, 0x40000000 | which],
                                         [seed & 0xFFFFFFFF, seed >> 32])
            assert oracle.aux_word(seed, row, i, which) == block[i & 3] == philox_py.aux_word(seed, row, i, which)
    # never a per-draft block: those have bit 30 of the fourth counter word clear for every k < 2^31
    assert oracle.aux_word(seed, 7, 8, 0) != oracle.shared_word(seed, 7, 0, 8)


@pytest.mark.parametrize("K", [2, 3, 8])
def test_the_k_race_times_of_an_index_are_independent_exponentials(K):
    n = 200_000
    S = oracle.race_times(1234 + K, 1 << 20, n, 77, K, min_first=True)
    assert S.shape == (n, K) and (S > 0).all()
    U = np.exp(-S)
    for k in range(K):
        assert stats.kstest(S[:, k], "expon").pvalue > 1e-4, k
    # pairs: the joint law on an 8 x 8 grid of the unit square is flat
    for a in range(K):
        for b in range(a + 1, K):
            h, _, _ = np.histogram2d(U[:, a], U[:, b], bins=8, range=[[0, 1], [0, 1]])
            assert stats.chisquare(h.ravel()).pvalue > 1e-4, (a, b)
    # the minimum is Exp(K), sits at a uniformly random draft, and the excesses of the others over it
    # are Exp(1) again, independent of where it sits
    M, where = S.min(axis=1), S.argmin(axis=1)
    assert stats.kstest(M, "expon", args=(0, 1.0 / K)).pvalue > 1e-4
    assert stats.chisquare(np.bincount(where, minlength=K)).pvalue > 1e-4
    for k in range(K):
        rest = S[where != k, k] - M[where != k]
        assert stats.kstest(rest, "expon").pvalue > 1e-4, k
    # small times matter most (they win the races): the lower tail of every draft, finely
    for k in range(K):
        tail = S[:, k][S[:, k] < 0.05]
        assert abs(len(tail) / n - (1 - np.exp(-0.05))) < 4 * np.sqrt(0.05 / n)
        assert stats.kstest(tail, lambda s: (1 - np.exp(-s)) / (1 - np.exp(-0.05))).pvalue > 1e-4


def test_direct_and_min_first_times_differ_but_share_the_per_draft_words():
    a = oracle.race_times(9, 0, 50, 5, 4, min_first=False)
    b = oracle.race_times(9, 0, 50, 5, 4, min_first=True)
    assert not np.allclose(a, b)
    # away from the draft that holds the minimum, the excess over the minimum is the direct time
    M = b.min(axis=1, keepdims=True)
    mask = b > M
    np.testing.assert_allclose((b - M)[mask], a[mask], rtol=1e-12)
    assert (mask.sum(axis=1) == 3).all()


@pytest.mark.parametrize("K,V", [(1, 2), (2, 5), (3, 8), (4, 7)])
def test_matches_pure_python_algorithm(K, V):
    rng = np.random.default_rng(100 * K + V + 1)
    B = 120
    q32 = np.stack([_dirichlet(rng, V) for _ in range(B)]).astype(np.float32)
    p32 = np.stack([[_dirichlet(rng, V) for _ in range(K)] for _ in range(B)]).astype(np.float32)
    seed, off = 0xABCDEF0123, (1 << 33) + 5
    got = oracle.couple(p32, q32, K, kind=oracle.PROBS, seed=seed, row_offset=off, min_first=True)
    for b in range(B):
        X, Y, acc, keyX, keyY = gls_py.sample_gls(
            [[float(v) for v in p32[b, k]] for k in range(K)], [float(v) for v in q32[b]], seed, off + b,
            min_first=True)
        assert list(got["X"][b]) == X and got["Y"][b] == Y and bool(got["accept"][b]) == acc
        np.testing.assert_allclose(got["keyX"][b], keyX, rtol=1e-13)
        np.testing.assert_allclose(got["keyY"][b], keyY, rtol=1e-13)


@pytest.mark.parametrize("K,V,distinct", [(1, 2, False), (2, 5, False), (3, 8, False), (3, 5, True), (8, 6, True)])
def test_marginals_chi_square(K, V, distinct):
    # Proposition 1 (and its extension to distinct proposals): X^(k) ~ p^(k), Y ~ q
    rng = np.random.default_rng(K * 37 + V)
    B = 600_000
    q = _dirichlet(rng, V, 0.7).astype(np.float32)
    if distinct:
        ps = np.stack([_dirichlet(rng, V, 0.7) for _ in range(K)]).astype(np.float32)
        draft = np.broadcast_to(ps, (B, K, V))
    else:
        ps = np.tile(_dirichlet(rng, V, 0.7).astype(np.float32), (K, 1))
        draft = _bcast(ps[0], B)
    res = oracle.couple(draft, _bcast(q, B), K, kind=oracle.PROBS, seed=2025, min_first=True)
    qd = q.astype(np.float64) / q.astype(np.float64).sum()
    assert stats.chisquare(np.bincount(res["Y"], minlength=V), qd * B).pvalue > 1e-4
    for k in range(K):
        pd = ps[k].astype(np.float64) / ps[k].astype(np.float64).sum()
        assert stats.chisquare(np.bincount(res["X"][:, k], minlength=V), pd * B).pvalue > 1e-4, k
    # and jointly: pairs of drafts with one shared proposal are independent samples of it
    if not distinct and K >= 2:
        pd = ps[0].astype(np.float64) / ps[0].astype(np.float64).sum()
        joint = np.zeros((V, V))
        np.add.at(joint, (res["X"][:, 0], res["X"][:, 1]), 1)
        expect = np.outer(pd, pd) * B
        keep = expect > 5
        chi = ((joint - expect) ** 2 / expect)[keep].sum()
        assert stats.chi2.sf(chi, keep.sum() - 1) > 1e-4


@pytest.mark.parametrize("K", [1, 2, 4, 8])
def test_acceptance_rate_respects_the_list_matching_lemma(K):
    rng = np.random.default_rng(29)
    V, B = 10, 200_000
    p, q = _dirichlet(rng, V, 0.6).astype(np.float32), _dirichlet(rng, V, 0.6).astype(np.float32)
    res = oracle.couple(_bcast(p, B), _bcast(q, B), K, kind=oracle.PROBS, seed=41 + K, min_first=True)
    pd, qd = p.astype(np.float64) / p.astype(np.float64).sum(), q.astype(np.float64) / q.astype(np.float64).sum()
    bound = lml.lml_bound(pd, qd, K)
    rate = res["accept"].mean()
    assert rate >= bound - 4 * np.sqrt(bound * (1 - bound) / B), (K, rate, bound)
    # the two constructions are the same sampler in law: their acceptance rates agree
    other = oracle.couple(_bcast(p, B), _bcast(q, B), K, kind=oracle.PROBS, seed=41 + K)["accept"].mean()
    assert abs(rate - other) < 5 * np.sqrt(2 * 0.25 / B), (K, rate, other)


def test_winning_keys_are_exponential():
    rng = np.random.default_rng(19)
    V, B, K = 64, 100_000, 4
    zq = rng.normal(0, 2, V).astype(np.float32)
    zp = (zq + rng.normal(0, 1, V)).astype(np.float32)
    res = oracle.couple(_bcast(zp, B), _bcast(zq, B), K, kind=oracle.LOGITS, temp_target=0.8,
                        temp_draft_all=1.3, seed=3, min_first=True)
    assert stats.kstest(res["keyY"], "expon", args=(0, 1.0 / K)).pvalue > 1e-4
    for k in range(K):
        assert stats.kstest(res["keyX"][:, k], "expon").pvalue > 1e-4


def test_k1_is_the_two_party_gumbel_max_coupling_on_the_first_auxiliary_word():
    rng = np.random.default_rng(8)
    V, B, seed, off = 9, 400, 77, 1 << 34
    p = np.stack([_dirichlet(rng, V) for _ in range(B)]).astype(np.float32)
    q = np.stack([_dirichlet(rng, V) for _ in range(B)]).astype(np.float32)
    res = oracle.couple(p, q, 1, kind=oracle.PROBS, seed=seed, row_offset=off, min_first=True)
    for b in range(B):
        S = np.array([philox_py.race_time(philox_py.aux_word(seed, off + b, i, 0)) for i in range(V)])
        assert res["X"][b, 0] == np.argmin(S / p[b].astype(np.float64))
        assert res["Y"][b] == np.argmin(S / q[b].astype(np.float64))
        assert bool(res["accept"][b]) == (res["X"][b, 0] == res["Y"][b])


def test_pool_key_is_the_minimum_over_drafts_and_the_target_ignores_the_drafts():
    rng = np.random.default_rng(10)
    B, K, V = 300, 5, 40
    zq = rng.normal(0, 2, (B, V)).astype(np.float32)
    d1 = (zq[:, None, :] + rng.normal(0, 1, (B, K, V))).astype(np.float32)
    d2 = rng.normal(0, 3, (B, K, V)).astype(np.float32)
    a = oracle.couple(d1, zq, K, seed=12, min_first=True, partials=True)
    b = oracle.couple(d2, zq, K, seed=12, min_first=True)
    assert np.array_equal(a["Y"], b["Y"]) and np.array_equal(a["keyY"], b["keyY"])
    np.testing.assert_allclose(a["keyY"], a["keyYk"].min(axis=1), rtol=0)
    # importance-weight form goes through the same construction
    c = oracle.couple_is(zq, d1, seed=12, min_first=True)
    d = oracle.couple(d1, zq, K, kind=oracle.LOGW, seed=12, min_first=True)
    for name in ("X", "Y", "accept"):
        assert np.array_equal(c[name], d[name])
