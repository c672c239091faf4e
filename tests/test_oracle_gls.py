"""Pins for the CPU oracle of Algorithm 1 (CPU only).

Each test checks the C++ oracle against something the paper or the mathematics
fixes, not against itself: the marginal laws of Proposition 1 (and its
extension to distinct proposals), the race-time laws used in its proof, the
list matching lemma's lower bound, the three cases in which that bound is
exact (Remark 1), the two-party Gumbel-max coupling it must reduce to for
K = 1, drafter invariance of Y, and a pure-Python brute force on tiny inputs.
"""
import math

import numpy as np
import pytest
from scipy import stats

import oracle
from oracle import gls_py, lml, philox_py


def _dirichlet(rng, V, alpha=1.0):
    return rng.dirichlet(np.full(V, alpha))


def _bcast(vec, B):
    """[V] -> [B,V] without copying (row stride 0)."""
    return np.broadcast_to(np.asarray(vec, np.float32), (B, len(vec)))


# ---------------------------------------------------------------- brute force on tiny inputs
@pytest.mark.parametrize("K,V", [(1, 2), (2, 5), (3, 8), (4, 7)])
def test_matches_pure_python_algorithm(K, V):
    rng = np.random.default_rng(100 * K + V)
    B = 150
    q32 = np.stack([_dirichlet(rng, V) for _ in range(B)]).astype(np.float32)
    p32 = np.stack([[_dirichlet(rng, V) for _ in range(K)] for _ in range(B)]).astype(np.float32)
    seed, off = 0xABCDEF0123, 1 << 33
    got = oracle.couple(p32, q32, K, kind=oracle.PROBS, seed=seed, row_offset=off)
    for b in range(B):
        X, Y, acc, keyX, keyY = gls_py.sample_gls(
            [[float(v) for v in p32[b, k]] for k in range(K)], [float(v) for v in q32[b]], seed, off + b)
        assert list(got["X"][b]) == X
        assert got["Y"][b] == Y
        assert bool(got["accept"][b]) == acc
        np.testing.assert_allclose(got["keyX"][b], keyX, rtol=1e-13)
        np.testing.assert_allclose(got["keyY"][b], keyY, rtol=1e-13)


# ---------------------------------------------------------------- Proposition 1: marginals
@pytest.mark.parametrize("K,V,distinct", [(1, 2, False), (2, 5, False), (3, 8, False), (3, 5, True)])
def test_marginals_chi_square(K, V, distinct):
    rng = np.random.default_rng(K * 31 + V)
    B = 1_000_000
    q = _dirichlet(rng, V, 0.7).astype(np.float32)
    if distinct:
        ps = np.stack([_dirichlet(rng, V, 0.7) for _ in range(K)]).astype(np.float32)
        draft = np.broadcast_to(ps, (B, K, V))
    else:
        ps = np.tile(_dirichlet(rng, V, 0.7).astype(np.float32), (K, 1))
        draft = _bcast(ps[0], B)
    res = oracle.couple(draft, _bcast(q, B), K, kind=oracle.PROBS, seed=2024)
    qd = q.astype(np.float64) / q.astype(np.float64).sum()
    cy = np.bincount(res["Y"], minlength=V)
    assert stats.chisquare(cy, qd * B).pvalue > 1e-4
    for k in range(K):
        pd = ps[k].astype(np.float64) / ps[k].astype(np.float64).sum()
        cx = np.bincount(res["X"][:, k], minlength=V)
        assert stats.chisquare(cx, pd * B).pvalue > 1e-4, k


def test_marginals_with_softmax_and_temperature():
    # logits path: p = softmax(z / T); the X marginal must follow that law, which pins the
    # temperature's place and the normalisation
    rng = np.random.default_rng(5)
    V, K, B = 6, 2, 400_000
    zq = rng.normal(0, 2, V).astype(np.float32)
    zp = (zq + rng.normal(0, 1, V)).astype(np.float32)
    Tq, Tp = 0.7, 1.6
    res = oracle.couple(_bcast(zp, B), _bcast(zq, B), K, kind=oracle.LOGITS, temp_target=Tq,
                        temp_draft_all=Tp, seed=99)
    soft = lambda z, T: np.exp(z / T - np.max(z / T)) / np.exp(z / T - np.max(z / T)).sum()
    assert stats.chisquare(np.bincount(res["Y"], minlength=V), soft(zq.astype(np.float64), np.float32(Tq).astype(np.float64)) * B).pvalue > 1e-4
    for k in range(K):
        assert stats.chisquare(np.bincount(res["X"][:, k], minlength=V),
                               soft(zp.astype(np.float64), np.float32(Tp).astype(np.float64)) * B).pvalue > 1e-4
    # per-draft temperatures
    res2 = oracle.couple(_bcast(zp, B), _bcast(zq, B), K, kind=oracle.LOGITS, temp_target=Tq,
                         temp_draft=[0.5, 2.0], seed=99)
    for k, T in enumerate([0.5, 2.0]):
        assert stats.chisquare(np.bincount(res2["X"][:, k], minlength=V),
                               soft(zp.astype(np.float64), T) * B).pvalue > 1e-4
    assert np.array_equal(res2["Y"], res["Y"])


# ---------------------------------------------------------------- race-time laws (proof of Prop. 1)
@pytest.mark.parametrize("K", [1, 4])
def test_winning_keys_are_exponential(K):
    # min_i S_i / p_i ~ Exp(1) for normalised p; the pool's winner ~ Exp(K)
    rng = np.random.default_rng(17 + K)
    V, B = 64, 100_000
    zq = rng.normal(0, 2, V).astype(np.float32)
    zp = (zq + rng.normal(0, 1, V)).astype(np.float32)
    res = oracle.couple(_bcast(zp, B), _bcast(zq, B), K, kind=oracle.LOGITS, temp_target=0.8,
                        temp_draft_all=1.3, seed=3)
    assert stats.kstest(res["keyY"], "expon", args=(0, 1.0 / K)).pvalue > 1e-4
    for k in range(K):
        assert stats.kstest(res["keyX"][:, k], "expon").pvalue > 1e-4
    # the probability kind reports keys for p as given: scale 1 / sum(p)
    p_raw = np.exp(zp.astype(np.float64)).astype(np.float32)
    res = oracle.couple(_bcast(p_raw, B), _bcast(p_raw, B), K, kind=oracle.PROBS, seed=4)
    scale = 1.0 / p_raw.astype(np.float64).sum()
    assert stats.kstest(res["keyX"][:, 0], "expon", args=(0, scale)).pvalue > 1e-4


# ---------------------------------------------------------------- Theorem 1 and Remark 1
def test_lml_fast_evaluation_matches_literal_double_sum():
    rng = np.random.default_rng(11)
    for V in (2, 10, 257, 1024):
        p, q = _dirichlet(rng, V, 0.5) + 1e-12, _dirichlet(rng, V, 0.5) + 1e-12
        for K in (1, 3, 8):
            a, b = lml.lml_bound_literal(p, q, K), lml.lml_bound(p, q, K)
            assert abs(a - b) < 1e-10, (V, K, a, b)
            assert lml.lml_relaxed(p, q, K) <= a + 1e-12
    p = _dirichlet(rng, 50)
    assert abs(lml.lml_bound(p, p, 4) - 1.0) < 1e-12


@pytest.mark.parametrize("K", [1, 2, 4, 8])
def test_acceptance_rate_respects_lml(K):
    rng = np.random.default_rng(23)
    V, B = 10, 200_000
    p, q = _dirichlet(rng, V).astype(np.float32), _dirichlet(rng, V).astype(np.float32)
    res = oracle.couple(_bcast(p, B), _bcast(q, B), K, kind=oracle.PROBS, seed=K)
    rate = res["accept"].mean()
    pd, qd = p.astype(np.float64) / p.astype(np.float64).sum(), q.astype(np.float64) / q.astype(np.float64).sum()
    bound = lml.lml_bound(pd, qd, K)
    sigma = math.sqrt(max(rate * (1 - rate), 1e-9) / B)
    assert rate >= bound - 4 * sigma, (rate, bound)
    if K == 1:
        # exact for K = 1 (Remark 1), and above the two-party Gumbel-max bound
        assert abs(rate - lml.k1_matching_probability(pd, qd)) < 4 * sigma + 1e-9
        assert rate >= lml.gumbel_two_party_bound(pd, qd) - 4 * sigma
    # conditional form: Pr[accept | Y = j] >= (1 + q_j / (K p_j))^-1
    for j in range(V):
        sel = res["Y"] == j
        n = int(sel.sum())
        if n < 2000:
            continue
        r = res["accept"][sel].mean()
        lb = 1.0 / (1.0 + qd[j] / (K * pd[j]))
        assert r >= lb - 4 * math.sqrt(max(r * (1 - r), 1e-9) / n), (j, r, lb)
    # accept is exactly "Y is in the list", match_k the first position
    inlist = (res["X"] == res["Y"][:, None])
    assert np.array_equal(res["accept"].astype(bool), inlist.any(axis=1))
    first = np.where(inlist.any(axis=1), inlist.argmax(axis=1), -1)
    assert np.array_equal(res["match_k"], first)


def test_acceptance_rate_grows_with_K():
    rng = np.random.default_rng(29)
    V, B = 12, 100_000
    p, q = _dirichlet(rng, V).astype(np.float32), _dirichlet(rng, V).astype(np.float32)
    rates = [oracle.couple(_bcast(p, B), _bcast(q, B), K, kind=oracle.PROBS, seed=5)["accept"].mean()
             for K in (1, 2, 4, 8, 16)]
    # same seed: lists are nested in K, so on every row accept can only switch on... Y changes with K,
    # hence only the rate is compared, with slack for sampling noise
    for lo, hi in zip(rates, rates[1:]):
        assert hi >= lo - 0.01
    assert rates[-1] > rates[0] + 0.05


def test_identical_distributions_always_accept():
    rng = np.random.default_rng(31)
    B, V = 2000, 300
    z = rng.normal(0, 3, (B, V)).astype(np.float32)
    for K in (1, 3, 8):
        res = oracle.couple(z, z, K, kind=oracle.LOGITS, temp_target=0.9, temp_draft_all=0.9, seed=K)
        assert res["accept"].all()


def test_one_hot_proposal():
    rng = np.random.default_rng(37)
    V, B, K = 9, 200_000, 3
    p = np.zeros(V, np.float32)
    p[4] = 1.0
    q = _dirichlet(rng, V).astype(np.float32)
    res = oracle.couple(_bcast(p, B), _bcast(q, B), K, kind=oracle.PROBS, seed=8)
    assert (res["X"] == 4).all()
    qd = q.astype(np.float64) / q.astype(np.float64).sum()
    rate = res["accept"].mean()
    assert abs(rate - qd[4]) < 4 * math.sqrt(qd[4] * (1 - qd[4]) / B)


# ---------------------------------------------------------------- K = 1: two-party Gumbel-max coupling
def test_k1_equals_gumbel_max_on_the_same_stream():
    # Gumbel-max: argmax_i (ln p_i + G_i), G_i = -ln(-ln U_i); the same U drive both parties
    rng = np.random.default_rng(41)
    B, V = 300, 37
    seed = 77
    p = np.stack([_dirichlet(rng, V) for _ in range(B)]).astype(np.float32)
    q = np.stack([_dirichlet(rng, V) for _ in range(B)]).astype(np.float32)
    res = oracle.couple(p, q, 1, kind=oracle.PROBS, seed=seed)
    for b in range(B):
        U = np.array([philox_py.uniform(philox_py.shared_word(seed, b, 0, i)) for i in range(V)])
        G = -np.log(-np.log(U))
        assert res["X"][b, 0] == int(np.argmax(np.log(p[b].astype(np.float64)) + G))
        assert res["Y"][b] == int(np.argmax(np.log(q[b].astype(np.float64)) + G))


# ---------------------------------------------------------------- structure of the pool and invariance
def test_pool_is_min_over_drafts_and_partials_agree():
    rng = np.random.default_rng(43)
    B, V, K = 500, 64, 5
    zq = rng.normal(0, 2, (B, V)).astype(np.float32)
    zp = rng.normal(0, 2, (B, K, V)).astype(np.float32)
    res = oracle.couple(zp, zq, K, kind=oracle.LOGITS, seed=6, partials=True)
    # Y is the per-draft target-side winner with the smallest key
    kbest = res["keyYk"].argmin(axis=1)
    assert np.array_equal(res["Y"], res["Yk"][np.arange(B), kbest])
    np.testing.assert_array_equal(res["keyY"], res["keyYk"].min(axis=1))
    # the flattened K*V race with the augmented target (q/K, ..., q/K) picks the same index
    for b in range(20):
        zz = zq[b].astype(np.float64)
        qn = np.exp(zz - zz.max()) / np.exp(zz - zz.max()).sum()
        T = np.array([[philox_py.race_time(philox_py.shared_word(6, b, k, i)) for i in range(V)]
                      for k in range(K)]).reshape(-1)
        flat = int(np.argmin(T / np.tile(qn / K, K)))
        assert flat % V == res["Y"][b]


def test_target_sample_ignores_the_drafts():
    rng = np.random.default_rng(47)
    B, V, K = 400, 128, 4
    zq = rng.normal(0, 2, (B, V)).astype(np.float32)
    a = oracle.couple(rng.normal(0, 2, (B, V)).astype(np.float32), zq, K, seed=12)
    b = oracle.couple(rng.normal(0, 5, (B, K, V)).astype(np.float32), zq, K, seed=12, temp_draft_all=3.0)
    assert np.array_equal(a["Y"], b["Y"])
    assert np.array_equal(a["keyY"], b["keyY"])
    assert not np.array_equal(a["X"], b["X"])


def test_row_offset_and_seed_define_the_stream():
    rng = np.random.default_rng(53)
    B, V, K = 64, 50, 3
    zq = rng.normal(0, 2, (B, V)).astype(np.float32)
    zp = rng.normal(0, 2, (B, V)).astype(np.float32)
    full = oracle.couple(zp, zq, K, seed=9, row_offset=1000)
    part = oracle.couple(zp[16:48], zq[16:48], K, seed=9, row_offset=1016)
    assert np.array_equal(full["X"][16:48], part["X"])
    assert np.array_equal(full["Y"][16:48], part["Y"])
    other = oracle.couple(zp, zq, K, seed=10, row_offset=1000)
    assert not np.array_equal(full["X"], other["X"])
    single = oracle.couple(zp, zq, K, seed=9, row_offset=1000, threads=1)
    assert np.array_equal(full["X"], single["X"]) and np.array_equal(full["Y"], single["Y"])


# ---------------------------------------------------------------- inputs: bf16, degenerate rows
def test_bf16_inputs_are_widened_exactly():
    rng = np.random.default_rng(59)
    B, V, K = 50, 200, 2
    z = rng.normal(0, 2, (B, V)).astype(np.float32)
    bits = (z.view(np.uint32) >> 16).astype(np.uint16)          # truncate to bf16
    widened = (bits.astype(np.uint32) << 16).view(np.float32)
    a = oracle.couple(bits, bits, K, dtype=oracle.BF16, seed=1)
    b = oracle.couple(widened, widened, K, dtype=oracle.F32, seed=1)
    for name in ("X", "Y", "accept", "keyX", "keyY"):
        assert np.array_equal(a[name], b[name])


def test_degenerate_and_masked_rows():
    V, K = 16, 2
    z = np.zeros((4, V), np.float32)
    z[0, :] = -np.inf                       # nothing has mass
    z[1, :] = -np.inf
    z[1, 5] = 0.0                           # a single atom
    z[2, 3] = np.nan                        # NaN carries no mass
    z[3, 7] = np.inf                        # +inf carries no mass either
    res = oracle.couple(z, z, K, seed=2)
    assert res["Y"][0] == -1 and (res["X"][0] == -1).all() and res["accept"][0] == 0
    assert res["match_k"][0] == -1 and np.isinf(res["keyY"][0])
    assert res["Y"][1] == 5 and (res["X"][1] == 5).all() and res["accept"][1] == 1
    many = oracle.couple(np.broadcast_to(z[2], (5000, V)), np.broadcast_to(z[2], (5000, V)), K, seed=3)
    assert not (many["Y"] == 3).any() and not (many["X"] == 3).any()
    many = oracle.couple(np.broadcast_to(z[3], (5000, V)), np.broadcast_to(z[3], (5000, V)), K, seed=3)
    assert not (many["Y"] == 7).any() and (many["Y"] >= 0).all()
    p = np.array([[0.5, -1.0, np.nan, 0.0, 0.5]], np.float32)
    many = oracle.couple(np.broadcast_to(p[0], (5000, 5)), np.broadcast_to(p[0], (5000, 5)), 1,
                         kind=oracle.PROBS, seed=4)
    assert set(np.unique(many["Y"])) == {0, 4}


def test_gap_is_relative_distance_to_runner_up():
    rng = np.random.default_rng(61)
    B, V, K = 40, 30, 2
    p = np.stack([_dirichlet(rng, V) for _ in range(B)]).astype(np.float32)
    res = oracle.couple(p, p, K, kind=oracle.PROBS, seed=21, partials=True)
    for b in range(B):
        for k in range(K):
            keys = np.array([philox_py.race_time(philox_py.shared_word(21, b, k, i)) / float(p[b, i])
                             for i in range(V)])
            srt = np.sort(keys)
            assert abs(res["gapX"][b, k] - (srt[1] - srt[0]) / srt[0]) < 1e-9
            assert abs(res["gapYk"][b, k] - (srt[1] - srt[0]) / srt[0]) < 1e-9


# ---------------------------------------------------------------- importance-weight form (Appendix C)
def test_importance_form_is_the_logweight_kind_and_respects_conditional_bound():
    rng = np.random.default_rng(67)
    B, N, L = 3000, 256, 3
    rho, s2 = 0.9, 0.25
    x = rng.normal(size=B)
    u = rng.normal(size=(B, N))
    y = x[:, None] + math.sqrt(s2) * rng.normal(size=(B, L))
    ratio = lambda uu, m, v: -0.5 * math.log(v) - 0.5 * (uu - m) ** 2 / v + 0.5 * uu ** 2
    enc = ratio(u, rho * x[:, None], 1 - rho ** 2).astype(np.float32)
    dec = np.stack([ratio(u, rho * y[:, l:l + 1] / (1 + s2), 1 - rho ** 2 / (1 + s2)) for l in range(L)],
                   axis=1).astype(np.float32)
    a = oracle.couple_is(enc, dec, seed=31)
    b = oracle.couple(dec, enc, L, kind=oracle.LOGW, seed=31)
    for name in ("X", "Y", "accept", "match_k", "keyX", "keyY"):
        assert np.array_equal(a[name], b[name])
    # log-weights shifted by a constant per row / per decoder describe the same normalised weights
    c = oracle.couple_is(enc + np.float32(2.0), dec - np.float32(4.0), seed=31)
    assert np.array_equal(a["X"], c["X"]) and np.array_equal(a["Y"], c["Y"])
    # conditional bound given the candidates: E[sum_l (L + lam_q,Y / lam_p,Y^(l))^-1] <= Pr[accept]
    lam = lambda w: np.exp(w - w.max(axis=-1, keepdims=True)) / np.exp(w - w.max(axis=-1, keepdims=True)).sum(axis=-1, keepdims=True)
    lq = lam(enc.astype(np.float64))[np.arange(B), a["Y"]]
    lp = lam(dec.astype(np.float64))[np.arange(B)[:, None], np.arange(L)[None, :], a["Y"][:, None]]
    bound = lml.conditional_bound(lq, lp).mean()
    rate = a["accept"].mean()
    assert rate >= bound - 4 * math.sqrt(rate * (1 - rate) / B), (rate, bound)
    # the encoder's index is distributed as lam_q: pooled chi-square through the probability integral
    assert a["accept"].mean() > 0.3
