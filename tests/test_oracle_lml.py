"""Pins for the oracle's batched evaluation of Theorem 1's bound (CPU only).

The strictly positive case is pinned in test_oracle_gls.py (literal double sum, p = q, the K = 1
closed form against measured matching rates).  Here: the treatment of entries without mass
against the limit of the literal double sum, and the conversion from logits / log-weights /
probabilities.
"""
import numpy as np
import pytest

from oracle import lml


def test_entries_without_mass_follow_the_limit_of_the_double_sum():
    rng = np.random.default_rng(4)
    for trial in range(20):
        V = int(rng.integers(4, 40))
        p = rng.dirichlet(np.full(V, 0.5))
        q = rng.dirichlet(np.full(V, 0.5))
        zp = rng.random(V) < 0.25
        zq = (rng.random(V) < 0.25) & ~zp
        both = rng.random(V) < 0.1
        p[zp | both] = 0.0
        q[zq | both] = 0.0
        if p.sum() == 0 or q.sum() == 0:
            continue
        p /= p.sum(); q /= q.sum()
        eps = 1e-13
        pe = np.where(p > 0, p, eps); qe = np.where(q > 0, q, eps)
        pe /= pe.sum(); qe /= qe.sum()
        for K in (1, 3, 8):
            got = lml.lml_bound_support(p, q, K)
            lim = lml.lml_bound_literal(pe, qe, K)
            assert abs(got - lim) < 1e-9 * max(1.0, V), (trial, K, got, lim)
            assert 0.0 <= got <= 1.0 + 1e-12


def test_support_form_equals_plain_form_on_positive_inputs_and_disjoint_supports_give_zero():
    rng = np.random.default_rng(5)
    p = rng.dirichlet(np.ones(50)); q = rng.dirichlet(np.ones(50))
    for K in (1, 2, 16):
        assert abs(lml.lml_bound_support(p, q, K) - lml.lml_bound(p, q, K)) < 1e-13
    a = np.array([0.5, 0.5, 0.0, 0.0]); b = np.array([0.0, 0.0, 0.3, 0.7])
    assert lml.lml_bound_support(a, b, 4) == 0.0
    # p = q on a sub-support: the bound is 1 whatever K is
    c = np.array([0.2, 0.0, 0.8, 0.0])
    assert abs(lml.lml_bound_support(c, c, 5) - 1.0) < 1e-13


@pytest.mark.parametrize("kind", ["logits", "logw", "probs"])
def test_rows_from_raw_inputs(kind):
    rng = np.random.default_rng(6)
    B, V = 5, 300
    tq = rng.normal(0, 2, (B, V)).astype(np.float32)
    td = (tq + rng.normal(0, 1, (B, V))).astype(np.float32)
    td[0, :7] = -np.inf
    tq[1, 5:9] = -np.inf
    tp, tt = 1.3, 0.7
    if kind == "probs":
        d, t = np.exp(td), np.exp(tq)
        p = d.astype(np.float64) / d.astype(np.float64).sum(1, keepdims=True)
        q = t.astype(np.float64) / t.astype(np.float64).sum(1, keepdims=True)
    else:
        cp = 1.0 / float(np.float32(tp)) if kind == "logits" else 1.0
        cq = 1.0 / float(np.float32(tt)) if kind == "logits" else 1.0
        with np.errstate(over="ignore"):
            p = np.exp(td.astype(np.float64) * cp); p /= p.sum(1, keepdims=True)
            q = np.exp(tq.astype(np.float64) * cq); q /= q.sum(1, keepdims=True)
        d, t = td, tq
    out = lml.lml_rows(d, t, [1, 4], kind=kind, temp_draft=tp, temp_target=tt)
    for b in range(B):
        for n, K in enumerate((1, 4)):
            assert abs(out["bound"][b, n] - lml.lml_bound_support(p[b], q[b], K)) < 1e-12
            assert out["relaxed"][b, n] <= out["bound"][b, n] + 1e-12
        assert abs(out["tv"][b] - 0.5 * np.abs(p[b] - q[b]).sum()) < 1e-12
        # K = 1 is the exact matching probability of the two-party coupling: at least (1-tv)/(1+tv)
        assert out["bound"][b, 0] >= (1 - out["tv"][b]) / (1 + out["tv"][b]) - 1e-12
