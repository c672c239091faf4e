"""Lower bounds and closed forms for the matching probability (test infrastructure).

Theorem 1 (list matching lemma) and its relaxed form, the K = 1 closed form of
Remark 1, the two-party Gumbel-max bound of the introduction and the
conditional bound of Theorem 2 / Appendix C, in numpy fp64.  The literal O(V^2)
double sum is kept beside the sorted O(V log V) evaluation so that each checks
the other.
"""
import numpy as np


def lml_bound_literal(p, q, K):
    """Theorem 1, eq. (1), written as the double sum it is.  p, q: 1-D, strictly positive."""
    p = np.asarray(p, np.float64)
    q = np.asarray(q, np.float64)
    total = 0.0
    for j in range(len(q)):
        denom = np.sum(np.maximum(q / q[j], p / p[j]) + (K - 1) * q / q[j])
        total += K / denom
    return float(total)


def lml_bound(p, q, K):
    """Theorem 1, eq. (1), in O(V log V).

    max{q_i/q_j, p_i/p_j} = q_i/q_j  iff  q_i/p_i >= q_j/p_j, so after sorting by
    r = q/p the inner sum splits into a suffix sum of q and a prefix sum of p.
    """
    p = np.asarray(p, np.float64)
    q = np.asarray(q, np.float64)
    order = np.argsort(q / p, kind="stable")
    ps, qs = p[order], q[order]
    # for position j in sorted order: i >= j (r_i >= r_j) contribute q_i/q_j, i < j contribute p_i/p_j
    q_suffix = np.cumsum(qs[::-1])[::-1]
    p_prefix = np.cumsum(ps) - ps
    denom = q_suffix / qs + p_prefix / ps + (K - 1) * qs.sum() / qs
    return float(np.sum(K / denom))


def lml_relaxed(p, q, K):
    """The relaxed bound below Theorem 1's proof: sum_j q_j (1 + q_j / (K p_j))^-1."""
    p = np.asarray(p, np.float64)
    q = np.asarray(q, np.float64)
    return float(np.sum(q / (1.0 + q / (K * p))))


def k1_matching_probability(p, q):
    """Remark 1, K = 1: Pr[Y = X] = sum_j 1 / sum_i max{q_i/q_j, p_i/p_j} (exact)."""
    return lml_bound(p, q, 1)


def tv_distance(p, q):
    return 0.5 * float(np.sum(np.abs(np.asarray(p, np.float64) - np.asarray(q, np.float64))))


def gumbel_two_party_bound(p, q):
    """Introduction: Pr[X = Y] >= (1 - d_TV) / (1 + d_TV) for the two-party Gumbel-max coupling."""
    d = tv_distance(p, q)
    return (1.0 - d) / (1.0 + d)


def conditional_bound(lam_q_at_y, lam_p_at_y):
    """Theorem 2 in importance-weight form (Appendix C): sum_k (K + lam_q,j / lam_p,j^(k))^-1.

    lam_q_at_y: [B] normalised encoder weights at the selected index;
    lam_p_at_y: [B,K] normalised decoder weights at that index.  Returns [B].
    """
    lam_q_at_y = np.asarray(lam_q_at_y, np.float64)
    lam_p_at_y = np.asarray(lam_p_at_y, np.float64)
    K = lam_p_at_y.shape[1]
    with np.errstate(divide="ignore"):
        ratio = lam_q_at_y[:, None] / lam_p_at_y
    return np.sum(1.0 / (K + ratio), axis=1)


def lml_bound_support(p, q, K):
    """Theorem 1, eq. (1), for distributions that may have entries without mass.

    The limits of the formula: an index j with p_j = 0 or q_j = 0 adds no term (its inner sum
    is infinite, or its numerator side vanishes), while as a summand i such an index still
    contributes the mass it has on the other side: q_i/q_j if p_i = 0 (its ratio q/p is
    infinite), p_i/p_j if q_i = 0 (ratio 0).  With strictly positive inputs this is lml_bound.
    """
    p = np.asarray(p, np.float64)
    q = np.asarray(q, np.float64)
    keep = (p > 0) | (q > 0)
    p, q = p[keep], q[keep]
    with np.errstate(divide="ignore"):
        r = np.where(p > 0, q / np.where(p > 0, p, 1.0), np.inf)
    order = np.argsort(r, kind="stable")
    ps, qs = p[order], q[order]
    q_suffix = np.cumsum(qs[::-1])[::-1]
    p_prefix = np.cumsum(ps) - ps
    both = (ps > 0) & (qs > 0)
    denom = q_suffix[both] / qs[both] + p_prefix[both] / ps[both] + (K - 1) * qs.sum() / qs[both]
    return float(np.sum(K / denom))


def distributions(values, kind, temp=1.0):
    """Rows of fp64 probabilities from rows of logits (softmax of x / T, T read as the float32
    the sampler takes), log-weights (normalised exp) or probabilities (divided by their sum)."""
    x = np.asarray(values, np.float64)
    if kind == "probs":
        w = np.where(np.isfinite(x) & (x > 0), x, 0.0)
    else:
        t = float(np.float32(temp)) if kind == "logits" else 1.0
        ok = np.isfinite(x)
        m = np.max(np.where(ok, x, -np.inf), axis=-1, keepdims=True)
        with np.errstate(invalid="ignore"):
            w = np.where(ok, np.exp((np.where(ok, x, 0.0) - m) / t), 0.0)
    return w / w.sum(axis=-1, keepdims=True)


def lml_rows(draft, target, ks, kind="logits", temp_draft=1.0, temp_target=1.0):
    """Per row and per list size: Theorem 1's bound, its relaxed form, and the TV distance."""
    p = distributions(draft, kind, temp_draft)
    q = distributions(target, kind, temp_target)
    B = p.shape[0]
    bound = np.empty((B, len(ks)))
    relaxed = np.empty((B, len(ks)))
    for b in range(B):
        both = (p[b] > 0) & (q[b] > 0)
        for n, K in enumerate(ks):
            bound[b, n] = lml_bound_support(p[b], q[b], K)
            relaxed[b, n] = lml_relaxed(p[b][both], q[b][both], K)
    tv = 0.5 * np.abs(p - q).sum(axis=1)
    return {"bound": bound, "relaxed": relaxed, "tv": tv}
