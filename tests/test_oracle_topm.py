"""Pins for the oracle's candidate-list form of Algorithm 1 (Section 4.4), CPU only.

A list of (token id, value) pairs denotes the distribution that is zero off the list, so the
list form must agree with the dense oracle (itself pinned elsewhere) on rows that carry -inf
logits / zero probabilities outside the lists; the X and Y marginals must follow the truncated,
renormalised distributions; and a pure-Python evaluation must agree on tiny cases.
"""
import numpy as np
import pytest
from scipy import stats

import oracle
from oracle import philox_py


def _lists(rng, B, K, V, Md, Mt, shared):
    """Per row a pool of tokens with base logits; every list draws its tokens from the pool and
    perturbs the base logits, so the lists overlap but are not equal."""
    pool_size = max(Md, Mt) + 6
    pools = np.stack([rng.choice(V, size=pool_size, replace=False) for _ in range(B)])
    base = rng.normal(0, 2, size=(B, pool_size))

    def pick(M, noise):
        sel = np.stack([rng.choice(pool_size, size=M, replace=False) for _ in range(B)])
        ids = np.take_along_axis(pools, sel, 1).astype(np.int32)
        val = (np.take_along_axis(base, sel, 1) + noise * rng.normal(size=(B, M))).astype(np.float32)
        return ids, val
    t_ids, t_val = pick(Mt, 0.0)
    if shared:
        d_ids, d_val = pick(Md, 0.7)
    else:
        parts = [pick(Md, 0.7) for _ in range(K)]
        d_ids = np.stack([p[0] for p in parts], 1)
        d_val = np.stack([p[1] for p in parts], 1)
    return d_ids, d_val, t_ids, t_val


def _dense(ids, val, V, fill):
    out = np.full(ids.shape[:-1] + (V,), fill, np.float32)
    np.put_along_axis(out, ids.astype(np.int64), val, axis=-1)
    return out


@pytest.mark.parametrize("shared", [True, False])
@pytest.mark.parametrize("kind", ["logits", "probs", "logw"])
def test_list_form_equals_dense_form_with_no_mass_off_the_lists(shared, kind):
    rng = np.random.default_rng(11 + shared)
    B, K, V, Md, Mt = 300, 3, 500, 20, 35
    d_ids, d_val, t_ids, t_val = _lists(rng, B, K, V, Md, Mt, shared)
    code = {"logits": oracle.LOGITS, "probs": oracle.PROBS, "logw": oracle.LOGW}[kind]
    if kind == "probs":
        d_val, t_val = np.exp(d_val).astype(np.float32), np.exp(t_val).astype(np.float32)
    fill = 0.0 if kind == "probs" else -np.inf
    kw = dict(kind=code, temp_target=0.8, temp_draft_all=1.3, seed=5, row_offset=(1 << 34) + 7)
    got = oracle.couple_topm(d_ids, d_val, t_ids, t_val, K, **kw)
    ref = oracle.couple(_dense(d_ids, d_val, V, fill), _dense(t_ids, t_val, V, fill), K, **kw)
    for name in ("X", "Y", "accept", "match_k"):
        assert np.array_equal(got[name], ref[name]), name
    np.testing.assert_allclose(got["keyX"], ref["keyX"], rtol=1e-12)
    np.testing.assert_allclose(got["keyY"], ref["keyY"], rtol=1e-12)
    np.testing.assert_allclose(got["gapY"], ref["gapY"], rtol=1e-9)
    assert 0.2 < got["accept"].mean() < 1.0


def test_marginals_follow_the_truncated_renormalised_distributions():
    # one row of lists repeated over 4e5 rows of randomness: chi-square of X^(k) and Y
    rng = np.random.default_rng(3)
    n, K, V = 400_000, 2, 64
    d_ids = np.array([[3, 17, 40, 5, 63]], np.int32).repeat(n, 0)
    t_ids = np.array([[17, 3, 8, 63, 21, 40]], np.int32).repeat(n, 0)
    d_val = np.array([[0.3, 1.2, -0.5, 0.0, 0.8]], np.float32).repeat(n, 0)
    t_val = np.array([[1.0, 0.2, -1.0, 0.5, 0.1, 0.0]], np.float32).repeat(n, 0)
    out = oracle.couple_topm(d_ids, d_val, t_ids, t_val, K, temp_target=0.7, temp_draft_all=1.5, seed=9)
    p = np.exp(d_val[0] / 1.5); p /= p.sum()
    q = np.exp(t_val[0].astype(np.float64) / np.float64(np.float32(0.7))); q /= q.sum()
    for k in range(K):
        counts = np.array([(out["X"][:, k] == t).sum() for t in d_ids[0]])
        assert counts.sum() == n
        assert stats.chisquare(counts, p * n).pvalue > 1e-4
    counts = np.array([(out["Y"] == t).sum() for t in t_ids[0]])
    assert counts.sum() == n
    assert stats.chisquare(counts, q * n).pvalue > 1e-4
    # tokens that are on one list only can never be where the two sides meet
    both = set(d_ids[0]) & set(t_ids[0])
    assert set(np.unique(out["Y"][out["accept"] == 1])) <= both


def test_pure_python_evaluation_on_tiny_lists():
    rng = np.random.default_rng(8)
    B, K, V, Md, Mt = 40, 3, 30, 4, 5
    d_ids, d_val, t_ids, t_val = _lists(rng, B, K, V, Md, Mt, shared=False)
    seed, base = 77, 12
    out = oracle.couple_topm(d_ids, d_val, t_ids, t_val, K, seed=seed, row_offset=base)
    for b in range(B):
        q = np.exp(t_val[b].astype(np.float64)); q /= q.sum()
        pool = [(philox_py.race_time(philox_py.shared_word(seed, base + b, k, int(t))) / q[e], int(t), k)
                for k in range(K) for e, t in enumerate(t_ids[b])]
        assert out["Y"][b] == min(pool)[1]
        assert abs(out["keyY"][b] / min(pool)[0] - 1) < 1e-12
        for k in range(K):
            p = np.exp(d_val[b, k].astype(np.float64)); p /= p.sum()
            keys = [(philox_py.race_time(philox_py.shared_word(seed, base + b, k, int(t))) / p[e], int(t))
                    for e, t in enumerate(d_ids[b, k])]
            assert out["X"][b, k] == min(keys)[1]
        assert out["accept"][b] == int(out["Y"][b] in out["X"][b])


def test_empty_slots_duplicates_and_lists_without_mass():
    ids_d = np.array([[5, -1, 9, 5]], np.int32)
    val_d = np.array([[0.0, 50.0, 1.0, 2.0]], np.float32)          # the big value sits in an empty slot
    ids_t = np.array([[9, 5, -1]], np.int32)
    val_t = np.array([[0.5, 0.5, 9.0]], np.float32)
    n = 20000
    out = oracle.couple_topm(ids_d.repeat(n, 0), val_d.repeat(n, 0), ids_t.repeat(n, 0), val_t.repeat(n, 0), 1, seed=3)
    assert set(np.unique(out["X"])) == {5, 9} and set(np.unique(out["Y"])) == {5, 9}
    # id 5 appears twice with weights e^0 and e^2; with one shared race time the larger always wins,
    # so token 5 is drawn with probability e^2 / (e^2 + e^1) of the two contenders 5 (as e^2) and 9
    share = (out["X"][:, 0] == 5).mean()
    assert abs(share - np.e ** 2 / (np.e ** 2 + np.e)) < 0.01
    # a target list without mass: Y = -1, no acceptance
    none = oracle.couple_topm(ids_d, val_d, np.array([[-1, -1, -1]], np.int32), val_t, 2, seed=1)
    assert none["Y"][0] == -1 and none["accept"][0] == 0 and none["match_k"][0] == -1
    ninf = oracle.couple_topm(ids_d, np.full((1, 4), -np.inf, np.float32), ids_t, val_t, 2, seed=1)
    assert (ninf["X"] == -1).all() and ninf["accept"][0] == 0


def test_full_lists_reduce_to_the_dense_sampler():
    # lists that enumerate the whole vocabulary in a scrambled order give Algorithm 1 itself
    rng = np.random.default_rng(21)
    B, K, V = 200, 4, 97
    tq = rng.normal(0, 2, (B, V)).astype(np.float32)
    td = (tq + rng.normal(0, 1, (B, V))).astype(np.float32)
    perm_t = np.stack([rng.permutation(V) for _ in range(B)]).astype(np.int32)
    perm_d = np.stack([rng.permutation(V) for _ in range(B)]).astype(np.int32)
    got = oracle.couple_topm(perm_d, np.take_along_axis(td, perm_d.astype(np.int64), 1),
                             perm_t, np.take_along_axis(tq, perm_t.astype(np.int64), 1), K, seed=4)
    ref = oracle.couple(td, tq, K, seed=4)
    for name in ("X", "Y", "accept", "match_k"):
        assert np.array_equal(got[name], ref[name])
