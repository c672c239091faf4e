"""Pins for the oracle's Algorithm 2 (drafter-invariant multi-draft speculative decoding), CPU only.

The verification loop is pinned to what Section 4.2 states about it: the output follows the
target model's autoregressive law exactly (sequence-level correctness), the first token is
Algorithm 1's target sample, a block emits one more token than it accepted, and under the
strong variant the emitted tokens do not depend on the drafts at all.
"""
import math

import numpy as np
import pytest
from scipy import stats

import oracle
from oracle import gls_py


def _markov(rng, V, conc=1.0):
    """Row-stochastic table M[prev, next] and its log."""
    M = rng.dirichlet(np.full(V, conc), size=V)
    return M, np.log(M).astype(np.float32)


def _speculate(logMb, logMs, S, L, K, n_tokens, seed, strong=False, draft_temp=1.0, min_first=False):
    """Run blocks of (draft L tokens with K drafts, verify) until every sequence has n_tokens."""
    V = logMb.shape[0]
    ctx = np.zeros(S, np.int64)                       # context = the last emitted token, start at 0
    out = [[] for _ in range(S)]
    base = 0
    n_blocks = 0
    while min(len(o) for o in out) < n_tokens:
        prev = np.repeat(ctx[:, None], K, axis=1)     # last token of each draft's prefix
        tokens = np.zeros((S, L, K), np.int32)
        target = np.zeros((S, L + 1, K, V), np.float32)
        for j in range(L):
            target[:, j] = logMb[prev]
            draft = np.ascontiguousarray(logMs[prev])  # [S, K, V]
            res = oracle.couple(draft, draft[:, 0], K, seed=seed, row_offset=base + j * S,
                                temp_draft_all=draft_temp, min_first=min_first)
            tokens[:, j] = res["X"]
            prev = res["X"].astype(np.int64)
        target[:, L] = logMb[prev]
        ver = oracle.verify(target, tokens, seed=seed, row_offset=base, row_stride_s=1, row_stride_j=S,
                            strong=strong, min_first=min_first)
        for s in range(S):
            n = ver["n_out"][s]
            out[s].extend(int(t) for t in ver["Y"][s, :n])
            ctx[s] = ver["Y"][s, n - 1]
        base += (L + 1) * S
        n_blocks += 1
    return np.array([o[:n_tokens] for o in out]), n_blocks


@pytest.mark.parametrize("strong,min_first", [(False, False), (True, False), (False, True), (True, True)])
def test_output_follows_the_target_models_autoregressive_law(strong, min_first):
    rng = np.random.default_rng(3)
    V, S, L, K, N = 3, 60_000, 2, 2, 3
    Mb, logMb = _markov(rng, V)
    _, logMs = _markov(rng, V)
    seqs, _ = _speculate(logMb, logMs, S, L, K, N, seed=11, strong=strong, min_first=min_first)
    Mb32 = np.exp(logMb.astype(np.float64))
    Mb32 /= Mb32.sum(axis=1, keepdims=True)
    expected = np.zeros(V ** N)
    for code in range(V ** N):
        y = [(code // V ** (N - 1 - t)) % V for t in range(N)]
        pr, prev = 1.0, 0
        for t in y:
            pr *= Mb32[prev, t]
            prev = t
        expected[code] = pr
    codes = (seqs * (V ** np.arange(N - 1, -1, -1))).sum(axis=1)
    counts = np.bincount(codes, minlength=V ** N)
    assert stats.chisquare(counts, expected * S).pvalue > 1e-4


@pytest.mark.parametrize("min_first", [False, True])
def test_first_token_is_algorithm_1_and_block_length_is_accepted_plus_one(min_first):
    rng = np.random.default_rng(5)
    S, K, V = 4000, 3, 12
    q = rng.normal(0, 2, (S, V)).astype(np.float32)
    p = (q + rng.normal(0, 1, (S, V))).astype(np.float32)
    one = oracle.couple(p, q, K, seed=21, min_first=min_first)  # rows 0..S-1
    target = np.repeat(np.repeat(q[:, None, None, :], 2, axis=1), K, axis=2)   # [S, 2, K, V]
    ver = oracle.verify(target, one["X"][:, None, :], seed=21, row_stride_s=1, row_stride_j=S, min_first=min_first)
    assert np.array_equal(ver["Y"][:, 0], one["Y"])
    np.testing.assert_array_equal(ver["key"][:, 0], one["keyY"])
    assert np.array_equal(ver["n_out"], 1 + one["accept"].astype(np.int32))
    assert np.array_equal(ver["active"], (one["X"] == one["Y"][:, None]).astype(np.uint8))
    assert ((ver["Y"][:, 1] >= 0) == (one["accept"] == 1)).all()


@pytest.mark.parametrize("min_first", [False, True])
def test_matches_a_pure_python_transcription_on_tiny_inputs(min_first):
    rng = np.random.default_rng(7)
    S, L, K, V = 60, 3, 3, 5
    target = rng.normal(0, 1.5, (S, L + 1, K, V)).astype(np.float32)
    tokens = rng.integers(0, V, (S, L, K)).astype(np.int32)
    # make acceptance likely: half of the draft tokens are replaced by what the verifier will pick
    seed = 31
    for strong in (False, True):
        ver = oracle.verify(target, tokens, seed=seed, temp_target=0.8, strong=strong, min_first=min_first)
        for s in range(S):
            viable = [True] * K
            Y = []
            for j in range(L + 1):
                row = s * (L + 1) + j
                times = gls_py.race_times(seed, row, K, V, min_first)
                best, arg = math.inf, -1
                kref = viable.index(True)
                for k in range(K):
                    if not (strong or viable[k]):
                        continue
                    z = target[s, j, k if viable[k] else kref].astype(np.float64) / np.float64(np.float32(0.8))
                    q = np.exp(z - z.max()) / np.exp(z - z.max()).sum()
                    for i in range(V):
                        key = times[k][i] / q[i]
                        if key < best or (key == best and i < arg):
                            best, arg = key, i
                Y.append(arg)
                if j == L:
                    break
                viable = [viable[k] and tokens[s, j, k] == arg for k in range(K)]
                if not any(viable):
                    break
            assert list(ver["Y"][s, :ver["n_out"][s]]) == Y
            assert ver["n_out"][s] == len(Y)
            assert (ver["Y"][s, len(Y):] == -1).all()


def test_strong_variant_ignores_the_draft_tokens():
    rng = np.random.default_rng(9)
    S, L, K, V = 500, 3, 4, 6
    q = rng.normal(0, 1, (S, L + 1, 1, V)).astype(np.float32)
    target = np.repeat(q, K, axis=2)                       # every draft row equals the same q^(j)
    tok_a = rng.integers(0, V, (S, L, K)).astype(np.int32)
    tok_b = rng.integers(0, V, (S, L, K)).astype(np.int32)
    a = oracle.verify(target, tok_a, seed=5, strong=True)
    b = oracle.verify(target, tok_b, seed=5, strong=True)
    n = np.minimum(a["n_out"], b["n_out"])
    for s in range(S):
        assert np.array_equal(a["Y"][s, :n[s]], b["Y"][s, :n[s]])
    # the conditional variant does depend on the tokens through the viable set
    c = oracle.verify(target, tok_a, seed=5)
    d = oracle.verify(target, tok_b, seed=5)
    assert np.array_equal(c["Y"][:, 0], d["Y"][:, 0])
    differ = sum(1 for s in range(S) if min(c["n_out"][s], d["n_out"][s]) > 1 and c["Y"][s, 1] != d["Y"][s, 1])
    assert differ > 0


def test_block_efficiency_grows_with_the_number_of_drafts():
    rng = np.random.default_rng(13)
    V, S, L = 8, 4000, 4
    Mb, logMb = _markov(rng, V, 0.5)
    logMs = (logMb + rng.normal(0, 0.5, logMb.shape)).astype(np.float32)
    eff = []
    for K in (1, 2, 4, 8):
        _, blocks = _speculate(logMb, logMs, S, L, K, 12, seed=17)
        eff.append(blocks)
    assert eff[0] >= eff[1] >= eff[2] >= eff[3] and eff[3] < eff[0]
