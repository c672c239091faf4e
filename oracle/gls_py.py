"""Algorithm 1 in pure Python for tiny inputs (test infrastructure).

A second, independent statement of the sampler used to pin the C++ oracle on
small cases: probabilities come in as Python floats (already normalised by the
caller), randomness from philox_py, and the three selections of Algorithm 1
are written with min() over explicit lists.
"""
import math

from . import philox_py


def race_times(seed, row, K, V, min_first=False):
    """S[k][i].  min_first: index i's K times are its smallest one, M = -ln(U0) / K, at draft
    kappa = floor(K r / 2^32), and M plus the per-(k, i) word's time at every other draft."""
    S = [[philox_py.race_time(philox_py.shared_word(seed, row, k, i)) for i in range(V)]
         for k in range(K)]
    if min_first:
        for i in range(V):
            M = philox_py.race_time(philox_py.aux_word(seed, row, i, 0)) / K
            kappa = (philox_py.aux_word(seed, row, i, 1) * K) >> 32
            for k in range(K):
                S[k][i] = M if k == kappa else M + S[k][i]
    return S


def sample_gls(p_list, q, seed, row, min_first=False):
    """p_list: K proposal distributions (lists of V floats); q: target distribution.

    Returns (X list of K indices, Y, accept).  Zero-probability entries never win.
    """
    K, V = len(p_list), len(q)
    S = race_times(seed, row, K, V, min_first)

    def argmin(keys):
        best, arg = math.inf, -1
        for i, key in enumerate(keys):
            if key < best:
                best, arg = key, i
        return arg, best

    # step 3: Y = argmin_i min_k S_i^(k) / q_i
    pooled = [min(S[k][i] for k in range(K)) / q[i] if q[i] > 0 else math.inf for i in range(V)]
    Y, keyY = argmin(pooled)
    # step 4: X^(k) = argmin_i S_i^(k) / p_i^(k)
    X, keyX = [], []
    for k in range(K):
        arg, best = argmin([S[k][i] / p_list[k][i] if p_list[k][i] > 0 else math.inf
                            for i in range(V)])
        X.append(arg)
        keyX.append(best)
    # step 5
    return X, Y, (Y in X), keyX, keyY
