"""The list-decoding compression scheme on the synthetic Gaussian source (test infrastructure).

Section 5.1 (coding scheme), Appendix C (importance-sampling form) and Appendix D.2 (Gaussian
source: decoder target distribution, MMSE estimator, experiment parameters), written out step by
step on top of the oracle's index selection (oracle.compress_select).  Used to pin the oracle against
the distortion figures the paper tabulates for this source.

Per trial:  A ~ N(0,1);  T_k = A + N(0, s_z) for each of the K decoders;  N candidates
U_i ~ p_W = N(0, 1 + s_e) and bins l_i uniform on {0..Lmax-1} (common randomness);  the encoder
draws Y with weights p_{W|A}(U_i|a) / p_W(U_i), sends M = l_Y;  decoder k draws X^(k) with weights
p_{W|T}(U_i|t_k) 1{l_i = M} / p_W(U_i), outputs W_k = U_{X^(k)} and the MMSE estimate
g(W_k, T_k);  the trial's distortion is the smallest squared error among the decoders.
"""
import numpy as np

import oracle


def _log_normal(u, mean, var):
    return -0.5 * np.log(2.0 * np.pi * var) - 0.5 * (u - mean) ** 2 / var


def gaussian_trials(n_trials, K, l_max, var_w_given_a, *, N=1 << 15, var_t_given_a=0.5, seed=0,
                    shared_randomness=False, rng_seed=0, chunk=512):
    """Run the scheme; returns dict(distortion_db, mse, match_rate, encoder_index_error).

    shared_randomness=True is the paper's baseline: every decoder uses the same set of race
    times (and the encoder's pool is that one set).
    """
    s_e, s_z = float(var_w_given_a), float(var_t_given_a)
    var_w = 1.0 + s_e
    var_t = 1.0 + s_z
    var_w_given_t = var_w - 1.0 / var_t              # Appendix D.2, decoder target distribution
    denom = s_e + s_z + s_e * s_z                      # Appendix D.2, MMSE estimator
    rng = np.random.default_rng(rng_seed)
    sq_err = np.empty(n_trials)
    matched = np.empty(n_trials, bool)
    done = 0
    while done < n_trials:
        n = min(chunk, n_trials - done)
        a = rng.standard_normal(n)
        t = a[:, None] + np.sqrt(s_z) * rng.standard_normal((n, K))
        u = np.sqrt(var_w) * rng.standard_normal((n, N))
        bins = rng.integers(0, l_max, size=(n, N))
        log_pw = _log_normal(u, 0.0, var_w)
        enc = (_log_normal(u, a[:, None], s_e) - log_pw).astype(np.float32)
        dec_full = np.stack([_log_normal(u, t[:, k:k + 1] / var_t, var_w_given_t) - log_pw
                             for k in range(K)], axis=1).astype(np.float32)          # [n, K, N]
        rows = done
        bins8 = bins.astype(np.uint8)
        if not shared_randomness:
            sel = oracle.compress_select(enc, dec_full, bins8, seed=seed, row_offset=rows)
            y, x = sel["Y"], sel["X"]
        else:
            # baseline: one set of race times for the encoder and for every decoder
            per_dec = [oracle.compress_select(enc, np.ascontiguousarray(dec_full[:, k:k + 1]), bins8,
                                              seed=seed, row_offset=rows) for k in range(K)]
            y = per_dec[0]["Y"]
            x = np.stack([r["X"][:, 0] for r in per_dec], axis=1)
        w = np.take_along_axis(u, x.astype(np.int64), 1)                             # [n, K]
        a_hat = (s_z * w + s_e * t) / denom
        sq_err[done:done + n] = ((a_hat - a[:, None]) ** 2).min(axis=1)
        matched[done:done + n] = (x == y[:, None]).any(axis=1)
        done += n
    mse = float(sq_err.mean())
    return {"distortion_db": 10.0 * np.log10(mse), "mse": mse, "match_rate": float(matched.mean()),
            "se_db": float(10.0 / np.log(10.0) * sq_err.std(ddof=1) / np.sqrt(n_trials) / mse)}
