"""Pins for the oracle's binned index selection and the Gaussian-source compression scheme (CPU only).

What fixes it: the selection with a single bin is the importance-weight form of Algorithm 1; with
bins it equals two plain selections around an explicit mask; the index-matching probability obeys
the bound of the error-probability proposition (Section 5.2); matched trials reach the closed-form
MMSE distortion of Appendix D.2; more decoders and more rate help, and independent race times per
decoder beat the shared-randomness baseline (Section 5.3's qualitative findings).

The distortion figures tabulated in Appendix D.2 are NOT used as a pin: with the parameters the
appendix states (N = 2^15, variance of T given A 0.5, the listed variances of W given A) the scheme
as written in Section 5.1 / Appendix C matches indices with probability 0.29 at one bit and 0.75 at
six bits for one decoder -- in line with the paper's own bound, which caps what the tabulated
distortions would require -- and lands 7 to 20 dB above the table.  Parity with that table is
unpinned.
"""
import numpy as np

import oracle
from oracle import compress


def _weights(rng, B, L, N):
    enc = rng.normal(0, 2, (B, N)).astype(np.float32)
    dec = (enc[:, None, :] + rng.normal(0, 1.5, (B, L, N))).astype(np.float32)
    return enc, dec


def test_single_bin_is_the_importance_weight_form():
    rng = np.random.default_rng(1)
    enc, dec = _weights(rng, 60, 3, 700)
    a = oracle.compress_select(enc, dec, np.zeros((60, 700), np.uint8), seed=5, row_offset=9)
    b = oracle.couple_is(enc, dec, seed=5, row_offset=9)
    for name in ("X", "Y", "accept", "match_k"):
        assert np.array_equal(a[name], b[name]), name
    np.testing.assert_allclose(a["keyX"], b["keyX"], rtol=1e-12)
    assert (a["message"] == 0).all()


def test_bins_equal_two_plain_selections_around_an_explicit_mask():
    rng = np.random.default_rng(2)
    B, L, N, l_max = 80, 4, 900, 8
    enc, dec = _weights(rng, B, L, N)
    bins = rng.integers(0, l_max, (B, N)).astype(np.uint8)
    got = oracle.compress_select(enc, dec, bins, seed=6, row_offset=1 << 33)
    y = oracle.couple_is(enc, dec, seed=6, row_offset=1 << 33)["Y"]          # Y ignores the decoders
    msg = np.take_along_axis(bins, y[:, None].astype(np.int64), 1)
    masked = np.where((bins == msg)[:, None, :], dec, -np.inf).astype(np.float32)
    ref = oracle.couple_is(enc, masked, seed=6, row_offset=1 << 33)
    assert np.array_equal(got["Y"], y) and np.array_equal(got["message"], msg[:, 0])
    for name in ("X", "accept", "match_k"):
        assert np.array_equal(got[name], ref[name]), name
    np.testing.assert_allclose(got["keyX"], ref["keyX"], rtol=1e-12)
    # every decoder answers inside the announced bin
    assert (np.take_along_axis(bins, got["X"].astype(np.int64), 1) == msg).all()


def _bound(K, l_max, s_e, s_z, n=200_000, seed=0):
    """Monte-Carlo value of E[(1 + 2^i / (K Lmax))^-1] with i the conditional information density."""
    rng = np.random.default_rng(seed)
    a = rng.standard_normal(n)
    w = a + np.sqrt(s_e) * rng.standard_normal(n)
    t = a + np.sqrt(s_z) * rng.standard_normal(n)
    var_wt = 1.0 + s_e - 1.0 / (1.0 + s_z)
    log_ratio = (-0.5 * np.log(s_e) - 0.5 * (w - a) ** 2 / s_e) - \
                (-0.5 * np.log(var_wt) - 0.5 * (w - t / (1.0 + s_z)) ** 2 / var_wt)
    return float(np.mean(1.0 / (1.0 + np.exp(log_ratio) / (K * l_max))))


def test_matching_probability_obeys_the_error_probability_bound():
    for K, l_max, s_e in ((1, 2, 0.05), (2, 4, 0.02), (4, 16, 0.01)):
        r = compress.gaussian_trials(1200, K, l_max, s_e, N=1 << 13, seed=11, rng_seed=K)
        bound = _bound(K, l_max, s_e, 0.5)
        assert r["match_rate"] >= bound - 0.04, (K, l_max, r["match_rate"], bound)
        assert r["match_rate"] <= min(1.0, 3.0 * bound + 0.2)      # and is not trivially 1


def test_matched_trials_reach_the_closed_form_mmse_distortion():
    s_e, s_z = 0.05, 0.5
    r = compress.gaussian_trials(1500, 1, 256, s_e, N=1 << 13, seed=12, rng_seed=3)
    assert r["match_rate"] > 0.95
    floor = s_e * s_z / (s_e + s_z + s_e * s_z)                     # Appendix D.2, error of the MMSE estimate
    # mismatches (a few dozen trials, and those with an atypical source) add their share times a
    # squared error of the order of the prior variance: at most three times it is allowed for
    assert 0.85 * floor < r["mse"] < floor + (1.0 - r["match_rate"]) * 3.0 + 0.15 * floor


def test_more_decoders_more_rate_and_independent_race_times_help():
    common = dict(N=1 << 12, seed=13, rng_seed=4)
    k1 = compress.gaussian_trials(1500, 1, 4, 0.02, **common)
    k4 = compress.gaussian_trials(1500, 4, 4, 0.02, **common)
    k4_more_rate = compress.gaussian_trials(1500, 4, 32, 0.02, **common)
    k4_shared = compress.gaussian_trials(1500, 4, 4, 0.02, shared_randomness=True, **common)
    assert k4["match_rate"] > k1["match_rate"] + 0.1
    assert k4_more_rate["match_rate"] > k4["match_rate"] + 0.05
    assert k4["match_rate"] > k4_shared["match_rate"] + 0.05
    assert k4["distortion_db"] < k1["distortion_db"] - 1.0
    assert k4["distortion_db"] < k4_shared["distortion_db"] - 0.5
