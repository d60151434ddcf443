"""Pins for the oracle's diagnostics (appendix on differential privacy).

What fixes each piece independently of the oracle's own code:
  * squared norms: integer inputs whose sums of squares are known exactly, one row at a time
    (a transposed or shared accumulator fails), and numpy's norm routine;
  * the lemma on the law of C(a): for a fixed gradient a, ||C(a)||^2 / ||a||^2 over fresh common
    randomness is chi-square with m degrees of freedom (mean, variance, Kolmogorov-Smirnov
    against scipy's CDF) -- this ties the projection oracle to the statistic;
  * the privacy loss: scipy's normal log-density (a library routine the oracle does not call),
    the closed form the proof of the privacy theorem arrives at, antisymmetry, the value 0 for
    equal norms, and the Kullback-Leibler divergence of the two laws at ||p||^2 = m sigma1^2;
  * the library's host-arithmetic entry point against all of the above (no GPU needed).
"""
import ctypes
import math

import numpy as np
import pytest
from scipy import stats

import oracle
from oracle import diagnostics as dg


def test_squared_norms_exact_cases():
    P = np.array([[3.0, -4.0, 0.0], [1.0, 2.0, 2.0], [0.0, 0.0, 0.0], [-12.0, 5.0, 84.0]], dtype=np.float32)
    assert dg.projection_sqnorms(P).tolist() == [25.0, 9.0, 0.0, 7225.0]
    assert dg.projection_sqnorms(-P).tolist() == [25.0, 9.0, 0.0, 7225.0]
    assert dg.projection_sqnorms(P.T.copy()).tolist() == [154.0, 45.0, 7060.0]   # rows, not columns
    rng = np.random.default_rng(3)
    Q = rng.standard_normal((5, 1000)).astype(np.float32)
    want = np.linalg.norm(Q.astype(np.float64), axis=1) ** 2
    assert np.allclose(dg.projection_sqnorms(Q), want, rtol=1e-13, atol=0)
    with pytest.raises(ValueError):
        dg.projection_sqnorms(np.zeros(4))


def test_projection_norm_follows_the_chi_square_law():
    rng = np.random.default_rng(11)
    d, m, S = 48, 6, 4000
    a = rng.standard_normal(d) * np.linspace(0.2, 3.0, d)
    na2 = float(a @ a)
    ratio = np.empty(S)
    for s in range(S):
        P = oracle.compress(7000 + s, s % 5, a[None, :], m)           # [1][m], one machine's message
        ratio[s] = dg.projection_sqnorms(P)[0] / na2                   # ~ chi^2_m
    assert abs(ratio.mean() - m) < 4.5 * math.sqrt(2.0 * m / S)
    assert abs(ratio.var() - 2.0 * m) < 0.1 * 2.0 * m
    assert stats.kstest(ratio, stats.chi2(m).cdf).pvalue > 1e-3


def _closed_form(sq, m, s1, s2):
    return 0.5 * sq * (1.0 / s2 ** 2 - 1.0 / s1 ** 2) + m * math.log(s2 / s1)


def test_privacy_loss_against_library_densities_and_the_closed_form():
    rng = np.random.default_rng(5)
    for m, s1, s2 in [(1, 1.0, 2.0), (7, 0.3, 0.31), (64, 5.0, 4.5), (500, 1e-3, 1.1e-3)]:
        p = rng.standard_normal(m) * s1
        want = stats.norm.logpdf(p, scale=s1).sum() - stats.norm.logpdf(p, scale=s2).sum()
        got = dg.privacy_loss(p, s1, s2)
        assert math.isclose(got, want, rel_tol=1e-10, abs_tol=1e-10)
        assert math.isclose(got, _closed_form(float(p @ p), m, s1, s2), rel_tol=1e-10, abs_tol=1e-10)
        assert math.isclose(dg.privacy_loss(p, s2, s1), -got, rel_tol=1e-12, abs_tol=1e-12)
        assert dg.privacy_loss(p, s1, s1) == 0.0
    # at ||p||^2 = m sigma1^2 (its mean under the first law) the loss is the KL divergence of the laws
    m, s1, s2 = 16, 2.0, 3.0
    p = np.full(m, s1)
    kl = m * (math.log(s2 / s1) + s1 ** 2 / (2 * s2 ** 2) - 0.5)
    assert math.isclose(dg.privacy_loss(p, s1, s2), kl, rel_tol=1e-13)
    assert kl > 0


def test_library_privacy_loss_matches_the_oracle():
    import paper_2309_13307_amd as core
    from paper_2309_13307_amd import binding
    rng = np.random.default_rng(9)
    for m, s1, s2 in [(1, 1.0, 2.0), (7, 0.3, 0.31), (64, 5.0, 4.5), (4096, 12.0, 12.5)]:
        p = (rng.standard_normal(m) * s1).astype(np.float32)
        sq = float(dg.projection_sqnorms(p[None, :])[0])
        assert math.isclose(core.core_privacy_loss(sq, m, s1, s2), dg.privacy_loss(p, s1, s2),
                            rel_tol=1e-10, abs_tol=1e-9)
    assert core.core_privacy_loss(0.0, 3, 2.0, 2.0) == 0.0
    L = core.load_library()
    out = ctypes.c_double(0.0)
    bad = binding.ERR_INVALID_ARGUMENT
    assert L.core_privacy_loss(1.0, 4, 1.0, 2.0, None) == bad
    assert L.core_privacy_loss(1.0, 0, 1.0, 2.0, ctypes.byref(out)) == bad
    assert L.core_privacy_loss(-1.0, 4, 1.0, 2.0, ctypes.byref(out)) == bad
    assert L.core_privacy_loss(1.0, 4, 0.0, 2.0, ctypes.byref(out)) == bad
    assert L.core_privacy_loss(1.0, 4, 1.0, float("nan"), ctypes.byref(out)) == bad
    assert L.core_privacy_loss(float("inf"), 4, 1.0, 2.0, ctypes.byref(out)) == bad
    assert L.core_privacy_loss(float("nan"), 4, 1.0, 2.0, ctypes.byref(out)) == bad
