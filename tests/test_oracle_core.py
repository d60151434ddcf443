"""Pins for the oracle's compression / client mean / reconstruction.

Algorithm 1 and Eq. (reconstruction) (Section 3), Eq. (tildefdef) (Section 4),
Lemma 3.1 (unbiasedness), the proof of Lemma 3.2 (second moment, which gives an
equality before its last relaxation), and the lemma on the law of C(a) in the
differential-privacy appendix.
"""
import os

import numpy as np
import pytest
from scipy import stats

import oracle


def _dense_xi(seed, rnd, m, d):
    """Xi (m x d) assembled one entry at a time."""
    Xi = np.empty((m, d))
    for j in range(m):
        for i in range(d):
            Xi[j, i] = oracle.xi(seed, rnd, j, i)
    return Xi


def _read_cases(golden_dir):
    out = {}
    with open(os.path.join(golden_dir, "core_small_cases.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, *vals = line.split()
            out[name] = np.array([float(v) for v in vals])
    return out


def test_golden_case_A(golden_dir):
    g = _read_cases(golden_dir)
    G = np.array([np.arange(1.0, 9.0), np.arange(8.0, 0.0, -1.0)])
    P, pbar, gt = oracle.core_round(42, 0, G, 4)
    np.testing.assert_allclose(P[0], g["A.P0"], rtol=0, atol=1e-9)
    np.testing.assert_allclose(P[1], g["A.P1"], rtol=0, atol=1e-9)
    np.testing.assert_allclose(pbar, g["A.pbar"], rtol=0, atol=1e-9)
    np.testing.assert_allclose(gt, g["A.gtilde"], rtol=0, atol=1e-9)
    # the separate entry points agree with the fused one
    P2 = oracle.compress(42, 0, G, 4)
    np.testing.assert_array_equal(P2, P)
    np.testing.assert_array_equal(oracle.client_mean(P2), pbar)
    np.testing.assert_array_equal(oracle.reconstruct(42, 0, pbar, 0.25, 0, 8), gt)


def test_golden_case_B_ragged_tail(golden_dir):
    g = _read_cases(golden_dir)
    a = np.array([[1.0, -2.0, 3.0, -4.0, 5.0]])
    P, pbar, gt = oracle.core_round(42, 0, a, 2)
    np.testing.assert_allclose(P[0], g["B.p"], rtol=0, atol=1e-9)
    np.testing.assert_allclose(pbar, g["B.p"], rtol=0, atol=1e-9)
    np.testing.assert_allclose(gt, g["B.gtilde"], rtol=0, atol=1e-9)


@pytest.mark.parametrize("d,m,n", [(1, 1, 1), (3, 2, 1), (4, 5, 2), (7, 3, 4), (8, 8, 3), (13, 4, 2)])
def test_brute_force_small(d, m, n):
    """p = Xi a and a~ = Xi^T p / m with numpy's dense products on an entry-by-entry Xi."""
    seed, rnd = 1234 + d, 3 * m + n
    rng = np.random.default_rng(100 * d + 10 * m + n)
    G = rng.standard_normal((n, d))
    Xi = _dense_xi(seed, rnd, m, d)
    P_ref = G @ Xi.T
    pbar_ref = P_ref.mean(axis=0)
    gt_ref = Xi.T @ pbar_ref / m
    P, pbar, gt = oracle.core_round(seed, rnd, G, m)
    np.testing.assert_allclose(P, P_ref, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(pbar, pbar_ref, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(gt, gt_ref, rtol=1e-13, atol=1e-13)


def test_single_vector_special_case():
    """n = m = 1: the scalar <a, xi> times xi (first paragraph of Section 3)."""
    a = np.array([[0.5, -1.5, 2.0, 0.25, 3.0, -0.75]])
    xi = oracle.xi_range(77, 4, 0, 0, 6)
    P, pbar, gt = oracle.core_round(77, 4, a, 1)
    s = float(a[0] @ xi)
    assert abs(P[0, 0] - s) < 1e-14 and abs(pbar[0] - s) < 1e-14
    np.testing.assert_allclose(gt, s * xi, rtol=1e-14, atol=1e-14)


def test_input_dtypes_are_taken_as_stored():
    rng = np.random.default_rng(5)
    G32 = rng.standard_normal((3, 37)).astype(np.float32)
    P64 = oracle.compress(9, 1, G32.astype(np.float64), 6)
    P32 = oracle.compress(9, 1, G32, 6)
    np.testing.assert_array_equal(P32, P64)
    # bf16 bit patterns: the upper half of the fp32 word, widened exactly
    bits = (G32.view(np.uint32) >> 16).astype(np.uint16)
    widened = (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    Pb = oracle.compress(9, 1, bits, 6)
    np.testing.assert_array_equal(Pb, oracle.compress(9, 1, widened, 6))


def test_column_subset_and_coordinate_ranges():
    rng = np.random.default_rng(6)
    G = rng.standard_normal((2, 50))
    P = oracle.compress(21, 8, G, 12)
    sub = oracle.compress(21, 8, G, jidx=[11, 0, 5])
    np.testing.assert_array_equal(sub, P[:, [11, 0, 5]])
    pbar = oracle.client_mean(P)
    full = oracle.reconstruct(21, 8, pbar, 1.0 / 12, 0, 50)
    np.testing.assert_array_equal(oracle.reconstruct(21, 8, pbar, 1.0 / 12, 7, 22), full[7:29])
    np.testing.assert_array_equal(oracle.reconstruct(21, 8, pbar, 1.0 / 12, 48, 2), full[48:50])


def test_linearity_and_client_mean_commute():
    """a -> p and p -> a~ are linear; the round on n clients equals CORE of the mean gradient."""
    rng = np.random.default_rng(7)
    d, m, n = 29, 6, 5
    G = rng.standard_normal((n, d))
    H = rng.standard_normal((n, d))
    P1 = oracle.compress(3, 2, G, m)
    P2 = oracle.compress(3, 2, H, m)
    P12 = oracle.compress(3, 2, 2.0 * G - 3.0 * H, m)
    np.testing.assert_allclose(P12, 2.0 * P1 - 3.0 * P2, rtol=1e-12, atol=1e-12)
    _, pbar, gt = oracle.core_round(3, 2, G, m)
    Pm, pbar_m, gt_m = oracle.core_round(3, 2, G.mean(axis=0, keepdims=True), m)
    np.testing.assert_allclose(pbar_m, pbar, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(gt_m, gt, rtol=1e-12, atol=1e-12)
    r1 = oracle.reconstruct(3, 2, P1[0], 1.0 / m, 0, d)
    r2 = oracle.reconstruct(3, 2, P2[0], 1.0 / m, 0, d)
    r12 = oracle.reconstruct(3, 2, P1[0] + 0.5 * P2[0], 1.0 / m, 0, d)
    np.testing.assert_allclose(r12, r1 + 0.5 * r2, rtol=1e-12, atol=1e-12)
    # scale n/m on the mean is the Algorithm-2 form (sum over machines)
    rn = oracle.reconstruct(3, 2, pbar, n / m, 0, d)
    np.testing.assert_allclose(rn, n * gt, rtol=1e-12, atol=1e-12)


def test_fresh_vectors_each_round():
    a = np.ones((1, 16))
    p0 = oracle.compress(1, 0, a, 4)
    p1 = oracle.compress(1, 1, a, 4)
    assert np.abs(p0 - p1).min() > 1e-6
    np.testing.assert_array_equal(p0, oracle.compress(1, 0, a, 4))


def _estimates(a, m, seeds):
    d = a.shape[0]
    out = np.empty((len(seeds), d))
    for t, s in enumerate(seeds):
        _, _, gt = oracle.core_round(int(s), 0, a[None, :], m)
        out[t] = gt
    return out


def test_lemma_unbiased():
    """Lemma 3.1: E a~ = a.  Per-coordinate variance (|a|^2 + a_i^2)/m follows from
    E[xi xi^T A xi xi^T] = tr(A) I + 2A (proof of Lemma 3.2) with A = e_i e_i^T."""
    rng = np.random.default_rng(8)
    d, m, S = 12, 3, 40000
    a = rng.standard_normal(d) * np.linspace(0.2, 2.0, d)
    est = _estimates(a, m, np.arange(1000, 1000 + S))
    sd = np.sqrt((a @ a + a * a) / m / S)
    assert np.all(np.abs(est.mean(axis=0) - a) < 4.5 * sd)
    # the sample variance per coordinate matches the closed form too
    var_ref = (a @ a + a * a) / m
    assert np.all(np.abs(est.var(axis=0) / var_ref - 1.0) < 0.08)


def test_second_moment_identity():
    """E|a~ - a|^2_A = (tr(A)|a|^2 + |a|^2_A)/m; with A = I this is (d+1)|a|^2/m.
    (First display of the proof of Lemma 3.2 combined with E[xi xi^T A xi xi^T] = tr(A) I + 2A.)"""
    rng = np.random.default_rng(9)
    d, m, S = 8, 4, 40000
    a = rng.standard_normal(d)
    est = _estimates(a, m, np.arange(5000, 5000 + S))
    err = est - a
    sq = (err ** 2).sum(axis=1)
    expected = (d + 1) * (a @ a) / m
    assert abs(sq.mean() - expected) < 4.5 * sq.std() / np.sqrt(S)
    # and it is well inside the bound the lemma states: 3 tr(A)|a|^2/m - |a|^2_A/m
    assert sq.mean() < (3 * d - 1) * (a @ a) / m
    B = rng.standard_normal((d, d))
    A = B @ B.T
    sqA = np.einsum("si,ij,sj->s", err, A, err)
    expectedA = (np.trace(A) * (a @ a) + a @ A @ a) / m
    assert abs(sqA.mean() - expectedA) < 4.5 * sqA.std() / np.sqrt(S)
    assert sqA.mean() < 3 * np.trace(A) * (a @ a) / m - (a @ A @ a) / m


def test_second_moment_scales_as_one_over_m():
    rng = np.random.default_rng(10)
    d, S = 6, 20000
    a = rng.standard_normal(d)
    for m in (1, 2, 8):
        est = _estimates(a, m, np.arange(90000, 90000 + S))
        sq = ((est - a) ** 2).sum(axis=1)
        assert abs(sq.mean() - (d + 1) * (a @ a) / m) < 4.5 * sq.std() / np.sqrt(S)


def test_compression_law():
    """C(a) ~ N(0, |a|^2 I_m) (lemma on the law of C(a), privacy appendix)."""
    rng = np.random.default_rng(11)
    d, m, S = 40, 8, 6000
    a = rng.standard_normal(d)
    P = np.empty((S, m))
    for s in range(S):
        P[s] = oracle.compress(s + 1, 7, a[None, :], m)[0]
    Z = P / np.linalg.norm(a)
    assert stats.kstest(Z.ravel(), "norm").pvalue > 1e-3
    C = Z.T @ Z / S
    assert np.abs(C - np.eye(m)).max() < 5.0 * np.sqrt(2.0 / S)
    chi = (Z ** 2).sum(axis=1)
    assert stats.kstest(chi, "chi2", args=(m,)).pvalue > 1e-3


def test_large_m_recovers_the_vector():
    """(1/m) Xi^T Xi -> I: with m large the reconstruction error shrinks like sqrt((d+1)/m)."""
    rng = np.random.default_rng(12)
    d, m = 4, 40000
    a = rng.standard_normal((1, d))
    _, _, gt = oracle.core_round(17, 0, a, m)
    rel = np.linalg.norm(gt - a[0]) / np.linalg.norm(a[0])
    assert rel < 4.0 * np.sqrt((d + 1) / m)


def test_bad_arguments_raise():
    with pytest.raises(ValueError):
        oracle.reconstruct(1, 0, np.zeros(0), 1.0, 0, 4)
    with pytest.raises(TypeError):
        oracle.compress(1, 0, np.zeros((1, 4), dtype=np.int32), 2)
