"""Pins that run the oracle's round inside CORE-GD (Algorithm 2) on a tiny ridge problem.

Closed form x* = (A^T A + lam I)^-1 A^T b; the exact expected one-step change on a
quadratic (second-order expansion in the proof of Theorem 4.2, which is an equality
when f is quadratic, with the moments of Lemma 3.1 / proof of Lemma 3.2); and the
contraction factor of Theorem 4.2 in the regime it assumes (m <= tr(A)/L,
h = m / (4 tr(A))).
"""
import numpy as np

from oracle import coregd


def _problem(d=16, rows=32, n=4, lam=1e-2, seed=0, decay=1.0):
    rng = np.random.default_rng(seed)
    U, _ = np.linalg.qr(rng.standard_normal((rows, d)))
    V, _ = np.linalg.qr(rng.standard_normal((d, d)))
    s = np.arange(1, d + 1, dtype=np.float64) ** (-decay)
    A = (U * s) @ V.T
    x_true = rng.standard_normal(d)
    b = A @ x_true + 0.01 * rng.standard_normal(rows)
    return A, b, lam, n


def test_client_gradients_average_to_the_full_gradient():
    A, b, lam, n = _problem()
    x = np.random.default_rng(1).standard_normal(A.shape[1])
    G = coregd.client_gradients(A, b, lam, x, n)
    full = A.T @ (A @ x - b) + lam * x
    np.testing.assert_allclose(G.mean(axis=0), full, rtol=1e-12, atol=1e-12)
    xs = coregd.ridge_solution(A, b, lam)
    assert np.linalg.norm(A.T @ (A @ xs - b) + lam * xs) < 1e-12


def test_exact_one_step_expectation_on_a_quadratic():
    A, b, lam, n = _problem()
    d = A.shape[1]
    H = A.T @ A + lam * np.eye(d)
    x = np.random.default_rng(2).standard_normal(d)
    g = A.T @ (A @ x - b) + lam * x
    f0 = coregd.ridge_loss(A, b, lam, x)
    m, h, S = 4, 0.3, 20000
    expected = f0 - h * (g @ g) + 0.5 * h * h * ((1 + 1.0 / m) * (g @ H @ g)
                                                 + np.trace(H) * (g @ g) / m)
    vals = np.empty(S)
    for s in range(S):
        _, losses = coregd.core_gd(A, b, lam, n, m, h, 1, seed=100 + s, x0=x)
        vals[s] = losses[1]
    assert abs(vals.mean() - expected) < 4.5 * vals.std() / np.sqrt(S)


def test_theorem_contraction_in_its_regime():
    # flat-ish spectrum so that tr(H)/L is comfortably above m
    A, b, lam, n = _problem(decay=0.25)
    d = A.shape[1]
    H = A.T @ A + lam * np.eye(d)
    ev = np.linalg.eigvalsh(H)
    L, mu, trH = ev[-1], ev[0], ev.sum()
    m = 2
    assert m <= trH / L
    h = m / (4.0 * trH)
    rate = 1.0 - 3.0 * m * mu / (16.0 * trH)
    xs = coregd.ridge_solution(A, b, lam)
    fstar = coregd.ridge_loss(A, b, lam, xs)
    x0 = np.zeros(d)
    gap0 = coregd.ridge_loss(A, b, lam, x0) - fstar
    S, K = 400, 25
    gaps = np.empty((S, K + 1))
    for s in range(S):
        _, losses = coregd.core_gd(A, b, lam, n, m, h, K, seed=7000 + s, x0=x0)
        gaps[s] = losses - fstar
    mean_gap = gaps.mean(axis=0)
    sem = gaps.std(axis=0) / np.sqrt(S)
    for k in range(1, K + 1):
        assert mean_gap[k] <= rate ** k * gap0 + 4.5 * sem[k]
    assert mean_gap[K] < mean_gap[0]


def test_core_gd_reaches_the_closed_form_solution():
    A, b, lam, n = _problem(d=8, rows=16, lam=0.1)
    d = A.shape[1]
    H = A.T @ A + lam * np.eye(d)
    ev = np.linalg.eigvalsh(H)
    m = 8
    # the step the proof optimises before it specialises m <= tr(A)/L
    h = m / (3.0 * ev.sum() + 2.0 * m * ev[-1])
    xs = coregd.ridge_solution(A, b, lam)
    fstar = coregd.ridge_loss(A, b, lam, xs)
    x, losses = coregd.core_gd(A, b, lam, n, m, h, 600, seed=5)
    assert losses[-1] - fstar < 1e-6 * (losses[0] - fstar)
    assert np.linalg.norm(x - xs) < 1e-2 * np.linalg.norm(xs)


def test_core_agd_is_heavy_ball_with_the_estimated_gradient():
    """With a large budget m the estimator is nearly the gradient, so CORE-AGD must track the
    deterministic heavy-ball iteration it is built on, and reach the closed-form minimiser."""
    A, b, lam, n = _problem(d=6, rows=12, lam=0.05, decay=0.5)
    d = A.shape[1]
    H = A.T @ A + lam * np.eye(d)
    ev = np.linalg.eigvalsh(H)
    h = 1.0 / ev[-1]
    beta = np.sqrt(h * ev[0])
    xs = coregd.ridge_solution(A, b, lam)
    # deterministic heavy ball
    x = np.zeros(d); xp = x.copy(); traj = []
    for k in range(60):
        y = x + (1 - beta) * (x - xp)
        g = A.T @ (A @ y - b) + lam * y
        xp = x; x = y - h * g; traj.append(x.copy())
    m = 20000
    xc, losses = coregd.core_agd(A, b, lam, n, m, h, beta, 60, seed=3)
    assert np.linalg.norm(xc - traj[-1]) < 0.05 * np.linalg.norm(xs)
    assert np.linalg.norm(xc - xs) < 0.05 * np.linalg.norm(xs)
    assert losses[-1] < losses[0]
    # one step from a given (x, x_prev) pair: x1 = y - h * gtilde with y the extrapolated point
    from oracle import core_round
    x0 = np.arange(1.0, d + 1.0)
    G = coregd.client_gradients(A, b, lam, x0, n)   # x_prev = x0 on the first step, so y = x0
    _, _, gt = core_round(11, 0, G, 8)
    x1, _ = coregd.core_agd(A, b, lam, n, 8, 0.1, 0.3, 1, seed=11, x0=x0)
    np.testing.assert_allclose(x1, x0 - 0.1 * gt, rtol=1e-14, atol=1e-14)
    # second step uses y = x1 + (1-beta)(x1 - x0)
    y1 = x1 + 0.7 * (x1 - x0)
    G1 = coregd.client_gradients(A, b, lam, y1, n)
    _, _, gt1 = core_round(11, 1, G1, 8)
    x2, _ = coregd.core_agd(A, b, lam, n, 8, 0.1, 0.3, 2, seed=11, x0=x0)
    np.testing.assert_allclose(x2, y1 - 0.1 * gt1, rtol=1e-13, atol=1e-13)
    # third step: the momentum term is built from the two last iterates x2, x1 (not from y1)
    y2 = x2 + 0.7 * (x2 - x1)
    G2 = coregd.client_gradients(A, b, lam, y2, n)
    _, _, gt2 = core_round(11, 2, G2, 8)
    x3, _ = coregd.core_agd(A, b, lam, n, 8, 0.1, 0.3, 3, seed=11, x0=x0)
    np.testing.assert_allclose(x3, y2 - 0.1 * gt2, rtol=1e-13, atol=1e-13)


def test_decentralized_core_gd_reduces_to_the_centralized_one():
    """With enough gossip steps every machine holds the exact mean of the projections, and the
    decentralized iteration (reconstruction with n/m on the mean) is CORE-GD itself."""
    A, b, lam, n = _problem(d=8, rows=16, lam=0.1)
    d = A.shape[1]
    ev = np.linalg.eigvalsh(A.T @ A + lam * np.eye(d))
    m = 4
    h = m / (3.0 * ev.sum() + 2.0 * m * ev[-1])
    W = coregd.ring_gossip_matrix(n)
    np.testing.assert_allclose(W.sum(axis=0), 1.0)
    np.testing.assert_allclose(W, W.T)
    x_c, losses_c = coregd.core_gd(A, b, lam, n, m, h, 30, seed=9)
    X, losses_d = coregd.decentralized_core_gd(A, b, lam, n, m, h, 30, 9, W, gossip_steps=200)
    for c in range(n):
        np.testing.assert_allclose(X[c], x_c, rtol=1e-9, atol=1e-9)
    np.testing.assert_allclose(losses_d, losses_c, rtol=1e-9, atol=1e-12)
    # with few gossip steps the copies differ but still make progress
    X2, losses2 = coregd.decentralized_core_gd(A, b, lam, n, m, h, 30, 9, W, gossip_steps=2)
    assert np.abs(X2 - X2.mean(axis=0)).max() > 1e-6
    assert losses2[-1] < losses2[0]
    # two rounds with a single gossip step, replayed by hand: after round 0 the copies differ, and
    # in round 1 machine c must take its own gradient at its own copy
    from oracle import compress, reconstruct
    rows = A.shape[0] // n
    X1, _ = coregd.decentralized_core_gd(A, b, lam, n, m, h, 2, 9, W, gossip_steps=1)
    Xh = np.zeros((n, d))
    for k in range(2):
        G = np.stack([n * (A[c * rows:(c + 1) * rows].T @ (A[c * rows:(c + 1) * rows] @ Xh[c]
                                                         - b[c * rows:(c + 1) * rows])) + lam * Xh[c]
                      for c in range(n)])
        P = W @ compress(9, k, G, m)
        Xh = np.stack([Xh[c] - h * reconstruct(9, k, P[c], n / m, 0, d) / n for c in range(n)])
        if k == 0:
            assert np.abs(Xh - Xh.mean(axis=0)).max() > 1e-9
    np.testing.assert_allclose(X1, Xh, rtol=1e-12, atol=1e-14)
