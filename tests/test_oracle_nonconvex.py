"""Pins for the oracle's Algorithm 3 (CORE-GD for non-convex objectives, Section 5).

What fixes each piece independently of the oracle's own code:
  * the statistic p: by the lemma on the law of the projections, m (p/c)^2 / ||a||^2 is
    chi-square with m degrees of freedom -> its mean, variance and the exact probability of the
    event p < 2||a|| (scipy's chi-square CDF);
  * the step sizes: values worked out by hand for powers of two/sixteen, and the two
    inequalities of the proof of Theorem 5.1 that the step must satisfy once p >= 2||grad f||;
  * the test objective: finite differences, and its constants against sampled Hessians;
  * the loop: the comparison step's guarantees (f never rises, the iterate is the trial point
    exactly when f strictly dropped), a round replayed by hand from the round primitive, and
    the expected-descent inequality of Theorem 5.1 (Option II) by Monte Carlo.
"""
import math

import numpy as np
from scipy import stats

import oracle
from oracle import nonconvex as nc


def test_statistic_follows_the_chi_square_law():
    rng = np.random.default_rng(0)
    d, m, c, S = 64, 4, 2.5, 6000
    a = rng.standard_normal(d) * np.linspace(0.1, 2.0, d)
    na2 = float(a @ a)
    ratio = np.empty(S)
    for s in range(S):
        pbar = oracle.compress(900 + s, s % 7, a[None, :], m)[0]
        ratio[s] = (nc.norm_statistic(pbar, c) / c) ** 2 / na2
    assert abs(ratio.mean() - 1.0) < 4.5 * math.sqrt(2.0 / m / S)           # unbiased for ||a||^2
    assert abs(ratio.var() - 2.0 / m) < 0.08 * 2.0 / m + 0.02               # chi^2_m / m variance
    below = np.mean(c * np.sqrt(ratio) < 2.0)                                # event p < 2||a||
    exact = stats.chi2.cdf(m * 4.0 / c ** 2, m)
    assert abs(below - exact) < 4.5 * math.sqrt(exact * (1 - exact) / S)
    # scaling and sign conventions
    pbar = np.array([3.0, -4.0])
    assert nc.norm_statistic(pbar, 1.0) == math.sqrt(12.5)
    assert nc.norm_statistic(-pbar, 2.0) == 2.0 * math.sqrt(12.5)
    assert nc.norm_statistic(np.zeros(5), 4.0) == 0.0


def test_step_sizes_by_hand():
    big = 1e-9   # r1 so small that the first term never binds
    # d = m: the dimension factors cancel
    assert math.isclose(nc.step_size_option1(16, 16, big, 1.0, 1.0), 1 / 1600, rel_tol=1e-15)
    # d^(-3/4): 16^(-3/4) = 1/8 ; m^(3/4): 16^(3/4) = 8
    assert math.isclose(nc.step_size_option1(16, 1, big, 1.0, 1.0), 1 / 12800, rel_tol=1e-15)
    assert math.isclose(nc.step_size_option1(1, 16, big, 1.0, 1.0), 1 / 200, rel_tol=1e-15)
    # H^(-1/2), p^(-1/2)
    assert math.isclose(nc.step_size_option1(16, 16, big, 4.0, 1.0), 1 / 3200, rel_tol=1e-15)
    assert math.isclose(nc.step_size_option1(16, 16, big, 1.0, 4.0), 1 / 3200, rel_tol=1e-15)
    # first term m / (16 r1), and p = 0
    assert nc.step_size_option1(16, 8, 1e6, 1.0, 1.0) == 8 / 16e6
    assert nc.step_size_option1(16, 8, 2.0, 1.0, 0.0) == 0.25
    # Option II: (L Delta)^(-1/4): 16^(-1/4) = 1/2
    assert math.isclose(nc.step_size_option2(16, 16, big, 1.0, 2.0, 8.0), 1 / 3200, rel_tol=1e-15)
    assert math.isclose(nc.step_size_option2(16, 1, big, 4.0, 1.0, 1.0), 1 / 25600, rel_tol=1e-15)
    assert nc.step_size_option2(16, 8, 1e6, 1.0, 1.0, 1.0) == 8 / 16e6


def test_step_sizes_satisfy_the_inequalities_of_the_proof():
    rng = np.random.default_rng(1)
    for _ in range(200):
        d = int(rng.integers(4, 10 ** 6))
        m = int(rng.integers(1, d + 1))
        r1, H = 10 ** rng.uniform(-3, 3), 10 ** rng.uniform(-3, 3)
        gnorm = 10 ** rng.uniform(-4, 2)
        p = gnorm * rng.uniform(2.0, 10.0)                 # the event of Option I
        h = nc.step_size_option1(d, m, r1, H, p)
        assert 3 * h * h * r1 / (2 * m) * gnorm ** 2 <= 0.25 * h * gnorm ** 2 * (1 + 1e-12)
        assert 800 * H * h ** 3 * d ** 1.5 / (3 * m ** 1.5) * gnorm ** 3 <= 0.25 * h * gnorm ** 2 * (1 + 1e-12)
        # Option II: ||grad f||^2 <= 2 L (f - f*) <= 2 L Delta for an L-smooth f
        L, Delta = 10 ** rng.uniform(-2, 2), 10 ** rng.uniform(-2, 2)
        g2 = math.sqrt(2 * L * Delta) * rng.uniform(0.0, 1.0)
        h2 = nc.step_size_option2(d, m, r1, H, L, Delta)
        assert 3 * h2 * h2 * r1 / (2 * m) <= 0.25 * h2 * (1 + 1e-12)
        assert 800 * H * h2 ** 3 * d ** 1.5 / (3 * m ** 1.5) * g2 ** 3 <= 0.25 * h2 * g2 ** 2 * (1 + 1e-12)


def _robust_problem(N=96, d=24, n=4, seed=3):
    rng = np.random.default_rng(seed)
    A = rng.standard_normal((N, d)) / math.sqrt(d)
    x_true = rng.standard_normal(d)
    b = A @ x_true + 0.1 * rng.standard_normal(N)
    b[::7] += 5.0                                           # outliers: the loss is non-convex there
    return A, b, n


def test_robust_objective_gradients_and_constants():
    A, b, n = _robust_problem()
    N, d = A.shape
    rng = np.random.default_rng(4)
    r1, L, H = nc.robust_constants(A)
    neg_curv = False
    for trial in range(6):
        x = rng.standard_normal(d) * 2.0
        G = nc.robust_client_gradients(A, b, x, n)
        g = G.mean(axis=0)
        eps = 1e-6
        fd = np.array([(nc.robust_loss(A, b, x + eps * e) - nc.robust_loss(A, b, x - eps * e)) / (2 * eps)
                       for e in np.eye(d)])
        np.testing.assert_allclose(g, fd, rtol=1e-6, atol=1e-9)
        # Hessian by finite differences of the gradient
        Hm = np.array([(nc.robust_client_gradients(A, b, x + eps * e, n).mean(axis=0)
                        - nc.robust_client_gradients(A, b, x - eps * e, n).mean(axis=0)) / (2 * eps)
                       for e in np.eye(d)])
        ev = np.linalg.eigvalsh(0.5 * (Hm + Hm.T))
        assert np.trace(Hm) <= r1 and max(abs(ev[0]), abs(ev[-1])) <= L
        neg_curv |= ev[0] < -1e-3
        # Lipschitz Hessian along a random direction
        u = rng.standard_normal(d)
        u /= np.linalg.norm(u)
        t = 1e-3
        Hm2 = np.array([(nc.robust_client_gradients(A, b, x + t * u + eps * e, n).mean(axis=0)
                         - nc.robust_client_gradients(A, b, x + t * u - eps * e, n).mean(axis=0)) / (2 * eps)
                        for e in np.eye(d)])
        assert np.linalg.norm(Hm2 - Hm, 2) <= H * t * 1.01 + 1e-6
    assert neg_curv, "the test objective should be non-convex somewhere on the sampled points"


def test_loop_guarantees_and_a_round_replayed_by_hand():
    A, b, n = _robust_problem()
    d = A.shape[1]
    r1, L, H = nc.robust_constants(A)
    f = lambda x: nc.robust_loss(A, b, x)
    grads = lambda x: nc.robust_client_gradients(A, b, x, n)
    x0 = np.zeros(d)
    m = 8
    # the paper's constants make the steps tiny; a smaller H constant exercises both branches of
    # the comparison step without changing the code path
    for option, Hc in ((1, H), (1, 1e-9), (2, 1e-9)):
        out = nc.core_gd_nonconvex(f, grads, x0, m, 60, 21, option=option, r1=r1 * 1e-3, H=Hc,
                                   L=L, Delta=f(x0), c=4.0)
        fs = np.array(out["f"])
        assert np.all(np.diff(fs) <= 0.0)
        for k, took in enumerate(out["accepted"]):
            assert took == (out["f_trial"][k] < fs[k])
            assert fs[k + 1] == (out["f_trial"][k] if took else fs[k])
        assert f(out["x"]) == fs[-1]
    # replay round 0 of an Option I run from the primitives
    out = nc.core_gd_nonconvex(f, grads, x0, m, 1, 21, option=1, r1=r1, H=H, c=3.0)
    G = grads(x0)
    P = np.array([[float(G[c] @ oracle.xi_range(21, 0, j, 0, d)) for j in range(m)] for c in range(n)])
    pbar = P.mean(axis=0)
    p = 3.0 * math.sqrt(float(np.mean(pbar ** 2)))
    h = min(m / (16 * r1), H ** -0.5 * p ** -0.5 * (m / d) ** 0.75 / 1600)
    gt = sum(pbar[j] * oracle.xi_range(21, 0, j, 0, d) for j in range(m)) / m
    xt = x0 - h * gt
    assert math.isclose(out["p"][0], p, rel_tol=1e-12) and math.isclose(out["h"][0], h, rel_tol=1e-12)
    assert math.isclose(out["f_trial"][0], f(xt), rel_tol=1e-12)
    np.testing.assert_allclose(out["x"], xt if f(xt) < f(x0) else x0, rtol=1e-12, atol=1e-15)


def test_ties_keep_the_current_point_and_every_round_draws_fresh_vectors():
    assert nc.comparison_step(1.0, 1.0) is False
    assert nc.comparison_step(1.0, float("nan")) is False and nc.comparison_step(float("nan"), 0.0) is False
    assert nc.comparison_step(1.0, np.nextafter(1.0, 0.0)) is True
    A, b, n = _robust_problem()
    d = A.shape[1]
    grads = lambda x: nc.robust_client_gradients(A, b, x, n)
    x0 = np.full(d, 0.25)
    # a constant objective: the trial point never strictly improves, so x never moves
    out = nc.core_gd_nonconvex(lambda x: 1.0, grads, x0, 4, 6, 9, option=2, r1=0.5, H=1e-9, L=1.0, Delta=1.0)
    assert not any(out["accepted"]) and np.array_equal(out["x"], x0)
    # with x fixed the gradients are fixed, so p changes from round to round only through the
    # fresh vectors: round k must use counter first_round + k
    m, c, first = 4, 2.0, 17
    assert len(set(out["p"])) == len(out["p"])
    G = grads(x0)
    out = nc.core_gd_nonconvex(lambda x: 1.0, grads, x0, m, 3, 9, option=1, r1=0.5, H=1e-9, c=c, first_round=first)
    for k in range(3):
        pbar = np.array([np.mean([G[i] @ oracle.xi_range(9, first + k, j, 0, d) for i in range(n)]) for j in range(m)])
        assert math.isclose(out["p"][k], c * math.sqrt(float(np.mean(pbar ** 2))), rel_tol=1e-12)


def test_both_branches_of_the_comparison_step_occur():
    A, b, n = _robust_problem()
    d = A.shape[1]
    r1, L, H = nc.robust_constants(A)
    f = lambda x: nc.robust_loss(A, b, x)
    grads = lambda x: nc.robust_client_gradients(A, b, x, n)
    # a step far above the theorem's makes some trial points worse: they must be rejected
    # (r1 = m/48 makes the first term of the step equal to 3, about 1/(2L) here, with d/m = 12)
    out = nc.core_gd_nonconvex(f, grads, np.zeros(d), 2, 80, 5, option=2, r1=2 / 16.0 / 3.0, H=1e-12,
                               L=L, Delta=1e-6)
    acc = np.array(out["accepted"])
    assert acc.any() and (~acc).any()
    assert np.all(np.diff(out["f"]) <= 0.0)


def test_theorem_descent_in_expectation_option2():
    A, b, n = _robust_problem()
    d = A.shape[1]
    r1, L, H = nc.robust_constants(A)
    f = lambda x: nc.robust_loss(A, b, x)
    grads = lambda x: nc.robust_client_gradients(A, b, x, n)
    rng = np.random.default_rng(6)
    x0 = rng.standard_normal(d)
    Delta = f(x0)                      # f >= 0
    m, K, S = 8, 5, 300
    h = nc.step_size_option2(d, m, r1, H, L, Delta)
    lhs = np.empty(S)                  # f(x^K) + sum_i h/2 ||grad f(x^i)||^2 - f(x^0), expected <= 0
    for s in range(S):
        x = x0.copy()
        acc = 0.0
        for k in range(K):
            g = grads(x).mean(axis=0)
            acc += 0.5 * h * float(g @ g)
            out = nc.core_gd_nonconvex(f, grads, x, m, 1, 3000 + s, option=2, r1=r1, H=H, L=L,
                                       Delta=Delta, first_round=k)
            assert out["h"][0] == h
            x = out["x"]
        lhs[s] = f(x) + acc - f(x0)
    assert lhs.mean() <= 4.5 * lhs.std() / math.sqrt(S)
    assert lhs.mean() < 0.0 or abs(lhs.mean()) < 4.5 * lhs.std() / math.sqrt(S)
