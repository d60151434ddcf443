"""CORE-GD for non-convex objectives (Algorithm 3 of the paper, Section 5), fp64, CPU.

TEST INFRASTRUCTURE ONLY (see ``core_oracle.c``).

One iteration, in the algorithm's order:
  1. fresh xi_1..xi_m from the common generator (round counter k);
  2. machine i forms p_ij = <grad f_i(x^k), xi_j>; the projections are combined over machines
     (as the mean, Eq. (tildefdef), because f is the average of the f_i, Eq. (problem));
  3. every machine reconstructs the estimator of grad f(x^k);
  4. the scalar p is formed from the combined projections (see ``norm_statistic``);
  5. the step size h_k: Option I uses p, Option II uses the constants L and Delta;
  6. trial point xt = x^k - h_k * estimator;
  7. comparison step: x^{k+1} is whichever of x^k, xt has the smaller f.

Readings taken where the printed algorithm cannot be followed literally:
  * The printed definition of p is a plain average of the summed projections, with the two
    indices exchanged.  A plain average of zero-mean Gaussians cannot bound the gradient norm,
    yet the proof of Theorem 5.1 (Option I) needs the event p >= 2 ||grad f(x^k)|| with
    probability 1 - delta/N when m > log(N/delta).  By the lemma on the law of the projections
    (p_j ~ N(0, ||a||^2), independent over j), (1/m) sum_j pbar_j^2 is an unbiased estimate of
    ||grad f||^2 that concentrates like chi^2_m / m, so the statistic here is
        p = c * sqrt((1/m) sum_j pbar_j^2)
    with a caller-chosen constant c >= 2 (c = 4 makes P(p < 2||grad f||) <= 0.53^(m/2)).
  * Ties in the comparison step keep x^k (the trial point is taken only if f strictly drops).
"""
from __future__ import annotations

import math

import numpy as np

from . import core_round


def norm_statistic(pbar, c):
    """p = c * sqrt(mean_j pbar_j^2): the gradient-norm estimate of Algorithm 3 (reading above)."""
    pbar = np.asarray(pbar, dtype=np.float64)
    return c * math.sqrt(float(np.mean(pbar * pbar)))


def step_size_option1(d, m, r1, H, p):
    """min{ m/(16 r1), (1/1600) H^(-1/2) p^(-1/2) d^(-3/4) m^(3/4) }  (Algorithm 3, Option I).
    p = 0 (zero gradient) leaves the first term."""
    first = m / (16.0 * r1)
    if p <= 0.0:
        return first
    second = (1.0 / 1600.0) * H ** -0.5 * p ** -0.5 * d ** -0.75 * m ** 0.75
    return min(first, second)


def step_size_option2(d, m, r1, H, L, Delta):
    """min{ m/(16 r1), (1/1600) H^(-1/2) (L Delta)^(-1/4) d^(-3/4) m^(3/4) }  (Option II)."""
    first = m / (16.0 * r1)
    second = (1.0 / 1600.0) * H ** -0.5 * (L * Delta) ** -0.25 * d ** -0.75 * m ** 0.75
    return min(first, second)


def comparison_step(f_cur, f_trial):
    """True when the trial point replaces the current one (strict decrease)."""
    return bool(f_trial < f_cur)


def core_gd_nonconvex(f, client_grads, x0, m, rounds, seed, *, option, r1, H, c=4.0, L=None,
                      Delta=None, first_round=0):
    """Run Algorithm 3.  ``f(x) -> float`` and ``client_grads(x) -> [n, d]`` are the caller's.
    Returns a dict with the final x and, per round, f(x^k), p, h_k and the accept flag."""
    x = np.array(x0, dtype=np.float64)
    d = x.shape[0]
    fx = f(x)
    hist = {"f": [fx], "p": [], "h": [], "accepted": [], "f_trial": []}
    for k in range(rounds):
        G = np.asarray(client_grads(x), dtype=np.float64)
        _, pbar, gtilde = core_round(seed, first_round + k, G, m)
        p = norm_statistic(pbar, c)
        if option == 1:
            h = step_size_option1(d, m, r1, H, p)
        elif option == 2:
            h = step_size_option2(d, m, r1, H, L, Delta)
        else:
            raise ValueError("option must be 1 or 2")
        xt = x - h * gtilde
        ft = f(xt)
        take = comparison_step(fx, ft)
        if take:
            x, fx = xt, ft
        hist["p"].append(p)
        hist["h"].append(h)
        hist["accepted"].append(take)
        hist["f_trial"].append(ft)
        hist["f"].append(fx)
    hist["x"] = x
    return hist


# ---- a non-convex test objective with bounded Hessian trace (robust regression) ----------------
# f(x) = (1/N) sum_i phi(a_i^T x - b_i),  phi(t) = t^2 / (1 + t^2);  machine c owns a contiguous
# block of N/n rows and f_c is the mean of phi over its rows, so f = (1/n) sum_c f_c.
# phi'(t) = 2t/(1+t^2)^2, phi''(t) = (2 - 6t^2)/(1+t^2)^3 in [-1/2, 2], |phi'''| <= 4.67.

def robust_loss(A, b, x):
    t = A @ x - b
    return float(np.mean(t * t / (1.0 + t * t)))


def robust_client_gradients(A, b, x, n):
    rows = A.shape[0] // n
    G = np.empty((n, A.shape[1]), dtype=np.float64)
    for c in range(n):
        Ac, bc = A[c * rows:(c + 1) * rows], b[c * rows:(c + 1) * rows]
        t = Ac @ x - bc
        G[c] = Ac.T @ (2.0 * t / (1.0 + t * t) ** 2) / rows
    return G


def robust_constants(A):
    """Upper bounds (r1, L, H) for the robust-regression objective above:
    tr Hess <= 2 mean||a_i||^2, L <= 2 lambda_max(A^T A / N),
    third derivative <= 4.67 max||a_i|| lambda_max(A^T A / N)."""
    N = A.shape[0]
    lam_max = float(np.linalg.eigvalsh(A.T @ A / N)[-1])
    row2 = np.sum(A * A, axis=1)
    return 2.0 * float(row2.mean()), 2.0 * lam_max, 4.67 * math.sqrt(float(row2.max())) * lam_max
