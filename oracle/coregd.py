"""CORE-GD (Algorithm 2 of the paper) on a ridge-regression objective, fp64, CPU.

TEST INFRASTRUCTURE ONLY (see ``core_oracle.c``).

Objective (Eq. (problem), Section 1: f is the average of the machines' f_i):
    f(x)   = 1/2 ||A x - b||^2 + lam/2 ||x||^2
    f_c(x) = n/2 ||A_c x - b_c||^2 + lam/2 ||x||^2,   c = 1..n,  rows split over clients
so that f = (1/n) sum_c f_c and grad f_c = n A_c^T (A_c x - b_c) + lam x.

Each round follows Algorithm 2: fresh xi_1..xi_m from the common generator
(counter ``round = k``), machine c forms p_cj = <grad f_c(x^k), xi_j>, the
projections are combined over c (as the mean, Eq. (tildefdef)), every machine
reconstructs the estimator and steps x^{k+1} = x^k - h * estimator.
"""
from __future__ import annotations

import numpy as np

from . import core_round


def ridge_loss(A, b, lam, x):
    r = A @ x - b
    return 0.5 * float(r @ r) + 0.5 * lam * float(x @ x)


def ridge_solution(A, b, lam):
    """Closed form x* = (A^T A + lam I)^-1 A^T b."""
    d = A.shape[1]
    return np.linalg.solve(A.T @ A + lam * np.eye(d), A.T @ b)


def client_gradients(A, b, lam, x, n):
    """Rows of A split into n contiguous equal blocks; returns G [n, d] with G[c] = grad f_c(x)."""
    rows = A.shape[0] // n
    G = np.empty((n, A.shape[1]), dtype=np.float64)
    for c in range(n):
        Ac = A[c * rows:(c + 1) * rows]
        bc = b[c * rows:(c + 1) * rows]
        G[c] = n * (Ac.T @ (Ac @ x - bc)) + lam * x
    return G


def core_gd(A, b, lam, n, m, h, rounds, seed, x0=None, first_round=0):
    """Run Algorithm 2 for ``rounds`` rounds; returns (x, losses[rounds+1])."""
    d = A.shape[1]
    x = np.zeros(d) if x0 is None else np.array(x0, dtype=np.float64)
    losses = [ridge_loss(A, b, lam, x)]
    for k in range(rounds):
        G = client_gradients(A, b, lam, x, n)
        _, _, gtilde = core_round(seed, first_round + k, G, m)
        x = x - h * gtilde
        losses.append(ridge_loss(A, b, lam, x))
    return x, np.array(losses)


def core_agd(A, b, lam, n, m, h, beta, rounds, seed, x0=None, first_round=0):
    """CORE-AGD (appendix, heavy-ball form): y^k = x^k + (1-beta)(x^k - x^{k-1}), the machines
    project grad f_i(y^k), and x^{k+1} = y^k - h * estimator.  x^{-1} = x^0.
    Returns (x, losses[rounds+1])."""
    d = A.shape[1]
    x = np.zeros(d) if x0 is None else np.array(x0, dtype=np.float64)
    x_prev = x.copy()
    losses = [ridge_loss(A, b, lam, x)]
    for k in range(rounds):
        y = x + (1.0 - beta) * (x - x_prev)
        G = client_gradients(A, b, lam, y, n)
        _, _, gtilde = core_round(seed, first_round + k, G, m)
        x_prev = x
        x = y - h * gtilde
        losses.append(ridge_loss(A, b, lam, x))
    return x, np.array(losses)


def ring_gossip_matrix(n):
    """Symmetric doubly-stochastic gossip matrix of a ring: 1/2 on the diagonal, 1/4 to each neighbour."""
    W = np.zeros((n, n))
    for i in range(n):
        W[i, i] += 0.5
        W[i, (i + 1) % n] += 0.25
        W[i, (i - 1) % n] += 0.25
    return W


def decentralized_core_gd(A, b, lam, n, m, h, rounds, seed, W, gossip_steps, x0=None):
    """Decentralized CORE-GD (appendix): machine i projects its own gradient, the machines average
    the m-vectors p_i by `gossip_steps` multiplications with the gossip matrix W (the exact
    solution of the m-dimensional subproblem is the mean), and machine i reconstructs with the
    factor n/m from its own averaged vector and steps its own copy x_i.  Following Eq.
    (tildefdef) for the scale of the objective (f is the mean of the f_i), the step uses the
    reconstruction divided by n.  Returns (X [n, d], losses of the mean iterate)."""
    from . import compress, reconstruct
    d = A.shape[1]
    rows = A.shape[0] // n
    X = np.zeros((n, d)) if x0 is None else np.tile(np.asarray(x0, dtype=np.float64), (n, 1))
    losses = [ridge_loss(A, b, lam, X.mean(axis=0))]
    for k in range(rounds):
        G = np.empty((n, d))
        for c in range(n):
            Ac, bc = A[c * rows:(c + 1) * rows], b[c * rows:(c + 1) * rows]
            G[c] = n * (Ac.T @ (Ac @ X[c] - bc)) + lam * X[c]
        P = compress(seed, k, G, m)                 # [n, m]: machine i's own projections
        for _ in range(gossip_steps):
            P = W @ P
        for c in range(n):
            gt_sum = reconstruct(seed, k, P[c], n / m, 0, d)   # (n/m) sum_j p_j xi_j
            X[c] = X[c] - h * gt_sum / n
        losses.append(ridge_loss(A, b, lam, X.mean(axis=0)))
    return X, np.array(losses)
