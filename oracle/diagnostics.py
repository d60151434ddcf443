"""Diagnostics from the paper's appendix on differential privacy, fp64, CPU.

TEST INFRASTRUCTURE ONLY (see ``core_oracle.c``).

The appendix writes one machine's message as p = C(a) = Xi a, shows (lemma on the law of C(a)) that
p ~ N(0, ||a||^2 I_m), and defines the privacy loss of an output o as the log-ratio of the
probabilities (here: densities) of o under two adjacent inputs.  With gradient norms sigma1 and
sigma2 the two laws are N(0, sigma1^2 I_m) and N(0, sigma2^2 I_m).

Both functions are the definitions written out: the squared Euclidean norm as a sum of squares, and
the loss as the difference of two Gaussian log-densities (NOT the simplified closed form that the
proof of the privacy theorem derives from it; the tests check that the two agree).
"""
from __future__ import annotations

import math

import numpy as np


def projection_sqnorms(P):
    """sq[c] = sum_j P[c][j]^2 for the projections P [n][m] of every machine (lemma on the law of C(a):
    sq[c] / m estimates ||g_c||^2)."""
    P = np.asarray(P, dtype=np.float64)
    if P.ndim != 2:
        raise ValueError("P must be [n][m]")
    return np.array([math.fsum(float(v) * float(v) for v in row) for row in P], dtype=np.float64)


def gaussian_logdensity(p, sigma):
    """ln of the N(0, sigma^2 I_m) density at p: the product of m one-dimensional densities."""
    p = np.asarray(p, dtype=np.float64)
    return math.fsum(-0.5 * math.log(2.0 * math.pi * sigma * sigma) - float(v) * float(v) / (2.0 * sigma * sigma)
                     for v in p)


def privacy_loss(p, sigma1, sigma2):
    """Definition of the privacy loss at the released message p for adjacent gradients of norms
    sigma1 (the data at hand) and sigma2 (the adjacent data)."""
    return gaussian_logdensity(p, sigma1) - gaussian_logdensity(p, sigma2)
