"""Seeded synthetic inputs for the tests and the benchmark.

This module only draws inputs (client gradients, a ridge-regression problem); it contains none
of the method's arithmetic and is the one module shared by the GPU-side tests/bench and the
CPU oracle's callers.  The paper's own experiments use LibSVM data and CIFAR models that are
not available here; these inputs stand in for their shapes:

  config 1  d=1024,        m=16,   n=4,  fp32   tiny single round
  config 2  d=4096,        m=64,   n=8,  fp32   CORE-GD on ridge regression, 200 rounds
  config 3  d=2^20,        m=256,  n=8,  fp32   common vector + per-client perturbation
  config 4  d=25,557,032,  m=1024, n=8,  bf16   ResNet-50-sized gradient, 161 scale blocks
  config 5  d=124,439,808, m=4096, n=16, bf16   GPT-2-small-sized gradient, heavy tails, 5 rounds
  robust    d=2048,        m=64,   n=8,  fp32   non-convex robust regression for Algorithm 3
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np
import torch


@dataclass
class RoundCase:
    name: str
    d: int
    m: int
    n: int
    seed: int            # shared generator seed of the CORE round
    rounds: tuple        # round counters to run
    G: torch.Tensor      # [n, d] on the requested device, fp32 or bf16


def config1(device="cpu") -> RoundCase:
    G = np.random.default_rng(0).standard_normal((4, 1024)).astype(np.float32)
    return RoundCase("config1", 1024, 16, 4, 42, (0,), torch.from_numpy(G).to(device))


def config2_round(device="cpu") -> RoundCase:
    """One round of config 2's shape (d=4096, m=64, n=8, fp32) on gradient-like inputs: a common
    direction plus per-client noise.  The full CORE-GD run of config 2 is `ridge_problem`."""
    d, n = 4096, 8
    common = np.random.default_rng(20).standard_normal(d) / np.arange(1, d + 1) ** 0.5
    G = np.empty((n, d), dtype=np.float32)
    for c in range(n):
        G[c] = (common + 0.3 * np.random.default_rng(21 + c).standard_normal(d)).astype(np.float32)
    return RoundCase("config2", d, 64, n, 2, (0,), torch.from_numpy(G).to(device))


def config3(device="cpu") -> RoundCase:
    d, n = 1 << 20, 8
    common = np.random.default_rng(0).standard_normal(d)
    G = np.empty((n, d), dtype=np.float32)
    for c in range(n):
        G[c] = (common + 0.1 * np.random.default_rng(c + 1).standard_normal(d)).astype(np.float32)
    return RoundCase("config3", d, 256, n, 7, (0,), torch.from_numpy(G).to(device))


def _block_sigmas(d: int, nblocks: int, seed: int):
    """Contiguous equal-size blocks with log-uniform scales in [1e-4, 1e-1]."""
    rng = np.random.default_rng(seed)
    sig = 10.0 ** rng.uniform(-4.0, -1.0, nblocks)
    bounds = [(l * d) // nblocks for l in range(nblocks + 1)]
    return bounds, sig


def config4(device="cuda", d: int = 25_557_032, m: int = 1024, n: int = 8) -> RoundCase:
    """Per-layer-scaled Gaussian gradients stored in bf16 (drawn on `device` with a seeded torch
    generator; only within-run determinism is needed, the checker reads back the same bits)."""
    bounds, sig = _block_sigmas(d, 161, 4)
    scale = torch.empty(d, dtype=torch.float32, device=device)
    for l in range(161):
        scale[bounds[l]:bounds[l + 1]] = float(sig[l])
    gen = torch.Generator(device=device)
    G = torch.empty((n, d), dtype=torch.bfloat16, device=device)
    for c in range(n):
        gen.manual_seed(4000 + c)
        G[c] = (torch.randn(d, generator=gen, device=device, dtype=torch.float32) * scale).to(torch.bfloat16)
    return RoundCase("config4", d, m, n, 11, (0,), G)


def config5(device="cuda", d: int = 124_439_808, m: int = 4096, n: int = 16) -> RoundCase:
    """Heavy-tailed (Student-t, 3 degrees of freedom) gradients scaled by 1e-3, bf16."""
    gen = torch.Generator(device=device)
    G = torch.empty((n, d), dtype=torch.bfloat16, device=device)
    for c in range(n):
        gen.manual_seed(5000 + c)
        z = torch.randn(d, generator=gen, device=device, dtype=torch.float32)
        chi = torch.zeros(d, dtype=torch.float32, device=device)
        for _ in range(3):
            chi += torch.randn(d, generator=gen, device=device, dtype=torch.float32) ** 2
        G[c] = (1e-3 * z / torch.sqrt(chi / 3.0)).to(torch.bfloat16)
        del z, chi
    return RoundCase("config5", d, m, n, 13, (0, 1, 2, 3, 4), G)


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    """bf16 tensor -> uint16 bit patterns on the host (what the oracle takes as stored)."""
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def to_host(t: torch.Tensor) -> np.ndarray:
    """Device tensor as the host array the oracle consumes: fp32 as is, bf16 as bit patterns."""
    if t.dtype == torch.bfloat16:
        return bf16_bits(t)
    return t.detach().cpu().numpy()


@dataclass
class RidgeProblem:
    A: np.ndarray        # [rows, d] fp32
    b: np.ndarray        # [rows] fp32
    lam: float
    n: int
    m: int
    seed: int
    rounds: int


def ridge_problem(rows: int = 8192, d: int = 4096, n: int = 8, m: int = 64, lam: float = 1e-3,
                  rounds: int = 200) -> RidgeProblem:
    """A = U diag(s) V^T with Haar U, V (QR of Gaussians, signs fixed by diag R > 0) and
    s_k = 1/k; b = A x_true + 0.01 N(0,1)."""
    def haar(r, c, seed):
        Q, R = np.linalg.qr(np.random.default_rng(seed).standard_normal((r, c)))
        return Q * np.sign(np.diag(R))
    U = haar(rows, d, 0)
    V = haar(d, d, 1)
    s = 1.0 / np.arange(1, d + 1)
    A = (U * s) @ V.T
    x_true = np.random.default_rng(2).standard_normal(d)
    b = A @ x_true + 0.01 * np.random.default_rng(3).standard_normal(rows)
    return RidgeProblem(A.astype(np.float32), b.astype(np.float32), lam, n, m, 2, rounds)


@dataclass
class RobustProblem:
    A: np.ndarray        # [rows, d] fp32
    b: np.ndarray        # [rows] fp32, every 7th entry an outlier
    n: int
    m: int
    seed: int
    rounds: int


def robust_problem(rows: int = 4096, d: int = 2048, n: int = 8, m: int = 64, rounds: int = 40) -> RobustProblem:
    """Data of a robust-regression objective mean_i phi(a_i^T x - b_i) with a bounded, partly
    concave phi (the non-convex stand-in for Section 5): Gaussian rows of norm about 1,
    b = A x_true + 0.1 N(0,1), and +5 added to every 7th entry so that negative curvature occurs."""
    rng = np.random.default_rng(50)
    A = rng.standard_normal((rows, d)) / np.sqrt(d)
    x_true = rng.standard_normal(d)
    b = A @ x_true + 0.1 * rng.standard_normal(rows)
    b[::7] += 5.0
    return RobustProblem(A.astype(np.float32), b.astype(np.float32), n, m, 9, rounds)
