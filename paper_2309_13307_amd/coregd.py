"""CORE-GD (Algorithm 2 of arXiv 2309.13307) driver for a ridge-regression objective.

The library covers the three communication lines of Algorithm 2 (`core_round`); this harness
supplies what surrounds them on the device with torch: the client gradients
g_c = n A_c^T (A_c x - b_c) + lam x of f_c(x) = n/2 |A_c x - b_c|^2 + lam/2 |x|^2 (so that
f = (1/n) sum_c f_c = 1/2 |A x - b|^2 + lam/2 |x|^2, Eq. (problem)), and the update
x <- x - h * gtilde (last line of the loop in Algorithm 2).
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding


def step_size(s: np.ndarray, lam: float, m: int) -> float:
    """h = m / (3 tr(H) + 2 m L) for H = A^T A + lam I with singular values s of A.

    This maximises the decrease h - h^2 (3 tr(A)/(2m) + L) in the proof of Theorem 4.2 before the
    theorem specialises to m <= tr(A)/L (where it becomes Theta(m / tr(A)), the theorem's choice)."""
    d = s.shape[0]
    tr_h = float((s ** 2).sum() + d * lam)
    big_l = float(s.max() ** 2 + lam)
    return m / (3.0 * tr_h + 2.0 * m * big_l)


class RidgeCoreGD:
    """Holds A, b on the device and runs CORE-GD rounds through the C-ABI library."""

    def __init__(self, A: np.ndarray, b: np.ndarray, lam: float, n: int, m: int, seed: int,
                 device="cuda"):
        rows, d = A.shape
        assert rows % n == 0
        self.A = torch.from_numpy(np.ascontiguousarray(A, dtype=np.float32)).to(device)
        self.b = torch.from_numpy(np.ascontiguousarray(b, dtype=np.float32)).to(device)
        self.A3 = self.A.view(n, rows // n, d)
        self.lam, self.n, self.m, self.seed, self.d = lam, n, m, seed, d
        self.x = torch.zeros(d, dtype=torch.float32, device=device)
        self.ws = binding.alloc_workspace(d, m, n, device)
        self.pbar = torch.empty(m, dtype=torch.float32, device=device)
        self.gtilde = torch.empty(d, dtype=torch.float32, device=device)

    def client_gradients(self) -> torch.Tensor:
        r3 = (self.A @ self.x - self.b).view(self.n, -1, 1)
        G = self.n * torch.bmm(self.A3.transpose(1, 2), r3).squeeze(-1) + self.lam * self.x
        return G.contiguous()

    def loss(self) -> float:
        x = self.x.double()
        r = self.A.double() @ x - self.b.double()
        return float(0.5 * (r @ r) + 0.5 * self.lam * (x @ x))

    def round(self, k: int, h: float, G: torch.Tensor | None = None, fused: bool = True) -> torch.Tensor:
        """One round of Algorithm 2 with round counter k; returns the client gradients it used.
        fused: the step x <- x - h * gtilde runs in the epilogue of the reconstruction kernel."""
        if G is None:
            G = self.client_gradients()
        if fused:
            binding.core_round_update(self.seed, k, G, self.m, h, self.x, self.x, self.pbar, self.ws,
                                      gtilde=self.gtilde)
        else:
            binding.core_round(self.seed, k, G, self.m, pbar=self.pbar, gtilde=self.gtilde, ws=self.ws)
            self.x -= h * self.gtilde
        return G

    def capture_round(self, h: float, first_round: int = 0) -> "torch.cuda.CUDAGraph":
        """Record one iteration of Algorithm 2 (client gradients, the fused round, the round counter
        advancing on the device) into a HIP graph; every replay is the next round.  The iteration is
        launch-bound at this size, which is what the graph removes."""
        self.round_dev = torch.full((1,), first_round, dtype=torch.int64, device=self.x.device)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):            # library handles and workspaces are created outside capture
            for _ in range(2):
                self.client_gradients()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            G = self.client_gradients()
            binding.core_round_update_r(self.seed, self.round_dev, G, self.m, h, self.x, self.x, self.pbar,
                                        self.ws, gtilde=self.gtilde)
            binding.core_advance_round(self.round_dev)
        self._graph_G = G                        # keeps the captured buffer alive
        return graph

    def agd_round(self, k: int, h: float, beta: float) -> None:
        """One round of CORE-AGD (heavy-ball form).  State: self.x = x^k, self.y = y^k (the
        extrapolated point; equal to x^0 before the first round).  The kernel epilogue writes
        x^{k+1} = y^k - h * gtilde and y^{k+1} = x^{k+1} + (1-beta)(x^{k+1} - x^k)."""
        if not hasattr(self, "y"):
            self.y = self.x.clone()
            self.x_next = torch.empty_like(self.x)
        x_keep, self.x = self.x, self.y      # gradients are taken at y^k
        G = self.client_gradients()
        self.x = x_keep
        binding.core_round_update(self.seed, k, G, self.m, h, self.y, self.x_next, self.pbar, self.ws,
                                  x_cur=self.x, one_minus_beta=1.0 - beta, y_next=self.y)
        self.x, self.x_next = self.x_next, self.x


class DecentralizedRidgeCoreGD:
    """Decentralized CORE-GD (appendix of the paper) with the n machines batched on one GPU.

    Machine c keeps its own iterate X[c].  Per round: every machine projects its own gradient
    (`core_compress_batched` with P requested), the m-vectors are averaged by a few
    multiplications with the gossip matrix W (torch; on real hardware this is the only exchange),
    and machine c reconstructs from its own averaged vector with the factor n/m and takes its step
    in the kernel epilogue (`core_reconstruct_update`).  As in Eq. (tildefdef) the objective is the
    mean of the f_c, so the step is h/n times the n/m-scaled reconstruction."""

    def __init__(self, A: np.ndarray, b: np.ndarray, lam: float, n: int, m: int, seed: int,
                 W: np.ndarray, gossip_steps: int, device="cuda"):
        rows, d = A.shape
        assert rows % n == 0
        self.A3 = torch.from_numpy(np.ascontiguousarray(A, dtype=np.float32)).to(device).view(n, rows // n, d)
        self.b3 = torch.from_numpy(np.ascontiguousarray(b, dtype=np.float32)).to(device).view(n, rows // n, 1)
        self.W = torch.from_numpy(np.ascontiguousarray(W, dtype=np.float32)).to(device)
        self.lam, self.n, self.m, self.seed, self.d = lam, n, m, seed, d
        self.gossip_steps = gossip_steps
        self.X = torch.zeros((n, d), dtype=torch.float32, device=device)
        self.ws = binding.alloc_workspace(d, m, n, device)

    def round(self, k: int, h: float, batched: bool = True) -> None:
        r3 = torch.bmm(self.A3, self.X.unsqueeze(-1)) - self.b3                  # [n, rows/n, 1]
        G = (self.n * torch.bmm(self.A3.transpose(1, 2), r3).squeeze(-1) + self.lam * self.X).contiguous()
        P, _ = binding.core_compress_batched(self.seed, k, G, self.m, ws=self.ws)
        for _ in range(self.gossip_steps):
            P = self.W @ P
        P = P.contiguous()
        if batched:     # the common vectors are generated once for all machines
            binding.core_reconstruct_update_batched(self.seed, k, P, self.n / self.m, h / self.n, self.X)
        else:
            for c in range(self.n):
                binding.core_reconstruct_update(self.seed, k, P[c], self.n / self.m, h / self.n,
                                                self.X[c], self.X[c])


class RobustCoreGD:
    """Algorithm 3 (CORE-GD for non-convex objectives, Section 5) on a robust-regression objective
    f(x) = mean_i phi(a_i^T x - b_i), phi(t) = t^2 / (1 + t^2), rows split evenly over n machines.

    The library does the round, the statistic p, the Option I step size, the trial point and the
    comparison step; this harness evaluates the client gradients and f with torch.  Nothing in a
    round reads device memory from the host, so rounds can be queued back to back."""

    def __init__(self, A: np.ndarray, b: np.ndarray, n: int, m: int, seed: int, c: float = 4.0,
                 device="cuda"):
        rows, d = A.shape
        assert rows % n == 0
        self.A = torch.from_numpy(np.ascontiguousarray(A, dtype=np.float32)).to(device)
        self.b = torch.from_numpy(np.ascontiguousarray(b, dtype=np.float32)).to(device)
        self.A3 = self.A.view(n, rows // n, d)
        self.n, self.m, self.seed, self.d, self.c = n, m, seed, d, c
        self.rows_per = rows // n
        self.x = torch.zeros(d, dtype=torch.float32, device=device)
        self.x_trial = torch.empty_like(self.x)
        self.ws = binding.alloc_workspace(d, m, n, device)
        self.pbar = torch.empty(m, dtype=torch.float32, device=device)
        self.p = torch.zeros(1, dtype=torch.float32, device=device)
        self.h = torch.zeros(1, dtype=torch.float32, device=device)
        self.accepted = torch.zeros(1, dtype=torch.int32, device=device)
        self.f_cur = self.loss(self.x).reshape(1).clone()
        self.f_trial = torch.zeros(1, dtype=torch.float32, device=device)
        # bounds for this objective: phi'' <= 2, |phi'''| <= 4.67
        A64 = np.asarray(A, dtype=np.float64)
        lam_max = float(np.linalg.eigvalsh(A64.T @ A64 / rows)[-1])
        row2 = (A64 * A64).sum(axis=1)
        self.r1 = 2.0 * float(row2.mean())
        self.L = 2.0 * lam_max
        self.H = 4.67 * float(np.sqrt(row2.max())) * lam_max

    def loss(self, x: torch.Tensor) -> torch.Tensor:
        t = self.A @ x - self.b
        t2 = t * t
        return (t2 / (1.0 + t2)).mean()

    def client_gradients(self, x: torch.Tensor) -> torch.Tensor:
        t = self.A @ x - self.b
        w = (2.0 * t / (1.0 + t * t) ** 2).view(self.n, -1, 1)
        return (torch.bmm(self.A3.transpose(1, 2), w).squeeze(-1) / self.rows_per).contiguous()

    def round(self, k: int, r1: float | None = None, H: float | None = None,
              gtilde: torch.Tensor | None = None) -> torch.Tensor:
        """One iteration of Algorithm 3, Option I; returns the client gradients it used."""
        G = self.client_gradients(self.x)
        binding.core_round_trial(self.seed, k, G, self.m, self.c, self.r1 if r1 is None else r1,
                                 self.H if H is None else H, self.x, self.x_trial, self.pbar, self.p,
                                 self.h, self.ws, gtilde=gtilde)
        self.f_trial.copy_(self.loss(self.x_trial).reshape(1))
        binding.core_accept_trial(self.f_cur, self.f_trial, self.x, self.x_trial, self.accepted)
        return G

    def round_option2(self, k: int, h: float, gtilde: torch.Tensor | None = None) -> torch.Tensor:
        """One iteration of Algorithm 3, Option II: the step h is a constant of the run
        (`binding.core_step_size_option2`), so the trial point comes from the fused update entry
        point; the comparison step is the same."""
        G = self.client_gradients(self.x)
        binding.core_round_update(self.seed, k, G, self.m, h, self.x, self.x_trial, self.pbar, self.ws,
                                  gtilde=gtilde)
        self.f_trial.copy_(self.loss(self.x_trial).reshape(1))
        binding.core_accept_trial(self.f_cur, self.f_trial, self.x, self.x_trial, self.accepted)
        return G

    def capture_round(self, r1: float | None = None, H: float | None = None,
                      first_round: int = 0) -> "torch.cuda.CUDAGraph":
        """Record one whole iteration of Algorithm 3, Option I (client gradients, round, statistic,
        step, trial point, f at the trial point, comparison step, counter advance) into a HIP
        graph.  Nothing in the iteration reads device memory from the host, so a replay is the
        next iteration, accept or reject included."""
        self.round_dev = torch.full((1,), first_round, dtype=torch.int64, device=self.x.device)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):            # library handles and workspaces are created outside capture
            for _ in range(2):
                self.client_gradients(self.x)
                self.loss(self.x)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            G = self.client_gradients(self.x)
            binding.core_round_trial_r(self.seed, self.round_dev, G, self.m, self.c,
                                       self.r1 if r1 is None else r1, self.H if H is None else H,
                                       self.x, self.x_trial, self.pbar, self.p, self.h, self.ws)
            self.f_trial.copy_(self.loss(self.x_trial).reshape(1))
            binding.core_accept_trial(self.f_cur, self.f_trial, self.x, self.x_trial, self.accepted)
            binding.core_advance_round(self.round_dev)
        self._graph_G = G
        return graph
