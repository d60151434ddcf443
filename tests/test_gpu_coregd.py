"""Config 2: CORE-GD (Algorithm 2) on synthetic ridge regression, 200 rounds, d = 4096, m = 64,
n = 8, with the round done by the HIP library and the gradients / update by the torch harness.

Checks, per the paper: every sampled round's (pbar, gtilde) against the oracle fed the same
client gradients; the loss curve against the oracle's own fp64 run of Algorithm 2 from the same
start; the loss gap to the closed-form minimiser x* = (A^T A + lam I)^-1 A^T b shrinking at least
as fast as the bound that follows from the proof of Theorem 4.2 for the step used, within
Monte-Carlo slack (one trajectory)."""
import sys
import time

import numpy as np
import pytest
import torch

import oracle
from oracle import coregd as ocoregd
import paper_2309_13307_amd as core
from paper_2309_13307_amd import coregd, workloads
import parity

pytestmark = pytest.mark.gpu


def _say(msg):
    print(f"[case] {msg}", flush=True)
    sys.stdout.flush()


@pytest.mark.timeout(400)
def test_config2_core_gd_ridge():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    _say("config2: building the ridge problem (QR of an 8192x4096 Gaussian; ~20 s)")
    pr = workloads.ridge_problem()
    d = pr.A.shape[1]
    s = 1.0 / np.arange(1, d + 1)
    h = coregd.step_size(s, pr.lam, pr.m)
    A64, b64 = pr.A.astype(np.float64), pr.b.astype(np.float64)
    xs = ocoregd.ridge_solution(A64, b64, pr.lam)
    fstar = ocoregd.ridge_loss(A64, b64, pr.lam, xs)

    _say("config2: 200 rounds on the GPU")
    run = coregd.RidgeCoreGD(pr.A, pr.b, pr.lam, pr.n, pr.m, pr.seed)
    gaps = [run.loss() - fstar]
    sampled = set([0, 1, 2, 199] + list(range(10, 200, 10)))
    for k in range(pr.rounds):
        G = run.round(k, h)
        if k in sampled:
            torch.cuda.synchronize()
            G_host = G.cpu().numpy()
            P_ref, pbar_ref, gt_ref = oracle.core_round(pr.seed, k, G_host, pr.m)
            norms = parity.row_norms(G_host)
            parity.check_projections(run.pbar.cpu().numpy()[None, :], pbar_ref[None, :],
                                     np.array([norms.mean()]), d, pr.m, f"round {k} pbar")
            parity.check_gtilde(run.gtilde.cpu().numpy(), gt_ref, f"round {k} gtilde")
        gaps.append(run.loss() - fstar)
    gaps = np.array(gaps)

    _say("config2: the oracle's own 200 rounds (fp64)")
    x_ref, losses_ref = ocoregd.core_gd(A64, b64, pr.lam, pr.n, pr.m, h, pr.rounds, pr.seed)
    gaps_ref = losses_ref - fstar
    print("round   gap(GPU path)   gap(oracle)")
    for k in (0, 1, 2, 5, 10, 20, 50, 100, 150, 200):
        print(f"{k:5d}   {gaps[k]:.6e}   {gaps_ref[k]:.6e}")
    # fp32 gradients and an fp32 iterate against an all-fp64 run: the two curves stay together
    assert np.all(np.abs(gaps - gaps_ref) <= 2e-3 * gaps_ref + 1e-7)
    x_gpu = run.x.double().cpu().numpy()
    assert np.linalg.norm(x_gpu - x_ref) <= 1e-3 * np.linalg.norm(x_ref)
    # progress against the closed-form optimum
    assert gaps[-1] < 0.15 * gaps[0]
    assert np.all(gaps > 0)
    # expected contraction per round for this step is at most 1 - mu h (proof of Theorem 4.2 with
    # the strong-convexity step); one trajectory, so allow slack on the exponent
    mu = float(s.min() ** 2 + pr.lam)
    assert gaps[-1] <= gaps[0] * (1.0 - mu * h) ** (0.5 * pr.rounds)


    # the fused step and the separate torch update give the same iterates to fp32 rounding
    run2 = coregd.RidgeCoreGD(pr.A, pr.b, pr.lam, pr.n, pr.m, pr.seed)
    for k in range(20):
        run2.round(k, h, fused=False)
    run3 = coregd.RidgeCoreGD(pr.A, pr.b, pr.lam, pr.n, pr.m, pr.seed)
    for k in range(20):
        run3.round(k, h, fused=True)
    torch.cuda.synchronize()
    assert float((run2.x - run3.x).norm() / run2.x.norm()) < 1e-6

    # CORE-AGD (heavy-ball form) with the update and the next extrapolated point written by the
    # kernel epilogue, against the oracle's fp64 run
    _say("config2 problem: 60 rounds of CORE-AGD")
    beta = 0.2
    h_agd = 0.5 * h
    run4 = coregd.RidgeCoreGD(pr.A, pr.b, pr.lam, pr.n, pr.m, pr.seed)
    for k in range(60):
        run4.agd_round(k, h_agd, beta)
    torch.cuda.synchronize()
    x_agd_ref, losses_agd = ocoregd.core_agd(A64, b64, pr.lam, pr.n, pr.m, h_agd, beta, 60, pr.seed)
    x_agd = run4.x.double().cpu().numpy()
    print("CORE-AGD gap after 60 rounds: GPU path", run4.loss() - fstar, "oracle", losses_agd[-1] - fstar)
    assert np.linalg.norm(x_agd - x_agd_ref) <= 1e-3 * np.linalg.norm(x_agd_ref)
    assert abs((run4.loss() - fstar) - (losses_agd[-1] - fstar)) <= 5e-3 * (losses_agd[-1] - fstar)


def test_decentralized_core_gd_small():
    """Decentralized CORE-GD: per-machine projections, gossip averaging, reconstruction with n/m
    and the step in the kernel epilogue, against the oracle's fp64 run."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    _say("decentralized CORE-GD d=512 m=32 n=8, 12 rounds, 3 gossip steps on a ring")
    pr = workloads.ridge_problem(rows=1024, d=512, n=8, m=32, lam=1e-2, rounds=12)
    s = 1.0 / np.arange(1, 513)
    h = coregd.step_size(s, pr.lam, pr.m)
    W = ocoregd.ring_gossip_matrix(pr.n)
    run = coregd.DecentralizedRidgeCoreGD(pr.A, pr.b, pr.lam, pr.n, pr.m, pr.seed, W, 3)
    for k in range(pr.rounds):
        run.round(k, h)
    torch.cuda.synchronize()
    X_ref, losses = ocoregd.decentralized_core_gd(pr.A.astype(np.float64), pr.b.astype(np.float64), pr.lam,
                                                   pr.n, pr.m, h, pr.rounds, pr.seed, W, 3)
    X = run.X.double().cpu().numpy()
    assert np.linalg.norm(X - X_ref) <= 1e-4 * np.linalg.norm(X_ref)
    assert np.abs(X_ref - X_ref.mean(axis=0)).max() > 1e-6     # the copies really differ
    assert losses[-1] < losses[0]


@pytest.mark.timeout(300)
def test_graph_replayed_core_gd_matches_eager():
    """One iteration of Algorithm 2 recorded into a HIP graph with the round counter in device
    memory: every replay must be the next round, bit-identical to the eager loop that passes the
    counter by value, also with eager work and synchronisation between replays."""
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    pr = workloads.ridge_problem(rows=2048, d=1024, n=8, m=64, rounds=60)
    d = pr.A.shape[1]
    s = 1.0 / np.arange(1, d + 1)
    h = coregd.step_size(s, pr.lam, pr.m)
    first = (1 << 32) - 20                       # the counter crosses 2^32 during the run
    _say(f"graph-replayed CORE-GD: d={d} m={pr.m} n={pr.n}, {pr.rounds} rounds from round {first}")
    eager = coregd.RidgeCoreGD(pr.A, pr.b, pr.lam, pr.n, pr.m, pr.seed)
    xs = []
    for k in range(pr.rounds):
        eager.round(first + k, h)
        xs.append(eager.x.clone())
    torch.cuda.synchronize()

    run = coregd.RidgeCoreGD(pr.A, pr.b, pr.lam, pr.n, pr.m, pr.seed)
    graph = run.capture_round(h, first_round=first)
    torch.cuda.synchronize()
    assert run.round_dev.item() == first and float(run.x.abs().max()) == 0.0, "capture must not execute"
    scratch = torch.zeros(1 << 16, device="cuda")
    for k in range(pr.rounds):
        graph.replay()
        if k % 7 == 3:                           # eager work and a sync between replays
            scratch.add_(1.0)
            torch.cuda.synchronize()
        if k % 5 == 0 or k == pr.rounds - 1:
            torch.cuda.synchronize()
            assert torch.equal(run.x, xs[k]), f"replay {k} differs from eager round {first + k}"
    torch.cuda.synchronize()
    assert run.round_dev.item() == first + pr.rounds
    # the last round against the oracle, from the gradients the graph used
    G_host = run._graph_G.cpu().numpy()
    _, pbar_ref, gt_ref = oracle.core_round(pr.seed, first + pr.rounds - 1, G_host, pr.m)
    parity.check_gtilde(run.gtilde.cpu().numpy(), gt_ref, "last replayed round")

    # launch overhead: time 200 more rounds each way
    t = []
    for mode in ("eager", "graph"):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(200):
            if mode == "eager":
                eager.round(first + pr.rounds + k, h)
            else:
                graph.replay()
        torch.cuda.synchronize()
        t.append((time.perf_counter() - t0) / 200 * 1e6)
    _say(f"per round: eager {t[0]:.1f} us, graph replay {t[1]:.1f} us")
    assert torch.equal(run.x, eager.x)   # the timing above is reported, not asserted
