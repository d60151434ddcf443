"""Algorithm 3 (CORE-GD for non-convex objectives, Section 5) on the GPU against the oracle.

Pieces: the norm statistic p and the Option I step (device scalars), the trial point with the
step read from device memory, the comparison step (decision bit-exact for the same objective
values; x bit-identical to the trial point on accept and untouched on reject), the fused
`core_round_trial`, and a run of the whole loop on a robust-regression objective with every
round's quantities checked against the oracle fed the same client gradients.
"""
import math
import sys

import numpy as np
import pytest
import torch

import oracle
from oracle import nonconvex as onc
import paper_2309_13307_amd as core
from paper_2309_13307_amd import coregd, workloads
import parity

pytestmark = pytest.mark.gpu

STEP_REL = 2e-6      # p and h: one fp32 rounding of the inputs' fp64 result, a sqrt and a divide


def _say(msg):
    print(f"[case] {msg}", flush=True)
    sys.stdout.flush()


def _dev(a, dtype=torch.float32):
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda", dtype)


@pytest.mark.parametrize("m", [1, 5, 64, 257, 1000, 4096, 70001])
def test_nonconvex_step_matches_oracle(m):
    _say(f"nonconvex_step m={m}")
    rng = np.random.default_rng(m)
    pbar = (rng.standard_normal(m) * 10 ** rng.uniform(-3, 2)).astype(np.float32)
    p_out = torch.zeros(1, device="cuda")
    h_out = torch.zeros(1, device="cuda")
    for d, c, r1, H in ((4096, 4.0, 3.0, 2.0), (25_557_032, 2.0, 1e3, 1e-2), (16, 8.3, 1e-6, 1e-9),
                        (10 ** 6, 4.0, 1e9, 1.0)):
        core.core_nonconvex_step(d, _dev(pbar), c, r1, H, p_out, h_out)
        torch.cuda.synchronize()
        p_ref = onc.norm_statistic(pbar.astype(np.float64), c)
        h_ref = onc.step_size_option1(d, m, r1, H, p_ref)
        assert abs(p_out.item() - p_ref) <= STEP_REL * p_ref
        assert abs(h_out.item() - h_ref) <= STEP_REL * h_ref
    # p_out is optional; zero projections leave the first term
    core.core_nonconvex_step(4096, torch.zeros(m, device="cuda"), 4.0, 3.0, 2.0, None, h_out)
    torch.cuda.synchronize()
    assert h_out.item() == np.float32(m / 48.0)
    core.core_nonconvex_step(4096, torch.zeros(m, device="cuda"), 4.0, 3.0, 2.0, p_out, h_out)
    torch.cuda.synchronize()
    assert p_out.item() == 0.0


@pytest.mark.parametrize("d,m,offset", [(4096, 16, 0), (4099, 7, 0), (100_003, 64, 0), (70_001, 33, 1),
                                        (3, 2, 0), (1_048_576, 256, 0)])
def test_reconstruct_trial_matches_oracle(d, m, offset):
    _say(f"reconstruct_trial d={d} m={m} offset={offset}")
    rng = np.random.default_rng(d + m)
    pbar = rng.standard_normal(m).astype(np.float32)
    x = rng.standard_normal(d).astype(np.float32)
    h = np.float32(0.37)
    seed, rnd, scale = 77, 5, 1.0 / m
    xb = torch.zeros(d + 4, device="cuda")
    tb = torch.zeros(d + 4, device="cuda")
    gb = torch.zeros(d + 4, device="cuda")
    xd, td, gd = xb[offset:offset + d], tb[offset:offset + d], gb[offset:offset + d]
    xd.copy_(_dev(x))
    hd = _dev(np.array([h]))
    core.core_reconstruct_trial(seed, rnd, _dev(pbar), scale, hd, xd, td, gtilde=gd)
    torch.cuda.synchronize()
    gt_ref = oracle.reconstruct(seed, rnd, pbar.astype(np.float64), scale, 0, d)
    parity.check_gtilde(gd.cpu().numpy(), gt_ref, "gtilde of the trial call")
    step_gpu = x.astype(np.float64) - td.cpu().numpy().astype(np.float64)
    step_ref = float(h) * gt_ref
    # the step is recovered through x (|x| ~ 1): allow its fp32 rounding on top of the 1e-5 bar
    assert np.linalg.norm(step_gpu - step_ref) <= 1e-5 * np.linalg.norm(step_ref) + 1.2e-7 * np.linalg.norm(x)
    assert torch.equal(xd, _dev(x)), "x must not be written"
    # without gtilde, and against the host-h entry point: identical bits
    t2 = torch.zeros(d, device="cuda")
    core.core_reconstruct_trial(seed, rnd, _dev(pbar), scale, hd, xd.contiguous(), t2)
    t3 = torch.zeros(d, device="cuda")
    core.core_reconstruct_update(seed, rnd, _dev(pbar), scale, float(h), xd.contiguous(), t3)
    torch.cuda.synchronize()
    assert torch.equal(t2, td) and torch.equal(t3, td)


@pytest.mark.parametrize("d,offset", [(1, 0), (5, 0), (4096, 0), (100_003, 0), (70_001, 1), (1_048_577, 3)])
def test_accept_trial_decisions_and_copies(d, offset):
    _say(f"accept_trial d={d} offset={offset}")
    rng = np.random.default_rng(d)
    x0 = rng.standard_normal(d).astype(np.float32)
    xt = rng.standard_normal(d).astype(np.float32)
    nan = float("nan")
    cases = [(1.0, 0.5), (1.0, 1.0), (0.5, 1.0), (1.0, nan), (nan, 0.5), (-2.0, -2.0000002),
             (np.float32(1.0), np.nextafter(np.float32(1.0), np.float32(0.0))), (0.0, -0.0), (1e-30, 0.0)]
    for fc, ft in cases:
        xb = torch.zeros(d + 4, device="cuda")
        tb = torch.zeros(d + 4, device="cuda")
        xd, td = xb[offset:offset + d], tb[offset:offset + d]
        xd.copy_(_dev(x0))
        td.copy_(_dev(xt))
        f_cur = _dev(np.array([fc], dtype=np.float32))
        f_trial = _dev(np.array([ft], dtype=np.float32))
        acc = torch.full((1,), -7, dtype=torch.int32, device="cuda")
        core.core_accept_trial(f_cur, f_trial, xd, td, acc)
        torch.cuda.synchronize()
        take = onc.comparison_step(float(np.float32(fc)), float(np.float32(ft)))
        assert acc.item() == int(take), (fc, ft)
        want_x = xt if take else x0
        assert np.array_equal(xd.cpu().numpy().view(np.uint32), want_x.view(np.uint32))
        assert np.array_equal(td.cpu().numpy().view(np.uint32), xt.view(np.uint32))
        want_f = np.float32(ft) if take else np.float32(fc)
        got_f = f_cur.cpu().numpy()
        assert np.array_equal(got_f.view(np.uint32), np.array([want_f]).view(np.uint32))
        # the padding around an offset view is untouched
        assert xb[:offset].abs().sum().item() == 0.0 and xb[offset + d:].abs().sum().item() == 0.0


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_round_trial_equals_its_pieces(dtype):
    d, m, n = 50_003, 96, 5
    _say(f"round_trial vs pieces d={d} m={m} n={n} {dtype}")
    rng = np.random.default_rng(8)
    G = _dev(rng.standard_normal((n, d)).astype(np.float32) * 0.01).to(dtype)
    x = _dev(rng.standard_normal(d).astype(np.float32))
    ws = core.alloc_workspace(d, m, n)
    c, r1, H = 4.0, 2.0, 1e-4
    pbar = torch.zeros(m, device="cuda")
    p = torch.zeros(1, device="cuda")
    h = torch.zeros(1, device="cuda")
    xt = torch.zeros(d, device="cuda")
    gt = torch.zeros(d, device="cuda")
    core.core_round_trial(3, 11, G, m, c, r1, H, x, xt, pbar, p, h, ws, gtilde=gt)
    _, pbar2 = core.core_compress_batched(3, 11, G, m, ws=ws, want_P=False)
    p2 = torch.zeros(1, device="cuda")
    h2 = torch.zeros(1, device="cuda")
    core.core_nonconvex_step(d, pbar2, c, r1, H, p2, h2)
    xt2 = torch.zeros(d, device="cuda")
    gt2 = torch.zeros(d, device="cuda")
    core.core_reconstruct_trial(3, 11, pbar2, 1.0 / m, h2, x, xt2, gtilde=gt2)
    torch.cuda.synchronize()
    assert torch.equal(pbar, pbar2) and torch.equal(p, p2) and torch.equal(h, h2)
    assert torch.equal(xt, xt2) and torch.equal(gt, gt2)
    # and against the oracle
    G_host = workloads.to_host(G)
    _, pbar_ref, gt_ref = oracle.core_round(3, 11, G_host, m)
    norms = parity.row_norms(G_host)
    parity.check_projections(pbar.cpu().numpy()[None, :], pbar_ref[None, :], np.array([norms.mean()]), d, m)
    parity.check_gtilde(gt.cpu().numpy(), gt_ref)
    p_ref = onc.norm_statistic(pbar_ref, c)
    h_ref = onc.step_size_option1(d, m, r1, H, p_ref)
    assert abs(p.item() - p_ref) <= 1e-5 * p_ref and abs(h.item() - h_ref) <= 1e-5 * h_ref


@pytest.mark.timeout(300)
def test_algorithm3_on_robust_regression():
    pr = workloads.robust_problem()
    rows, d = pr.A.shape
    _say(f"Algorithm 3 on robust regression: d={d} m={pr.m} n={pr.n}, {pr.rounds} rounds x 3 settings")
    A64, b64 = pr.A.astype(np.float64), pr.b.astype(np.float64)
    f64 = lambda x: onc.robust_loss(A64, b64, x)
    for label, r1_scale, H_scale in (("the paper's constants", 1.0, 1.0), ("large steps", 2e-2, 1e-9),
                                     ("steps large enough for rejections", 4e-3, 1e-10)):
        run = coregd.RobustCoreGD(pr.A, pr.b, pr.n, pr.m, pr.seed)
        r1o, Lo, Ho = onc.robust_constants(A64)
        assert math.isclose(run.r1, r1o, rel_tol=1e-9) and math.isclose(run.H, Ho, rel_tol=1e-9)
        r1, H = run.r1 * r1_scale, run.H * H_scale
        gt = torch.zeros(d, device="cuda")
        fs = [run.f_cur.item()]
        n_acc = 0
        for k in range(pr.rounds):
            x_before = run.x.clone()
            f_before = run.f_cur.clone()
            G = run.round(k, r1=r1, H=H, gtilde=gt)
            torch.cuda.synchronize()
            G_host = G.cpu().numpy()
            xb = x_before.cpu().numpy().astype(np.float64)
            # the oracle's iteration from the same point and the same client gradients
            _, pbar_ref, gt_ref = oracle.core_round(pr.seed, k, G_host, pr.m)
            p_ref = onc.norm_statistic(pbar_ref, 4.0)
            h_ref = onc.step_size_option1(d, pr.m, r1, H, p_ref)
            norms = parity.row_norms(G_host)
            parity.check_projections(run.pbar.cpu().numpy()[None, :], pbar_ref[None, :],
                                     np.array([norms.mean()]), d, pr.m, f"{label} round {k}")
            parity.check_gtilde(gt.cpu().numpy(), gt_ref, f"{label} round {k}")
            assert abs(run.p.item() - p_ref) <= 1e-5 * p_ref
            assert abs(run.h.item() - h_ref) <= 1e-5 * h_ref
            xt_ref = xb - h_ref * gt_ref
            xt_gpu = run.x_trial.cpu().numpy().astype(np.float64)
            assert np.linalg.norm(xt_gpu - xt_ref) <= 1e-5 * np.linalg.norm(h_ref * gt_ref) + 1.2e-7 * np.linalg.norm(xb)
            # objective values: the harness's fp32 evaluation against fp64
            ft_gpu, fc_gpu = run.f_trial.item(), f_before.item()
            assert abs(ft_gpu - f64(xt_gpu)) <= 2e-6 and abs(fc_gpu - f64(xb)) <= 2e-6
            # the decision is the oracle's for the values the kernel saw
            take = onc.comparison_step(fc_gpu, ft_gpu)
            assert run.accepted.item() == int(take)
            want = run.x_trial if take else x_before
            assert torch.equal(run.x, want)
            assert run.f_cur.item() == (ft_gpu if take else fc_gpu)
            n_acc += int(take)
            fs.append(run.f_cur.item())
        fs = np.array(fs)
        assert np.all(np.diff(fs) <= 0.0), "the comparison step never lets f rise"
        _say(f"{label}: f {fs[0]:.6f} -> {fs[-1]:.6f}, accepted {n_acc}/{pr.rounds}, last h {run.h.item():.3e}")
        assert n_acc > 0
        if label == "large steps":
            assert fs[-1] < 0.9 * fs[0]
        if label == "steps large enough for rejections":
            assert 0 < n_acc < pr.rounds


@pytest.mark.timeout(300)
def test_algorithm3_option2_on_robust_regression():
    pr = workloads.robust_problem()
    rows, d = pr.A.shape
    _say(f"Algorithm 3, Option II on robust regression: d={d} m={pr.m} n={pr.n}")
    A64, b64 = pr.A.astype(np.float64), pr.b.astype(np.float64)
    f64 = lambda x: onc.robust_loss(A64, b64, x)
    grads64 = lambda x: onc.robust_client_gradients(A64, b64, x, pr.n)
    run = coregd.RobustCoreGD(pr.A, pr.b, pr.n, pr.m, pr.seed)
    Delta = f64(np.zeros(d))
    for label, r1, H in (("the paper's constants", run.r1, run.H), ("large steps", run.r1 * 2e-2, run.H * 1e-12)):
        run = coregd.RobustCoreGD(pr.A, pr.b, pr.n, pr.m, pr.seed)
        h = core.core_step_size_option2(d, pr.m, r1, H, run.L, Delta)
        assert math.isclose(h, onc.step_size_option2(d, pr.m, r1, H, run.L, Delta), rel_tol=1e-12)
        fs = [run.f_cur.item()]
        rounds = 20
        for k in range(rounds):
            x_before = run.x.clone()
            f_before = run.f_cur.item()
            G = run.round_option2(k, h)
            torch.cuda.synchronize()
            xb = x_before.cpu().numpy().astype(np.float64)
            _, _, gt_ref = oracle.core_round(pr.seed, k, G.cpu().numpy(), pr.m)
            xt_gpu = run.x_trial.cpu().numpy().astype(np.float64)
            step = h * gt_ref
            assert np.linalg.norm(xt_gpu - (xb - step)) <= 1e-5 * np.linalg.norm(step) + 1.2e-7 * np.linalg.norm(xb)
            take = onc.comparison_step(f_before, run.f_trial.item())
            assert run.accepted.item() == int(take)
            assert torch.equal(run.x, run.x_trial if take else x_before)
            fs.append(run.f_cur.item())
        fs = np.array(fs)
        assert np.all(np.diff(fs) <= 0.0)
        _say(f"Option II, {label}: h={h:.3e}, f {fs[0]:.6f} -> {fs[-1]:.6f}")
        # the oracle's own Option II run from the same start: same step, f within fp32 evaluation error
        ref = onc.core_gd_nonconvex(f64, grads64, np.zeros(d), pr.m, rounds, pr.seed, option=2, r1=r1, H=H,
                                    L=run.L, Delta=Delta)
        assert ref["h"][0] == onc.step_size_option2(d, pr.m, r1, H, run.L, Delta)
        if label == "large steps":
            assert fs[-1] < 0.95 * fs[0]
            assert abs(fs[-1] - ref["f"][-1]) <= 2e-3 * ref["f"][0]


@pytest.mark.timeout(300)
def test_graph_replayed_algorithm3_matches_eager():
    """A whole iteration of Algorithm 3 (gradients, round, statistic, step, trial point, f at the
    trial point, comparison step) recorded once into a HIP graph: each replay is the next
    iteration, with accepts and rejects decided on the device, bit-identical to the eager loop."""
    pr = workloads.robust_problem()
    d = pr.A.shape[1]
    rounds = 30
    _say(f"graph-replayed Algorithm 3: d={d} m={pr.m} n={pr.n}, {rounds} rounds")
    eager = coregd.RobustCoreGD(pr.A, pr.b, pr.n, pr.m, pr.seed)
    r1, H = eager.r1 * 4e-3, eager.H * 1e-10           # steps large enough for rejections
    trace = []
    for k in range(rounds):
        eager.round(k, r1=r1, H=H)
        trace.append((eager.x.clone(), eager.f_cur.clone(), eager.accepted.clone(), eager.h.clone(), eager.p.clone()))
    torch.cuda.synchronize()
    flags = [int(t[2].item()) for t in trace]
    assert 0 < sum(flags) < rounds, "the run should contain accepts and rejects"

    run = coregd.RobustCoreGD(pr.A, pr.b, pr.n, pr.m, pr.seed)
    graph = run.capture_round(r1=r1, H=H)
    torch.cuda.synchronize()
    assert run.round_dev.item() == 0 and float(run.x.abs().max()) == 0.0, "capture must not execute"
    scratch = torch.zeros(1 << 14, device="cuda")
    for k in range(rounds):
        graph.replay()
        if k % 4 == 1:                                   # eager work and a sync between replays
            scratch.add_(1.0)
            torch.cuda.synchronize()
        torch.cuda.synchronize()
        x, f, acc, h, p = trace[k]
        assert run.accepted.item() == acc.item(), f"replay {k}: accept flag"
        assert torch.equal(run.x, x) and torch.equal(run.f_cur, f), f"replay {k}: iterate / objective"
        assert torch.equal(run.h, h) and torch.equal(run.p, p), f"replay {k}: step / statistic"
    assert run.round_dev.item() == rounds
