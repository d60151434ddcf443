"""GPU parity tests: the HIP path (through the C ABI) against the CPU oracle on the same seeded
inputs.  Sizes here are ones the oracle finishes in seconds; they span several 256-coordinate
tiles, several 256-vector tiles, ragged tails in d, m and n, and every client-count template."""
import sys

import numpy as np
import pytest
import torch

import oracle
import paper_2309_13307_amd as core
from paper_2309_13307_amd import workloads
import parity

pytestmark = pytest.mark.gpu

DEV = "cuda"


def _say(msg):
    print(f"[case] {msg}", flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    core.load_library()


def _sync():
    torch.cuda.synchronize()


# ---------------------------------------------------------------------------------------------
# generator


@pytest.mark.parametrize("seed,rnd,j,q0,nb", [
    (42, 0, 0, 0, 1024),
    (7, 0, 255, 262143 - 5, 64),
    (0xDEADBEEF12345678, 0x1_0000_0003, 4095, (1 << 32) - 300, 300),
    (1, 5, (1 << 32) - 1, 12345, 257),
])
def test_philox_words_bit_exact(seed, rnd, j, q0, nb):
    _say(f"philox seed={seed} round={rnd} j={j} q0={q0} nb={nb}")
    got = core.core_debug_philox(seed, rnd, j, q0, nb).cpu().numpy().view(np.uint32)
    ref = oracle.words_range(seed, rnd, j, q0, nb)
    assert np.array_equal(got, ref)


# (seed, round, j0, nj, q0, nq): windows of vectors x blocks that cover the first block, a ragged
# count of lanes in both directions, several waves, the largest block index (d = 2^34), the largest
# vector index, a round counter with a non-zero high word and a seed with a non-zero high word.
PHILOX_WINDOWS = [
    (42, 0, 0, 70, 0, 70),
    (7, 0, 200, 300, 262143 - 5, 9),
    (0xDEADBEEF12345678, 0x1_0000_0003, 4090, 67, (1 << 32) - 300, 300),
    (1, 5, (1 << 32) - 130, 130, 12345, 5),
    (13, (1 << 63) + 9, 1023, 1, (1 << 32) - 1, 1),
    (0xFFFFFFFFFFFFFFFF, 0xFFFFFFFFFFFFFFFF, (1 << 32) - 1, 1, 77, 257),
]


@pytest.mark.parametrize("layout", ["scalar_keys", "projection", "reconstruction", "debug_xi", "projection_sub_tiles"])
@pytest.mark.parametrize("seed,rnd,j0,nj,q0,nq", PHILOX_WINDOWS)
def test_philox_words_bit_exact_in_every_kernel_layout(layout, seed, rnd, j0, nj, q0, nq):
    """Algorithm 1, REQUIRE line: all machines share one generator, so the uint32 stream must be
    the reference stream bit for bit.  Each layout runs the generator instantiation (which rounds
    have their keys in vector registers and use the three-input xor) in the lane arrangement of one
    family of production kernels: lanes over vectors with a wave-uniform block index (projection),
    lanes over blocks with a wave-uniform vector index (reconstruction, small-problem projection)."""
    _say(f"philox layout={layout} seed={seed:#x} round={rnd:#x} j0={j0} nj={nj} q0={q0} nq={nq}")
    got = core.core_debug_philox_layout(layout, seed, rnd, j0, nj, q0, nq).cpu().numpy().view(np.uint32)
    ref = np.stack([oracle.words_range(seed, rnd, j0 + jj, q0, nq) for jj in range(nj)])
    assert got.shape == ref.shape == (nj, nq, 4)
    assert np.array_equal(got, ref)


@pytest.mark.parametrize("seed,rnd,j,i0,count", [
    (42, 0, 0, 0, 1 << 20),
    (7, 3, 200, 5, 100003),
    (9, 1 << 33, 1023, (1 << 34) - 4096, 4096),
])
def test_xi_close_to_oracle(seed, rnd, j, i0, count):
    _say(f"xi seed={seed} round={rnd} j={j} i0={i0} count={count}")
    got = core.core_debug_xi(seed, rnd, j, i0, count).cpu().numpy().astype(np.float64)
    ref = oracle.xi_range(seed, rnd, j, i0, count)
    err = np.abs(got - ref)
    assert err.max() <= parity.XI_MAX_ABS, err.max()
    assert np.sqrt(np.mean(err ** 2)) <= parity.XI_RMS_ABS


# ---------------------------------------------------------------------------------------------
# full rounds on small shapes


def _run_and_check(seed, rnd, G_dev, m, d=None, what=""):
    n = G_dev.shape[0]
    d = G_dev.shape[1] if d is None else d
    G_host = workloads.to_host(G_dev[:, :d])
    P_ref, pbar_ref, gt_ref = oracle.core_round(seed, rnd, np.ascontiguousarray(G_host), m)
    norms = parity.row_norms(G_host)

    P, pbar = core.core_compress_batched(seed, rnd, G_dev, m, d=d)
    gt_recon = core.core_reconstruct(seed, rnd, d, torch.from_numpy(pbar_ref.astype(np.float32)).to(DEV), 1.0 / m)
    pbar2, gt = core.core_round(seed, rnd, G_dev, m, d=d)
    _sync()
    parity.check_projections(P.cpu().numpy(), P_ref, norms, d, m, what + " P")
    mean_norm = np.array([norms.mean()])
    parity.check_projections(pbar.cpu().numpy()[None, :], pbar_ref[None, :], mean_norm, d, m, what + " pbar")
    assert torch.equal(pbar, pbar2), "core_round and core_compress_batched disagree on pbar"
    # reconstruction alone, fed the oracle's pbar rounded to fp32
    gt_ref32 = oracle.reconstruct(seed, rnd, pbar_ref.astype(np.float32), 1.0 / m, 0, d)
    parity.check_gtilde(gt_recon.cpu().numpy(), gt_ref32, what + " reconstruct-only")
    # end to end
    if np.linalg.norm(gt_ref) > 0:
        parity.check_gtilde(gt.cpu().numpy(), gt_ref, what + " end-to-end")
    else:
        assert float(gt.abs().max()) == 0.0
    return P, pbar, gt


def test_config1_single_round():
    case = workloads.config1(DEV)
    _say("config1 d=1024 m=16 n=4 fp32")
    _run_and_check(case.seed, 0, case.G, case.m, what="config1")


SHAPES = [
    # d, m, n
    (1, 1, 1), (2, 3, 2), (3, 1, 3), (4, 2, 1), (5, 2, 1), (7, 5, 4), (8, 4, 2),
    (255, 16, 5), (256, 63, 8), (257, 64, 9), (1023, 65, 16), (1025, 255, 17),
    (4099, 257, 3), (5000, 300, 20), (20000, 1, 7), (70001, 513, 2), (12345, 1030, 33),
    (3000, 130, 32), (2500, 70, 29), (2000, 65, 50), (1500, 64, 64),   # wide passes: up to 64 clients
    (1500, 70, 44), (1300, 66, 47), (1100, 64, 55), (1000, 129, 58), (900, 65, 130),
]


@pytest.fixture(params=["default", "valu", "mfma", "q", "small"])
def variant(request):
    """Run a test once per projection kernel: the library's own choice, and each forced one."""
    core.core_debug_set_projection(request.param)
    yield request.param
    core.core_debug_set_projection("default")


@pytest.mark.parametrize("d,m,n", SHAPES)
def test_ragged_shapes_fp32(d, m, n, variant):
    _say(f"ragged fp32 d={d} m={m} n={n} variant={variant}")
    rng = np.random.default_rng(1000 * d + 10 * m + n)
    G = torch.from_numpy(rng.standard_normal((n, d)).astype(np.float32)).to(DEV)
    _run_and_check(31 + d, m + n, G, m, what=f"d={d} m={m} n={n}")


@pytest.mark.parametrize("d,m,n", [(5, 2, 1), (256, 64, 8), (1027, 70, 5), (9001, 260, 16), (40000, 33, 18)])
def test_ragged_shapes_bf16(d, m, n, variant):
    _say(f"ragged bf16 d={d} m={m} n={n} variant={variant}")
    rng = np.random.default_rng(7000 * d + 10 * m + n)
    G = torch.from_numpy(rng.standard_normal((n, d)).astype(np.float32)).to(DEV).to(torch.bfloat16)
    _run_and_check(77, d, G, m, what=f"bf16 d={d} m={m} n={n}")


def test_padded_rows_and_unaligned_views():
    """ld > d, rows starting at odd elements, and a gtilde that is only 4-byte aligned."""
    d, m, n, ld = 3001, 40, 3, 3100
    _say(f"strided d={d} m={m} n={n} ld={ld}")
    rng = np.random.default_rng(5)
    big = torch.from_numpy(rng.standard_normal((n, ld + 1)).astype(np.float32)).to(DEV)
    G = big[:, 1:]                      # [n, ld], row stride ld+1, base offset by one element
    assert G.stride(0) == ld + 1 and G.data_ptr() % 16 != 0
    G_host = G[:, :d].cpu().numpy()
    P_ref, pbar_ref, gt_ref = oracle.core_round(3, 9, np.ascontiguousarray(G_host), m)
    P, pbar = core.core_compress_batched(3, 9, G, m, d=d)
    buf = torch.zeros(d + 8, dtype=torch.float32, device=DEV)
    gt = buf[1:1 + d]
    assert gt.data_ptr() % 16 != 0
    core.core_round(3, 9, G, m, d=d, gtilde=gt)
    _sync()
    parity.check_projections(P.cpu().numpy(), P_ref, parity.row_norms(G_host), d, m, "strided")
    parity.check_gtilde(gt.cpu().numpy(), gt_ref, "strided")
    assert float(buf[0]) == 0.0 and float(buf[1 + d:].abs().max()) == 0.0, "wrote outside gtilde"


def test_single_vector_entry_point_and_scale():
    d, m = 6007, 129
    _say(f"core_compress d={d} m={m}")
    rng = np.random.default_rng(6)
    g = torch.from_numpy(rng.standard_normal(d).astype(np.float32)).to(DEV)
    p = core.core_compress(5, 2, g, m)
    P_ref = oracle.compress(5, 2, g.cpu().numpy()[None, :], m)
    _sync()
    parity.check_projections(p.cpu().numpy()[None, :], P_ref, parity.row_norms(g.cpu().numpy()[None, :]), d, m, "core_compress")
    # scale is applied as given: n/m on the mean is the sum-over-machines form of Algorithm 2
    a = core.core_reconstruct(5, 2, d, p, 1.0 / m)
    b = core.core_reconstruct(5, 2, d, p, 4.0 / m)
    _sync()
    np.testing.assert_allclose(b.cpu().numpy(), 4.0 * a.cpu().numpy(), rtol=1e-6, atol=0)


def test_zero_input_gives_zero():
    G = torch.zeros((3, 1000), dtype=torch.float32, device=DEV)
    pbar, gt = core.core_round(1, 0, G, 8)
    _sync()
    assert float(pbar.abs().max()) == 0.0 and float(gt.abs().max()) == 0.0


def test_results_are_reproducible_and_rounds_are_fresh():
    case = workloads.config1(DEV)
    ws = core.alloc_workspace(case.d, case.m, case.n)
    a = core.core_round(case.seed, 0, case.G, case.m, ws=ws)
    ws.fill_(255)  # stale scratch must not matter
    b = core.core_round(case.seed, 0, case.G, case.m, ws=ws)
    c = core.core_round(case.seed, 1, case.G, case.m, ws=ws)
    _sync()
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
    assert not torch.equal(a[0], c[0])
    # round r computed after other rounds equals round r computed cold
    d = core.core_round(case.seed, 1, case.G, case.m)
    _sync()
    assert torch.equal(c[0], d[0]) and torch.equal(c[1], d[1])


def test_client_mean_commutes_with_the_round():
    """Eq. (tildefdef): the round on n clients equals CORE of the mean gradient (up to fp32 rounding)."""
    rng = np.random.default_rng(8)
    d, m, n = 5000, 96, 6
    G = torch.from_numpy(rng.standard_normal((n, d)).astype(np.float32)).to(DEV)
    pbar, gt = core.core_round(4, 4, G, m)
    gm = G.double().mean(dim=0).float().contiguous()
    p1 = core.core_compress(4, 4, gm, m)
    _sync()
    assert parity.rel_l2(p1.cpu().numpy(), pbar.cpu().numpy()) < 5e-6


def test_many_clients_take_one_wide_pass_by_default():
    """More than 32 clients on a shape large enough for the lanes-over-vectors plan: the library's
    own choice is one generation of the normals for all 50 machines (Eq. (tildefdef): the same xi_j
    serve every machine), on chunks short enough for one level of fp32 sums."""
    d, m, n = 20000, 900, 50
    plan = core.core_debug_plan(d, m, n)
    assert plan["mode"] == 0 and plan["tiles_per_chunk"] <= 16
    _say(f"wide pass by default d={d} m={m} n={n}")
    rng = np.random.default_rng(50)
    G = torch.from_numpy(rng.standard_normal((n, d)).astype(np.float32)).to(DEV).to(torch.bfloat16)
    _run_and_check(9, 3, G, m, what=f"wide d={d} m={m} n={n}")


def test_estimator_moments_on_the_device():
    """Lemma 3.1 and the exact second moment from the proof of Lemma 3.2, checked on the HIP path
    itself over many rounds of fresh vectors (independent of the element-wise comparison with the
    oracle): E gtilde = gbar and E|gtilde - gbar|^2 = (d + 1)|gbar|^2 / m."""
    d, m, n, S = 24, 6, 3, 6000
    _say(f"estimator moments d={d} m={m} n={n} over {S} rounds")
    rng = np.random.default_rng(31)
    G_host = rng.standard_normal((n, d)).astype(np.float32)
    G = torch.from_numpy(G_host).to(DEV)
    gbar = G_host.astype(np.float64).mean(axis=0)
    ws = core.alloc_workspace(d, m, n)
    pbar = torch.empty(m, device=DEV)
    out = torch.empty((S, d), device=DEV)
    for r in range(S):
        core.core_round(5, r, G, m, pbar=pbar, gtilde=out[r], ws=ws)
    _sync()
    gt = out.double().cpu().numpy()
    # first moment: per-coordinate variance (|gbar|^2 + gbar_i^2)/m
    var_i = (gbar @ gbar + gbar ** 2) / m
    dev = np.abs(gt.mean(axis=0) - gbar) / np.sqrt(var_i / S)
    assert dev.max() < 4.5, dev.max()
    # second moment, with a confidence interval from the sample itself (heavy-tailed summand)
    sq = ((gt - gbar) ** 2).sum(axis=1)
    expect = (d + 1) * (gbar @ gbar) / m
    assert abs(sq.mean() - expect) < 4.5 * sq.std(ddof=1) / np.sqrt(S), (sq.mean(), expect)


def test_config3_full():
    case = workloads.config3(DEV)
    _say("config3 d=2^20 m=256 n=8 fp32 (oracle takes ~20 s)")
    _run_and_check(case.seed, 0, case.G, case.m, what="config3")


@pytest.mark.parametrize("d,m,n,bf16", [(5, 2, 1, False), (1030, 70, 3, False), (20001, 300, 8, True),
                                          (4096, 64, 20, False)])
def test_materialised_xi_variant(d, m, n, bf16):
    """The stored Xi holds the oracle's normals, and the round through it meets the same bars."""
    _say(f"materialised d={d} m={m} n={n} bf16={bf16}")
    rng = np.random.default_rng(d + m + n)
    G = torch.from_numpy(rng.standard_normal((n, d)).astype(np.float32)).to(DEV)
    if bf16:
        G = G.to(torch.bfloat16)
    G_host = workloads.to_host(G)
    P_ref, pbar_ref, gt_ref = oracle.core_round(19, 3, G_host, m)
    xi = core.alloc_xi(d, m)
    xi.fill_(float("nan"))
    P, pbar = core.core_compress_batched_store_xi(19, 3, G, m, xi)
    gt_from = core.core_reconstruct_from_xi(d, pbar, 1.0 / m, xi)
    xi2 = core.alloc_xi(d, m)
    pbar2, gt = core.core_round_materialized(19, 3, G, m, xi2)
    pbar3, gt3 = core.core_round(19, 3, G, m)
    _sync()
    # stored normals against the oracle, entry by entry on sampled vectors
    xi_h = xi.cpu().numpy()
    for j in sorted(set([0, m - 1, m // 2])):
        ref = oracle.xi_range(19, 3, j, 0, d)
        got = xi_h[:, j, :].reshape(-1)[:d].astype(np.float64)
        assert np.abs(got - ref).max() <= parity.XI_MAX_ABS
    assert torch.equal(xi, xi2)
    norms = parity.row_norms(G_host)
    parity.check_projections(P.cpu().numpy(), P_ref, norms, d, m, "materialised P")
    assert torch.equal(pbar, pbar2)
    # the regenerating round may use another projection kernel (summation order differs)
    assert parity.rel_l2(pbar3.cpu().numpy(), pbar.cpu().numpy()) < 2e-6
    parity.check_gtilde(gt.cpu().numpy(), gt_ref, "materialised end-to-end")
    assert torch.equal(gt, gt_from)
    # and it agrees with the regenerating path to fp32 rounding
    assert parity.rel_l2(gt.cpu().numpy(), gt3.cpu().numpy()) < 2e-6


@pytest.mark.parametrize("d,m,n,bf16", [(1030, 70, 3, False), (5000, 300, 8, True), (9001, 260, 16, True),
                                          (4100, 64, 21, False), (3000, 129, 11, True)])
def test_mfma_projection_variant(d, m, n, bf16):
    """The matrix-pipe A/B variant of the projection meets the same bars as the default kernel."""
    _say(f"mfma variant d={d} m={m} n={n} bf16={bf16}")
    rng = np.random.default_rng(3 * d + m + n)
    G = torch.from_numpy(rng.standard_normal((n, d)).astype(np.float32)).to(DEV)
    if bf16:
        G = G.to(torch.bfloat16)
    try:
        core.core_debug_set_projection("mfma")
        P, pbar, gt = _run_and_check(23, 5, G, m, what=f"mfma d={d} m={m} n={n}")
        core.core_debug_set_projection("valu")
        P2, pbar2 = core.core_compress_batched(23, 5, G, m)
        _sync()
    finally:
        core.core_debug_set_projection("default")
    assert parity.rel_l2(P.cpu().numpy(), P2.cpu().numpy()) < 2e-6


@pytest.mark.parametrize("d,m", [(5, 3), (4096, 64), (10007, 130)])
def test_fused_optimiser_step(d, m):
    """x_new = y - h * gtilde and y_next = x_new + (1-beta)(x_new - x_cur) in the kernel epilogue
    (last line of the loop of Algorithm 2; the two update lines of CORE-AGD)."""
    _say(f"fused update d={d} m={m}")
    rng = np.random.default_rng(d + m)
    pbar = rng.standard_normal(m).astype(np.float32)
    y = rng.standard_normal(d).astype(np.float32)
    xc = rng.standard_normal(d).astype(np.float32)
    h, omb, scale = 0.37, 0.8, 1.0 / m
    gt_ref = oracle.reconstruct(8, 2, pbar, scale, 0, d)
    xn_ref = y.astype(np.float64) - h * gt_ref
    yn_ref = xn_ref + omb * (xn_ref - xc.astype(np.float64))
    step = np.linalg.norm(h * gt_ref)

    def close(got, ref):
        return np.linalg.norm(got.cpu().numpy().astype(np.float64) - ref) <= 1e-5 * step + 2e-7 * np.linalg.norm(ref)

    pb = torch.from_numpy(pbar).to(DEV)
    yd, xcd = torch.from_numpy(y).to(DEV), torch.from_numpy(xc).to(DEV)
    # plain step, separate output, gtilde also written
    xn = torch.empty(d, dtype=torch.float32, device=DEV)
    gt = torch.empty(d, dtype=torch.float32, device=DEV)
    core.core_reconstruct_update(8, 2, pb, scale, h, yd, xn, gtilde=gt)
    _sync()
    parity.check_gtilde(gt.cpu().numpy(), gt_ref, "fused gtilde")
    assert close(xn, xn_ref)
    assert torch.equal(yd, torch.from_numpy(y).to(DEV)), "y must not be modified"
    # in place, no gtilde
    y2 = yd.clone()
    core.core_reconstruct_update(8, 2, pb, scale, h, y2, y2)
    _sync()
    assert torch.equal(y2, xn)
    # heavy-ball: y_next written over x_cur, x_new over y; and from 4-byte-aligned views
    buf = torch.zeros(3 * (d + 4) + 3, dtype=torch.float32, device=DEV)
    y3 = buf[1:1 + d]; y3.copy_(yd)
    c3 = buf[d + 6:2 * d + 6]; c3.copy_(xcd)
    core.core_reconstruct_update(8, 2, pb, scale, h, y3, y3, x_cur=c3, one_minus_beta=omb, y_next=c3)
    _sync()
    assert close(y3, xn_ref) and close(c3, yn_ref)
    # the same through aligned, distinct buffers
    xn4 = torch.empty_like(yd); yn4 = torch.empty_like(yd)
    core.core_reconstruct_update(8, 2, pb, scale, h, yd, xn4, x_cur=xcd, one_minus_beta=omb, y_next=yn4)
    _sync()
    assert torch.equal(xn4, xn) and close(yn4, yn_ref)
    assert torch.equal(yn4, c3) and torch.equal(xn4, y3)
    # bad combinations are refused
    with pytest.raises(core.CoreError):
        core.core_reconstruct_update(8, 2, pb, scale, h, yd, xn4, x_cur=xcd, one_minus_beta=omb, y_next=None)
    with pytest.raises(core.CoreError):
        core.core_reconstruct_update(8, 2, pb, scale, h, yd, xn4, x_cur=xcd, one_minus_beta=omb, y_next=xn4)


def _random_shapes(count, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        d = int(rng.choice([rng.integers(1, 40), rng.integers(40, 3000), rng.integers(3000, 40000)]))
        m = int(rng.choice([rng.integers(1, 20), rng.integers(20, 300), rng.integers(300, 800)]))
        n = int(rng.choice([rng.integers(1, 9), rng.integers(9, 17), rng.integers(17, 40)]))
        out.append((d, m, n, bool(rng.integers(0, 2)), int(rng.integers(0, 6))))
    return out


@pytest.mark.parametrize("d,m,n,bf16,pad", _random_shapes(24, 2024))
def test_random_shapes(d, m, n, bf16, pad, variant):
    """Seeded random shapes, both input types, padded rows: every kernel template and tail."""
    _say(f"random shape d={d} m={m} n={n} bf16={bf16} pad={pad} variant={variant}")
    rng = np.random.default_rng(d * 131 + m * 17 + n)
    full = torch.from_numpy((rng.standard_normal((n, d + pad)) * rng.uniform(1e-3, 10.0)).astype(np.float32)).to(DEV)
    if bf16:
        full = full.to(torch.bfloat16)
    G = full[:, :d] if pad else full
    assert G.stride(0) == d + pad
    _run_and_check(1000 + d, m * n, G, m, d=d, what=f"random d={d} m={m} n={n}")


def _random_long_shapes(count, seed):
    """Shapes with enough work for the lanes-over-vectors plans (tiles of 256, 64 and 8 / 16 / 32 vectors
    in every combination), small enough for the oracle: d m (n + 1) <= 2e8."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        d = int(rng.integers(60_000, 400_000))
        m = int(rng.choice([rng.integers(5, 64), rng.integers(64, 256), rng.integers(256, 700)]))
        n = int(rng.choice([1, 2, 3, 5, 8, 9, 17]))
        if -(-m // 64) * -(-d // 256) <= 1024 or d * m * (n + 1) > 2e8:
            continue
        out.append((d, m, n, bool(rng.integers(0, 2)), int(rng.integers(0, 6))))
    return out


@pytest.mark.parametrize("d,m,n,bf16,pad", _random_long_shapes(14, 77))
def test_random_long_shapes(d, m, n, bf16, pad):
    """Seeded random shapes on gradients long enough for the library to choose the lanes-over-vectors
    plans by itself, with whatever mix of tile sizes the vector count asks for; padded rows make some of
    them take the element-load paths."""
    plan = core.core_debug_plan(d, m, n)
    _say(f"random long shape d={d} m={m} n={n} bf16={bf16} pad={pad} plan={plan}")
    assert plan["mode"] == 0
    rng = np.random.default_rng(d * 131 + m * 17 + n)
    full = torch.from_numpy((rng.standard_normal((n, d + pad)) * rng.uniform(1e-3, 10.0)).astype(np.float32)).to(DEV)
    if bf16:
        full = full.to(torch.bfloat16)
    G = full[:, :d] if pad else full
    _run_and_check(2000 + d, m + n, G, m, d=d, what=f"random long d={d} m={m} n={n}")


def test_streams_and_graph_capture():
    """Entry points only enqueue on the given stream: they work on side streams, two streams with
    their own scratch can run at once, and a captured HIP graph replays to the eager result."""
    rng = np.random.default_rng(77)
    d, m, n = 30000, 300, 8
    _say(f"streams/graph d={d} m={m} n={n}")
    G = torch.from_numpy(rng.standard_normal((n, d)).astype(np.float32)).to(DEV)
    ws0 = core.alloc_workspace(d, m, n)
    ref_pbar, ref_gt = core.core_round(5, 1, G, m, ws=ws0)
    ref_pbar2, ref_gt2 = core.core_round(5, 2, G, m, ws=ws0)
    _sync()
    # two side streams, each with its own scratch and outputs
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    ws1, ws2 = core.alloc_workspace(d, m, n), core.alloc_workspace(d, m, n)
    out1 = (torch.empty(m, device=DEV), torch.empty(d, device=DEV))
    out2 = (torch.empty(m, device=DEV), torch.empty(d, device=DEV))
    for _ in range(3):
        with torch.cuda.stream(s1):
            core.core_round(5, 1, G, m, pbar=out1[0], gtilde=out1[1], ws=ws1)
        with torch.cuda.stream(s2):
            core.core_round(5, 2, G, m, pbar=out2[0], gtilde=out2[1], ws=ws2)
    _sync()
    assert torch.equal(out1[0], ref_pbar) and torch.equal(out1[1], ref_gt)
    assert torch.equal(out2[0], ref_pbar2) and torch.equal(out2[1], ref_gt2)
    # graph capture: no allocation, no synchronisation, no memset nodes inside the library
    gp, gg = torch.empty(m, device=DEV), torch.empty(d, device=DEV)
    x = torch.zeros(d, device=DEV)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        core.core_round(5, 1, G, m, pbar=gp, gtilde=gg, ws=ws1)
        core.core_reconstruct_update(5, 1, gp, 1.0 / m, 0.5, x, x)
    for rep in range(3):
        gp.zero_(); gg.zero_()
        x.fill_(1.0)
        torch.cuda.synchronize()
        graph.replay()
        # eager work between replays
        tmp = (G.float() * 2).sum()
        torch.cuda.synchronize()
        assert torch.equal(gp, ref_pbar) and torch.equal(gg, ref_gt), f"replay {rep}"
        assert parity.rel_l2((1.0 - x).cpu().numpy(), 0.5 * ref_gt.cpu().numpy()) < 1e-5
        assert bool(torch.isfinite(tmp))


@pytest.mark.parametrize("d,m,n,bf16", [
    (60000, 320, 8, False),     # one tile of 256 vectors + one tile of 64
    (40000, 600, 3, True),      # 512 + 64 + 24 as three tiles of 8
    (53000, 257, 16, True),     # 256 on the matrix pipe + 1 (a tile of 8), the tile in two passes of 8 clients
    (24000, 1100, 40, True),    # wide pass (chunks of 16 tiles) + 64 + 12 (a tile of 16), 40 clients in passes
    (300000, 130, 2, False),    # two tiles of 64 + 2 (a tile of 8)
    (66000, 200, 4, False),     # 200 vectors: one block of 256, all four waves busy
    (70001, 513, 2, False),     # 512 + 1
    (270000, 49, 5, True),      # seven tiles of 8
    (270000, 48, 5, True),      # three tiles of 16
    (270001, 32, 8, True),      # one tile of 32, rows not a multiple of 4: element loads
    (270000, 17, 3, False),     # three tiles of 8, the last with one vector
    (1300000, 5, 1, False),     # one tile of 8 with 5 vectors
    (90000, 190, 20, False),    # three tiles of 64 (the last with 62 lanes), 20 clients in passes of 16
    (40000, 447, 7, True),      # 256 + 2 x 64 + 63 (a full tile of 64: nothing pads less)
    (200000, 100, 9, True),     # 64 + 36 as five tiles of 8, 9 clients: passes of 8 + 1 in the small tiles
])
def test_ragged_vector_counts_split_between_the_projections(d, m, n, bf16):
    """Vector counts that are not multiples of 256, on shapes with enough work for the
    lanes-over-vectors plan: the library's own choice gives whole tiles of 256 to blocks of four
    waves, whole waves of the rest to blocks of 64 vectors whose waves share the chunk, and what is left
    to blocks of 8, 16 or 32 vectors whose lanes split between vectors and Philox blocks; all launches
    write the same per-chunk partial sums."""
    plan = core.core_debug_plan(d, m, n)
    _say(f"ragged vector count d={d} m={m} n={n} bf16={bf16} plan={plan}")
    assert plan["mode"] == 0
    rng = np.random.default_rng(d + 3 * m + n)
    G = torch.from_numpy(rng.standard_normal((n, d)).astype(np.float32)).to(DEV)
    if bf16:
        G = G.to(torch.bfloat16)
    _run_and_check(61, 2, G, m, what=f"ragged m d={d} m={m} n={n}")


@pytest.mark.parametrize("d,m,n", [(300, 20000, 2), (2000, 5, 100), (20000, 2100, 1)])
def test_extreme_aspect_ratios(d, m, n, variant):
    """Many vectors on a short gradient, many clients (several passes), one client on a long one."""
    _say(f"aspect d={d} m={m} n={n} variant={variant}")
    rng = np.random.default_rng(d + m + n)
    G = torch.from_numpy(rng.standard_normal((n, d)).astype(np.float32)).to(DEV)
    _run_and_check(404, 7, G, m, what=f"aspect d={d} m={m} n={n}")


@pytest.mark.parametrize("scale", [1e30, 1e-30, 1e-38])
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_value_ranges(scale, dtype, variant):
    """Very large and very small gradient entries (down to the edge of the normal range, where
    some entries and many partial sums are subnormal): fp32 arithmetic must neither overflow nor
    flush to zero; the usual bars hold because they are relative to |g|."""
    d, m, n = 3001, 70, 3
    _say(f"value range scale={scale} {dtype} variant={variant}")
    rng = np.random.default_rng(17)
    G32 = (rng.standard_normal((n, d)) * scale).astype(np.float32)
    G = torch.from_numpy(G32).to(DEV).to(dtype)
    assert float(G.float().abs().max()) > 0.0
    _run_and_check(77, 3, G, m, what=f"scale {scale} {dtype}")


def test_subnormal_gradients_are_not_flushed(variant):
    """Every entry subnormal (|g| ~ 1.6e-40): sums carry only the ~16 bits a subnormal of that size
    has, so the usual bars cannot hold, but a flush to zero anywhere (inputs, products or sums)
    would leave an error of order one.  Require 1e-3 of |g|."""
    d, m, n = 3001, 70, 3
    _say(f"subnormal gradients variant={variant}")
    rng = np.random.default_rng(18)
    G32 = (rng.standard_normal((n, d)) * 3e-42).astype(np.float32)
    G = torch.from_numpy(G32).to(DEV)
    norms = parity.row_norms(G32)
    assert norms.min() > 0.0
    P_ref, pbar_ref, gt_ref = oracle.core_round(5, 1, G32, m)
    P, pbar = core.core_compress_batched(5, 1, G, m)
    _, gt = core.core_round(5, 1, G, m)
    _sync()
    err = np.abs(P.cpu().numpy().astype(np.float64) - P_ref) / norms[:, None]
    assert err.max() < 1e-3, f"normalised projection error {err.max():.3e}"
    assert parity.rel_l2(gt.cpu().numpy(), gt_ref) < 1e-3


def test_host_threads_with_their_own_streams():
    """The library keeps no shared mutable state: host threads that call it at the same time, each
    on its own stream with its own scratch and outputs, get the single-thread results bit for bit."""
    import threading
    rng = np.random.default_rng(78)
    d, m, n, nthreads, rounds = 20000, 200, 4, 4, 8
    _say(f"host threads d={d} m={m} n={n} threads={nthreads}")
    G = torch.from_numpy(rng.standard_normal((n, d)).astype(np.float32)).to(DEV)
    ws0 = core.alloc_workspace(d, m, n)
    refs = []
    for r in range(rounds):
        pb, gt = core.core_round(9, r, G, m, ws=ws0)
        refs.append((pb.clone(), gt.clone()))
    _sync()
    results = [None] * nthreads
    errors = []

    def worker(t):
        try:
            torch.cuda.set_device(0)
            stream = torch.cuda.Stream()
            ws = core.alloc_workspace(d, m, n)
            outs = []
            with torch.cuda.stream(stream):
                for r in range(rounds):
                    pb = torch.empty(m, device=DEV)
                    gt = torch.empty(d, device=DEV)
                    core.core_round(9, r, G, m, pbar=pb, gtilde=gt, ws=ws)
                    outs.append((pb, gt))
            stream.synchronize()
            results[t] = outs
        except Exception as exc:   # surfaced in the main thread below
            errors.append(exc)

    threads = [threading.Thread(target=worker, args=(t,)) for t in range(nthreads)]
    for th in threads:
        th.start()
    for th in threads:
        th.join(timeout=100)
        assert not th.is_alive(), "worker did not finish"
    assert not errors, errors
    _sync()
    for t in range(nthreads):
        for r in range(rounds):
            assert torch.equal(results[t][r][0], refs[r][0]) and torch.equal(results[t][r][1], refs[r][1]), (t, r)


@pytest.mark.parametrize("d,m,nb,pad", [(1, 1, 1, 0), (4099, 7, 3, 0), (5000, 300, 4, 0), (20003, 65, 5, 5),
                                        (70001, 257, 8, 0), (12345, 64, 9, 3), (3000, 1030, 17, 0)])
def test_batched_reconstruction(d, m, nb, pad):
    """nb machines reconstruct from their own projection vectors with one generation of the common
    vectors: every row against the oracle's single-vector reconstruction, with and without the
    fused step, on padded (strided) arrays."""
    _say(f"batched reconstruction d={d} m={m} nb={nb} pad={pad}")
    rng = np.random.default_rng(d + m + nb)
    P_host = rng.standard_normal((nb, m)).astype(np.float32)
    X_host = rng.standard_normal((nb, d)).astype(np.float32)
    Pbuf = torch.zeros((nb, m + pad), device=DEV)
    Pbuf[:, :m] = torch.from_numpy(P_host).to(DEV)
    P = Pbuf[:, :m]
    Xbuf = torch.full((nb, d + pad), 7.0, device=DEV)
    Xbuf[:, :d] = torch.from_numpy(X_host).to(DEV)
    Gbuf = torch.full((nb, d + pad), -3.0, device=DEV)
    X, Gt = Xbuf[:, :d], Gbuf[:, :d]
    seed, rnd, scale, h = 21, 4, nb / m, 0.25
    core.core_reconstruct_update_batched(seed, rnd, P, scale, h, X, Gt)
    Gonly = torch.zeros((nb, d), device=DEV)
    core.core_reconstruct_update_batched(seed, rnd, P, scale, 0.0, None, Gonly)
    Xonly = torch.from_numpy(X_host).to(DEV)
    core.core_reconstruct_update_batched(seed, rnd, P, scale, h, Xonly, None)
    _sync()
    assert torch.equal(Gonly, Gt.contiguous()) and torch.equal(Xonly, X.contiguous())
    if pad:
        assert float((Xbuf[:, d:] - 7.0).abs().max()) == 0.0 and float((Gbuf[:, d:] + 3.0).abs().max()) == 0.0
    for v in range(nb):
        ref = oracle.reconstruct(seed, rnd, P_host[v].astype(np.float64), scale, 0, d)
        parity.check_gtilde(Gt[v].cpu().numpy(), ref, f"row {v}")
        step = X_host[v].astype(np.float64) - X[v].cpu().numpy().astype(np.float64)
        assert np.linalg.norm(step - h * ref) <= 1e-5 * np.linalg.norm(h * ref) + 1.2e-7 * np.linalg.norm(X_host[v])
    # one row through the single-vector entry point: same values up to the order of two roundings
    single = core.core_reconstruct(seed, rnd, d, P[0].contiguous(), scale)
    _sync()
    assert parity.rel_l2(single.cpu().numpy(), Gt[0].cpu().numpy()) < 1e-6
