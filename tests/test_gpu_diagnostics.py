"""Diagnostics of the privacy appendix on the GPU against the oracle.

`core_projection_sqnorms` on projections the library itself produced and on synthetic rows
(element by element against the oracle's exactly rounded sums), the law of the lemma on C(a) on
the device (the squared norm of one machine's message over the squared norm of its gradient is
chi-square with m degrees of freedom), and the argument checks that need a device pointer.
"""
import ctypes
import math
import sys

import numpy as np
import pytest
import torch
from scipy import stats

from oracle import diagnostics as odg
import paper_2309_13307_amd as core
from paper_2309_13307_amd import binding, workloads

pytestmark = pytest.mark.gpu

# fp64 sums of exact products in a different order than the oracle's exactly rounded sum:
# at most m roundings of 2^-53 each, relative to a sum of non-negative terms
SQ_REL = 1e-12


def _say(msg):
    print(f"[case] {msg}", flush=True)
    sys.stdout.flush()


@pytest.mark.parametrize("n,m", [(1, 1), (1, 255), (3, 256), (8, 257), (5, 1000), (16, 4096), (2, 70001)])
def test_sqnorms_match_oracle(n, m):
    _say(f"sqnorms n={n} m={m}")
    rng = np.random.default_rng(100 * n + m)
    P = (rng.standard_normal((n, m)) * 10.0 ** rng.uniform(-3, 3, size=(n, 1))).astype(np.float32)
    if n > 1:
        P[1] = 0.0                                       # a machine whose gradient vanished
    sq = torch.full((n,), float("nan"), dtype=torch.float64, device="cuda")
    core.core_projection_sqnorms(torch.from_numpy(P).cuda(), sq)
    torch.cuda.synchronize()
    want = odg.projection_sqnorms(P)
    got = sq.cpu().numpy()
    assert np.all(np.abs(got - want) <= SQ_REL * want), (got, want)
    if n > 1:
        assert got[1] == 0.0


def test_sqnorms_of_library_projections_follow_the_lemma():
    """sq[c] / |g_c|^2 ~ chi^2_m for the messages core_compress_batched produces."""
    case = workloads.config2_round("cuda")              # d = 4096, n = 8 gradient-like rows
    m = 512
    G_host = workloads.to_host(case.G).astype(np.float64)
    na2 = (G_host * G_host).sum(axis=1)
    ratios = []
    sq = torch.empty(case.n, dtype=torch.float64, device="cuda")
    for rnd in range(40):
        _say(f"lemma on the device, round {rnd}") if rnd % 10 == 0 else None
        P, _ = core.core_compress_batched(case.seed, rnd, case.G, m)
        core.core_projection_sqnorms(P, sq)
        torch.cuda.synchronize()
        want = odg.projection_sqnorms(P.cpu().numpy())
        got = sq.cpu().numpy()
        assert np.all(np.abs(got - want) <= SQ_REL * want)
        ratios.append(got / na2)
    ratios = np.concatenate(ratios)                     # 320 samples; rows of a round share Xi, rounds do not
    S = ratios.size
    assert abs(ratios.mean() - m) < 5.0 * math.sqrt(2.0 * m / 40)       # 40 independent rounds at least
    # every sample inside the central 1 - 1e-6 mass of chi^2_m
    lo, hi = stats.chi2.ppf([5e-7, 1 - 5e-7], m)
    assert ratios.min() > lo and ratios.max() < hi, (ratios.min(), ratios.max(), lo, hi, S)


def test_sqnorms_argument_checks():
    L = core.load_library()
    P = torch.zeros((4, 64), device="cuda")
    sq = torch.zeros(4, dtype=torch.float64, device="cuda")
    E = binding
    assert L.core_projection_sqnorms(64, 4, None, sq.data_ptr(), None) == E.ERR_INVALID_ARGUMENT
    assert L.core_projection_sqnorms(64, 4, P.data_ptr(), None, None) == E.ERR_INVALID_ARGUMENT
    assert L.core_projection_sqnorms(0, 4, P.data_ptr(), sq.data_ptr(), None) == E.ERR_INVALID_ARGUMENT
    assert L.core_projection_sqnorms(64, 0, P.data_ptr(), sq.data_ptr(), None) == E.ERR_INVALID_ARGUMENT
    assert L.core_projection_sqnorms(64, 4, P.data_ptr(), P.data_ptr() + 8, None) == E.ERR_INVALID_ARGUMENT
    assert L.core_projection_sqnorms(63, 4, P.data_ptr() + 2, sq.data_ptr(), None) == E.ERR_MISALIGNED
    assert L.core_projection_sqnorms(64, 4, P.data_ptr(), sq.data_ptr() + 4, None) == E.ERR_MISALIGNED
    with pytest.raises(ValueError):
        core.core_projection_sqnorms(P, torch.zeros(3, dtype=torch.float64, device="cuda"))
    with pytest.raises(ValueError):
        core.core_projection_sqnorms(P.t(), sq)
    torch.cuda.synchronize()
