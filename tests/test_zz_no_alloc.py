"""The entry point that allocates nothing (`core_round_static`): through the C ABI, against
`core_round` with a caller workspace, on two calls in a row, the second with a smaller input, so
that whatever the first call left in the library's fixed scratch array is still there."""
import sys

import numpy as np
import pytest
import torch

import oracle
import paper_2309_13307_amd as core
from paper_2309_13307_amd import binding, workloads
import parity

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _say(msg):
    print(f"[case] {msg}", flush=True)
    sys.stdout.flush()


def test_static_scratch_round_matches_core_round():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    L = core.load_library()
    # first call: the ResNet-50-sized case, which uses 68 MB of the 80 MiB array
    big = workloads.config4(DEV)
    need = core.core_workspace_bytes(big.d, big.m, big.n)
    assert 0 < need <= binding.STATIC_SCRATCH_BYTES
    rng = np.random.default_rng(12)
    small_G = torch.from_numpy(rng.standard_normal((3, 4099)).astype(np.float32)).to(DEV)
    cases = [("ResNet-50-sized", big.seed, 3, big.G, big.m), ("small, after the large one", 6, 2, small_G, 70)]
    for what, seed, rnd, G, m in cases:
        n, d = G.shape
        _say(f"core_round_static {what}: d={d} m={m} n={n}")
        ref_pbar, ref_gt = core.core_round(seed, rnd, G, m)              # caller-owned workspace
        pbar = torch.full((m,), float("nan"), device=DEV)
        gt = torch.full((d,), float("nan"), device=DEV)
        torch.cuda.synchronize()
        free_before, _ = torch.cuda.mem_get_info()
        rc = L.core_round_static(seed, rnd, d, m, n, G.data_ptr(), binding._dtype_code(G), G.stride(0),
                                 pbar.data_ptr(), gt.data_ptr(), torch.cuda.current_stream().cuda_stream)
        assert rc == 0, core.strerror(rc)
        torch.cuda.synchronize()
        # same kernels, same plan, same order of every sum: the two entry points agree bit for bit
        assert torch.equal(pbar, ref_pbar), what
        assert torch.equal(gt, ref_gt), what
        if what.startswith("small"):
            free_after, _ = torch.cuda.mem_get_info()
            assert free_after >= free_before, "the call must not take device memory"
            # and against the oracle, to the usual bars
            G_host = workloads.to_host(G)
            _, pbar_ref, gt_ref = oracle.core_round(seed, rnd, G_host, m)
            parity.check_projections(pbar.cpu().numpy()[None, :], pbar_ref[None, :],
                                     np.array([parity.row_norms(G_host).mean()]), d, m, what)
            parity.check_gtilde(gt.cpu().numpy(), gt_ref, what)
    # sizes beyond the fixed array are refused before anything is launched
    rc = L.core_round_static(1, 0, 124_439_808, 4096, 16, small_G.data_ptr(), 0, 124_439_808,
                             pbar.data_ptr(), gt.data_ptr(), None)
    assert rc == binding.ERR_STATIC_SCRATCH_TOO_SMALL
    assert "CORE_STATIC_SCRATCH_BYTES" in core.strerror(rc)
