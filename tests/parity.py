"""Tolerances and comparison helpers shared by the GPU parity tests.

Bars (fp32 device arithmetic against the fp64 oracle):
  - Philox words: bit-exact.
  - projections: |p_gpu - p_ref| <= 1e-4 * |g| * sqrt(d) * max(1, 1/sqrt(m)) element-wise (the
    stated bar), and additionally the error normalised by |g| (p/|g| is N(0,1)-sized) must have
    rms <= 3e-6 and max <= 2e-5 -- the level fp32 rounding plus the hardware log2/sqrt/sin/cos
    error (~1e-7 absolute on xi) actually supports, so that the end-to-end bar below can hold.
  - reconstruction: relative L2 error <= 1e-5.
"""
import numpy as np

P_ABS_FACTOR = 1e-4
P_NORMALISED_RMS = 3e-6
P_NORMALISED_MAX = 2e-5
GTILDE_REL_L2 = 1e-5
XI_MAX_ABS = 4e-6
XI_RMS_ABS = 5e-7


def row_norms(G_host):
    """fp64 Euclidean norm of each client's vector as stored (uint16 = bf16 bit patterns)."""
    G = np.asarray(G_host)
    if G.dtype == np.uint16:
        G = (G.astype(np.uint32) << 16).view(np.float32)
    return np.sqrt((G.astype(np.float64) ** 2).sum(axis=1))


def check_projections(P_gpu, P_ref, norms, d, m, what=""):
    """P_* are [n, k]; norms [n]."""
    P_gpu = np.asarray(P_gpu, dtype=np.float64)
    err = np.abs(P_gpu - P_ref)
    bound = P_ABS_FACTOR * norms[:, None] * np.sqrt(d) * max(1.0, 1.0 / np.sqrt(m))
    assert np.all(err <= bound), f"{what}: projection outside the stated bar, worst {np.max(err / bound):.3e}x"
    safe = np.where(norms > 0, norms, 1.0)[:, None]
    nerr = err / safe
    rms = float(np.sqrt(np.mean(nerr ** 2)))
    mx = float(nerr.max())
    assert rms <= P_NORMALISED_RMS, f"{what}: normalised projection error rms {rms:.3e}"
    assert mx <= P_NORMALISED_MAX, f"{what}: normalised projection error max {mx:.3e}"
    return rms, mx


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    den = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / den) if den > 0 else float(np.linalg.norm(a - b))


def check_gtilde(gt_gpu, gt_ref, what=""):
    r = rel_l2(gt_gpu, gt_ref)
    assert r <= GTILDE_REL_L2, f"{what}: reconstruction relative L2 error {r:.3e}"
    return r
