"""ctypes binding of the C ABI in ``include/core.h``.

Argument marshalling only: every step of the path runs in the HIP kernels of
``libcore_hip.so``.  torch is used for device memory and the stream handle.  There is no
CPU fallback: if the library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os

import torch

from . import build as _build

DTYPE_F32 = 0
DTYPE_BF16 = 1

OK = 0
ERR_INVALID_ARGUMENT = -1
ERR_MISALIGNED = -2
ERR_WORKSPACE_TOO_SMALL = -3
ERR_HIP = -4
ERR_NO_DEVICE = -5
ERR_STATIC_SCRATCH_TOO_SMALL = -6
STATIC_SCRATCH_BYTES = 80 << 20

EXPORTS = (
    "core_strerror", "core_last_hip_error", "core_workspace_bytes", "core_compress",
    "core_compress_batched", "core_reconstruct", "core_round", "core_debug_philox", "core_debug_xi",
    "core_xi_bytes", "core_compress_batched_store_xi", "core_reconstruct_from_xi",
    "core_round_materialized", "core_reconstruct_update", "core_round_update",
    "core_projection_sqnorms", "core_privacy_loss",
    "core_nonconvex_step", "core_step_size_option2", "core_reconstruct_trial", "core_round_trial",
    "core_accept_trial", "core_debug_plan", "core_round_update_r", "core_advance_round",
    "core_round_trial_r", "core_reconstruct_update_batched", "core_build_id",
    "core_debug_philox_layout", "core_debug_set_projection", "core_round_static",
)


class CoreError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: {strerror(code)} (code {code})")


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libcore_hip.so.  A library built from the sources at hand is loaded as it is; a missing
    or stale one (its build id differs from the hash of the sources) is rebuilt first, and if there
    is no compiler to do that the call fails rather than run an outdated binary."""
    global _lib
    if _lib is not None:
        return _lib
    if _build.is_stale():
        have, want = _build.built_id(), _build.source_id()
        if not os.path.exists(_build.hipcc_path()):
            raise RuntimeError(f"libcore_hip.so is {'missing' if have is None else 'stale'} (build id {have}, "
                               f"sources {want}) and there is no hipcc to build it")
        _build.build_library()
    L = ctypes.CDLL(_build.LIB_PATH)
    u64, u32, i32, vp, sz, f32 = (ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int, ctypes.c_void_p,
                                  ctypes.c_size_t, ctypes.c_float)
    L.core_strerror.argtypes = [i32]
    L.core_strerror.restype = ctypes.c_char_p
    L.core_last_hip_error.argtypes = []
    L.core_last_hip_error.restype = i32
    L.core_workspace_bytes.argtypes = [u64, u32, u32]
    L.core_workspace_bytes.restype = sz
    L.core_compress.argtypes = [u64, u64, u64, u32, vp, i32, vp, vp, sz, vp]
    L.core_compress.restype = i32
    L.core_compress_batched.argtypes = [u64, u64, u64, u32, u32, vp, i32, u64, vp, vp, vp, sz, vp]
    L.core_compress_batched.restype = i32
    L.core_reconstruct.argtypes = [u64, u64, u64, u32, vp, f32, vp, vp]
    L.core_reconstruct.restype = i32
    L.core_round.argtypes = [u64, u64, u64, u32, u32, vp, i32, u64, vp, vp, vp, sz, vp]
    L.core_round.restype = i32
    L.core_round_static.argtypes = [u64, u64, u64, u32, u32, vp, i32, u64, vp, vp, vp]
    L.core_round_static.restype = i32
    L.core_xi_bytes.argtypes = [u64, u32]
    L.core_xi_bytes.restype = sz
    L.core_compress_batched_store_xi.argtypes = [u64, u64, u64, u32, u32, vp, i32, u64, vp, vp, vp, sz,
                                                 vp, sz, vp]
    L.core_compress_batched_store_xi.restype = i32
    L.core_reconstruct_from_xi.argtypes = [u64, u32, vp, f32, vp, sz, vp, vp]
    L.core_reconstruct_from_xi.restype = i32
    L.core_round_materialized.argtypes = [u64, u64, u64, u32, u32, vp, i32, u64, vp, vp, vp, sz, vp, sz, vp]
    L.core_round_materialized.restype = i32
    L.core_reconstruct_update.argtypes = [u64, u64, u64, u32, vp, f32, f32, vp, vp, vp, f32, vp, vp, vp]
    L.core_reconstruct_update.restype = i32
    L.core_round_update.argtypes = [u64, u64, u64, u32, u32, vp, i32, u64, vp, f32, vp, vp, vp, f32, vp, vp,
                                    vp, sz, vp]
    L.core_round_update.restype = i32
    f64 = ctypes.c_double
    L.core_projection_sqnorms.argtypes = [u32, u32, vp, vp, vp]
    L.core_projection_sqnorms.restype = i32
    L.core_privacy_loss.argtypes = [f64, u32, f64, f64, ctypes.POINTER(ctypes.c_double)]
    L.core_privacy_loss.restype = i32
    L.core_nonconvex_step.argtypes = [u64, u32, vp, f32, f64, f64, vp, vp, vp]
    L.core_nonconvex_step.restype = i32
    L.core_step_size_option2.argtypes = [u64, u32, f64, f64, f64, f64, ctypes.POINTER(f64)]
    L.core_step_size_option2.restype = i32
    L.core_reconstruct_trial.argtypes = [u64, u64, u64, u32, vp, f32, vp, vp, vp, vp, vp]
    L.core_reconstruct_trial.restype = i32
    L.core_round_trial.argtypes = [u64, u64, u64, u32, u32, vp, i32, u64, vp, f32, f64, f64, vp, vp, vp, vp,
                                   vp, vp, sz, vp]
    L.core_round_trial.restype = i32
    L.core_accept_trial.argtypes = [u64, vp, vp, vp, vp, vp, vp]
    L.core_accept_trial.restype = i32
    L.core_round_update_r.argtypes = [u64, vp, u64, u32, u32, vp, i32, u64, vp, f32, vp, vp, vp, f32, vp, vp,
                                      vp, sz, vp]
    L.core_round_update_r.restype = i32
    L.core_round_trial_r.argtypes = [u64, vp, u64, u32, u32, vp, i32, u64, vp, f32, f64, f64, vp, vp, vp, vp,
                                     vp, vp, sz, vp]
    L.core_round_trial_r.restype = i32
    L.core_reconstruct_update_batched.argtypes = [u64, u64, u64, u32, u32, vp, u64, f32, f32, vp, vp, u64, vp]
    L.core_reconstruct_update_batched.restype = i32
    L.core_advance_round.argtypes = [vp, vp]
    L.core_advance_round.restype = i32
    L.core_debug_plan.argtypes = [u64, u32, u32, ctypes.POINTER(u64)]
    L.core_debug_plan.restype = i32
    L.core_debug_philox.argtypes = [u64, u64, u32, u64, u64, vp, vp]
    L.core_debug_philox.restype = i32
    L.core_debug_philox_layout.argtypes = [i32, u64, u64, u32, u32, u64, u64, vp, vp]
    L.core_debug_philox_layout.restype = i32
    L.core_debug_set_projection.argtypes = [i32]
    L.core_debug_set_projection.restype = i32
    L.core_build_id.argtypes = []
    L.core_build_id.restype = ctypes.c_char_p
    L.core_debug_xi.argtypes = [u64, u64, u32, u64, u64, vp, vp]
    L.core_debug_xi.restype = i32
    _lib = L
    return L


def strerror(code: int) -> str:
    return load_library().core_strerror(code).decode()


def _check(code: int, what: str) -> None:
    if code != OK:
        raise CoreError(code, what)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return DTYPE_F32
    if t.dtype == torch.bfloat16:
        return DTYPE_BF16
    raise TypeError(f"G must be float32 or bfloat16, got {t.dtype}")


def _require_cuda(*tensors) -> None:
    for t in tensors:
        if t is not None and not t.is_cuda:
            raise ValueError("all tensors must live on the GPU")


def core_workspace_bytes(d: int, m: int, n: int) -> int:
    return int(load_library().core_workspace_bytes(d, m, n))


def alloc_workspace(d: int, m: int, n: int, device="cuda") -> torch.Tensor:
    nbytes = core_workspace_bytes(d, m, n)
    if nbytes == 0:
        raise CoreError(ERR_INVALID_ARGUMENT, "core_workspace_bytes")
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def core_compress(seed: int, rnd: int, g: torch.Tensor, m: int, p: torch.Tensor | None = None,
                  ws: torch.Tensor | None = None) -> torch.Tensor:
    """p[j] = <g, xi_j>.  g: [d] fp32/bf16 on the GPU."""
    _require_cuda(g, p, ws)
    if g.dim() != 1 or not g.is_contiguous():
        raise ValueError("g must be a contiguous 1-D tensor")
    d = g.numel()
    if p is None:
        p = torch.empty(m, dtype=torch.float32, device=g.device)
    if ws is None:
        ws = alloc_workspace(d, m, 1, g.device)
    rc = load_library().core_compress(seed, rnd, d, m, g.data_ptr(), _dtype_code(g), p.data_ptr(),
                                      ws.data_ptr(), ws.numel(), _stream())
    _check(rc, "core_compress")
    return p


def core_compress_batched(seed: int, rnd: int, G: torch.Tensor, m: int, d: int | None = None,
                          P: torch.Tensor | None = None, pbar: torch.Tensor | None = None,
                          ws: torch.Tensor | None = None, want_P: bool = True):
    """P[c, j] = <G[c, :d], xi_j>, pbar = mean over clients.  G: [n, ld] with unit inner stride."""
    _require_cuda(G, P, pbar, ws)
    if G.dim() != 2 or G.stride(1) != 1:
        raise ValueError("G must be 2-D with unit stride along the coordinate axis")
    n, ld = G.shape[0], G.stride(0)
    if d is None:
        d = G.shape[1]
    if P is None and want_P:
        P = torch.empty((n, m), dtype=torch.float32, device=G.device)
    if pbar is None:
        pbar = torch.empty(m, dtype=torch.float32, device=G.device)
    if ws is None:
        ws = alloc_workspace(d, m, n, G.device)
    rc = load_library().core_compress_batched(seed, rnd, d, m, n, G.data_ptr(), _dtype_code(G), ld,
                                              P.data_ptr() if P is not None else None,
                                              pbar.data_ptr(), ws.data_ptr(), ws.numel(), _stream())
    _check(rc, "core_compress_batched")
    return P, pbar


def core_reconstruct(seed: int, rnd: int, d: int, pbar: torch.Tensor, scale: float,
                     gtilde: torch.Tensor | None = None) -> torch.Tensor:
    """gtilde[i] = scale * sum_j pbar[j] xi_j[i]."""
    _require_cuda(pbar, gtilde)
    if pbar.dtype != torch.float32 or pbar.dim() != 1 or not pbar.is_contiguous():
        raise ValueError("pbar must be a contiguous 1-D float32 tensor")
    m = pbar.numel()
    if gtilde is None:
        gtilde = torch.empty(d, dtype=torch.float32, device=pbar.device)
    rc = load_library().core_reconstruct(seed, rnd, d, m, pbar.data_ptr(), scale, gtilde.data_ptr(),
                                         _stream())
    _check(rc, "core_reconstruct")
    return gtilde


def core_round(seed: int, rnd: int, G: torch.Tensor, m: int, d: int | None = None,
               pbar: torch.Tensor | None = None, gtilde: torch.Tensor | None = None,
               ws: torch.Tensor | None = None):
    """One CORE round on n batched clients: returns (pbar [m], gtilde [d])."""
    _require_cuda(G, pbar, gtilde, ws)
    if G.dim() != 2 or G.stride(1) != 1:
        raise ValueError("G must be 2-D with unit stride along the coordinate axis")
    n, ld = G.shape[0], G.stride(0)
    if d is None:
        d = G.shape[1]
    if pbar is None:
        pbar = torch.empty(m, dtype=torch.float32, device=G.device)
    if gtilde is None:
        gtilde = torch.empty(d, dtype=torch.float32, device=G.device)
    if ws is None:
        ws = alloc_workspace(d, m, n, G.device)
    rc = load_library().core_round(seed, rnd, d, m, n, G.data_ptr(), _dtype_code(G), ld,
                                   pbar.data_ptr(), gtilde.data_ptr(), ws.data_ptr(), ws.numel(),
                                   _stream())
    _check(rc, "core_round")
    return pbar, gtilde


def core_round_static(seed: int, rnd: int, G: torch.Tensor, m: int, pbar: torch.Tensor, gtilde: torch.Tensor,
                      d: int | None = None) -> None:
    """core_round with the scratch in the library's fixed array: the call allocates nothing, so
    both outputs must be supplied."""
    _require_cuda(G, pbar, gtilde)
    if G.dim() != 2 or G.stride(1) != 1:
        raise ValueError("G must be 2-D with unit stride along the coordinate axis")
    n, ld = G.shape[0], G.stride(0)
    if d is None:
        d = G.shape[1]
    rc = load_library().core_round_static(seed, rnd, d, m, n, G.data_ptr(), _dtype_code(G), ld,
                                          pbar.data_ptr(), gtilde.data_ptr(), _stream())
    _check(rc, "core_round_static")


def _ptr(t):
    return t.data_ptr() if t is not None else None


def core_reconstruct_update(seed: int, rnd: int, pbar: torch.Tensor, scale: float, h: float,
                            y: torch.Tensor, x_new: torch.Tensor, x_cur: torch.Tensor | None = None,
                            one_minus_beta: float = 0.0, y_next: torch.Tensor | None = None,
                            gtilde: torch.Tensor | None = None) -> None:
    """x_new = y - h * scale * sum_j pbar[j] xi_j; optionally y_next = x_new + (1-beta)(x_new - x_cur)."""
    _require_cuda(pbar, y, x_new, x_cur, y_next, gtilde)
    d, m = y.numel(), pbar.numel()
    rc = load_library().core_reconstruct_update(seed, rnd, d, m, pbar.data_ptr(), scale, h, y.data_ptr(),
                                                x_new.data_ptr(), _ptr(x_cur), one_minus_beta,
                                                _ptr(y_next), _ptr(gtilde), _stream())
    _check(rc, "core_reconstruct_update")


def core_round_update(seed: int, rnd: int, G: torch.Tensor, m: int, h: float, y: torch.Tensor,
                      x_new: torch.Tensor, pbar: torch.Tensor, ws: torch.Tensor,
                      x_cur: torch.Tensor | None = None, one_minus_beta: float = 0.0,
                      y_next: torch.Tensor | None = None, gtilde: torch.Tensor | None = None,
                      d: int | None = None) -> None:
    """One iteration of Algorithm 2 / CORE-AGD apart from the gradient evaluation."""
    _require_cuda(G, y, x_new, pbar, ws, x_cur, y_next, gtilde)
    if G.dim() != 2 or G.stride(1) != 1:
        raise ValueError("G must be 2-D with unit stride along the coordinate axis")
    n, ld = G.shape[0], G.stride(0)
    if d is None:
        d = G.shape[1]
    rc = load_library().core_round_update(seed, rnd, d, m, n, G.data_ptr(), _dtype_code(G), ld,
                                          pbar.data_ptr(), h, y.data_ptr(), x_new.data_ptr(), _ptr(x_cur),
                                          one_minus_beta, _ptr(y_next), _ptr(gtilde), ws.data_ptr(),
                                          ws.numel(), _stream())
    _check(rc, "core_round_update")


def core_nonconvex_step(d: int, pbar: torch.Tensor, c: float, r1: float, H: float,
                        p_out: torch.Tensor | None, h_out: torch.Tensor) -> None:
    """Option I of Algorithm 3: p_out = c * sqrt(mean pbar^2), h_out = the step size (device scalars)."""
    _require_cuda(pbar, p_out, h_out)
    rc = load_library().core_nonconvex_step(d, pbar.numel(), pbar.data_ptr(), c, r1, H, _ptr(p_out),
                                            h_out.data_ptr(), _stream())
    _check(rc, "core_nonconvex_step")


def core_step_size_option2(d: int, m: int, r1: float, H: float, L: float, Delta: float) -> float:
    """Option II of Algorithm 3 (host arithmetic, fp64)."""
    out = ctypes.c_double(0.0)
    rc = load_library().core_step_size_option2(d, m, r1, H, L, Delta, ctypes.byref(out))
    _check(rc, "core_step_size_option2")
    return out.value


def core_projection_sqnorms(P: torch.Tensor, sq: torch.Tensor) -> None:
    """sq[c] = sum_j P[c][j]^2 (fp64) for the projections P [n][m] of every machine."""
    _require_cuda(P, sq)
    if P.dim() != 2 or not P.is_contiguous() or P.dtype != torch.float32:
        raise ValueError("P must be a contiguous fp32 [n][m] tensor")
    if sq.dtype != torch.float64 or sq.numel() != P.shape[0] or not sq.is_contiguous():
        raise ValueError("sq must be a contiguous fp64 tensor of n elements")
    rc = load_library().core_projection_sqnorms(P.shape[1], P.shape[0], P.data_ptr(), sq.data_ptr(), _stream())
    _check(rc, "core_projection_sqnorms")


def core_privacy_loss(sqnorm: float, m: int, sigma1: float, sigma2: float) -> float:
    """Privacy loss of one released message (privacy appendix; host arithmetic, fp64)."""
    out = ctypes.c_double(0.0)
    rc = load_library().core_privacy_loss(sqnorm, m, sigma1, sigma2, ctypes.byref(out))
    _check(rc, "core_privacy_loss")
    return out.value


def core_reconstruct_trial(seed: int, rnd: int, pbar: torch.Tensor, scale: float, h: torch.Tensor,
                           x: torch.Tensor, x_trial: torch.Tensor, gtilde: torch.Tensor | None = None) -> None:
    """x_trial = x - h * scale * sum_j pbar[j] xi_j with the step h read from device memory."""
    _require_cuda(pbar, h, x, x_trial, gtilde)
    rc = load_library().core_reconstruct_trial(seed, rnd, x.numel(), pbar.numel(), pbar.data_ptr(), scale,
                                               h.data_ptr(), x.data_ptr(), x_trial.data_ptr(), _ptr(gtilde),
                                               _stream())
    _check(rc, "core_reconstruct_trial")


def core_round_trial(seed: int, rnd: int, G: torch.Tensor, m: int, c: float, r1: float, H: float,
                     x: torch.Tensor, x_trial: torch.Tensor, pbar: torch.Tensor, p_out: torch.Tensor | None,
                     h_out: torch.Tensor, ws: torch.Tensor, gtilde: torch.Tensor | None = None,
                     d: int | None = None) -> None:
    """One iteration of Algorithm 3 (Option I) between the gradient evaluation and f(x_trial)."""
    _require_cuda(G, x, x_trial, pbar, p_out, h_out, ws, gtilde)
    if G.dim() != 2 or G.stride(1) != 1:
        raise ValueError("G must be 2-D with unit stride along the coordinate axis")
    n, ld = G.shape[0], G.stride(0)
    if d is None:
        d = G.shape[1]
    rc = load_library().core_round_trial(seed, rnd, d, m, n, G.data_ptr(), _dtype_code(G), ld,
                                         pbar.data_ptr(), c, r1, H, _ptr(p_out), h_out.data_ptr(),
                                         x.data_ptr(), x_trial.data_ptr(), _ptr(gtilde), ws.data_ptr(),
                                         ws.numel(), _stream())
    _check(rc, "core_round_trial")


def core_accept_trial(f_cur: torch.Tensor, f_trial: torch.Tensor, x: torch.Tensor, x_trial: torch.Tensor,
                      accepted: torch.Tensor) -> None:
    """Comparison step of Algorithm 3: x <- x_trial and f_cur <- f_trial iff f_trial < f_cur."""
    _require_cuda(f_cur, f_trial, x, x_trial, accepted)
    if accepted.dtype != torch.int32:
        raise TypeError("accepted must be an int32 tensor")
    rc = load_library().core_accept_trial(x.numel(), f_cur.data_ptr(), f_trial.data_ptr(), x.data_ptr(),
                                          x_trial.data_ptr(), accepted.data_ptr(), _stream())
    _check(rc, "core_accept_trial")


def core_round_update_r(seed: int, round_dev: torch.Tensor, G: torch.Tensor, m: int, h: float, y: torch.Tensor,
                        x_new: torch.Tensor, pbar: torch.Tensor, ws: torch.Tensor,
                        x_cur: torch.Tensor | None = None, one_minus_beta: float = 0.0,
                        y_next: torch.Tensor | None = None, gtilde: torch.Tensor | None = None,
                        d: int | None = None) -> None:
    """core_round_update with the round counter read from the device tensor `round_dev` (int64, one
    element) when the kernels run; for iterations recorded into a HIP graph."""
    _require_cuda(round_dev, G, y, x_new, pbar, ws, x_cur, y_next, gtilde)
    if round_dev.dtype != torch.int64 or round_dev.numel() != 1:
        raise TypeError("round_dev must be a one-element int64 tensor")
    if G.dim() != 2 or G.stride(1) != 1:
        raise ValueError("G must be 2-D with unit stride along the coordinate axis")
    n, ld = G.shape[0], G.stride(0)
    if d is None:
        d = G.shape[1]
    rc = load_library().core_round_update_r(seed, round_dev.data_ptr(), d, m, n, G.data_ptr(), _dtype_code(G),
                                            ld, pbar.data_ptr(), h, y.data_ptr(), x_new.data_ptr(),
                                            _ptr(x_cur), one_minus_beta, _ptr(y_next), _ptr(gtilde),
                                            ws.data_ptr(), ws.numel(), _stream())
    _check(rc, "core_round_update_r")


def core_round_trial_r(seed: int, round_dev: torch.Tensor, G: torch.Tensor, m: int, c: float, r1: float,
                       H: float, x: torch.Tensor, x_trial: torch.Tensor, pbar: torch.Tensor,
                       p_out: torch.Tensor | None, h_out: torch.Tensor, ws: torch.Tensor,
                       gtilde: torch.Tensor | None = None, d: int | None = None) -> None:
    """core_round_trial with the round counter read from the device tensor `round_dev`."""
    _require_cuda(round_dev, G, x, x_trial, pbar, p_out, h_out, ws, gtilde)
    if round_dev.dtype != torch.int64 or round_dev.numel() != 1:
        raise TypeError("round_dev must be a one-element int64 tensor")
    if G.dim() != 2 or G.stride(1) != 1:
        raise ValueError("G must be 2-D with unit stride along the coordinate axis")
    n, ld = G.shape[0], G.stride(0)
    if d is None:
        d = G.shape[1]
    rc = load_library().core_round_trial_r(seed, round_dev.data_ptr(), d, m, n, G.data_ptr(), _dtype_code(G), ld,
                                           pbar.data_ptr(), c, r1, H, _ptr(p_out), h_out.data_ptr(),
                                           x.data_ptr(), x_trial.data_ptr(), _ptr(gtilde), ws.data_ptr(),
                                           ws.numel(), _stream())
    _check(rc, "core_round_trial_r")


def core_reconstruct_update_batched(seed: int, rnd: int, P: torch.Tensor, scale: float, h: float,
                                    X: torch.Tensor | None, Gt: torch.Tensor | None = None,
                                    d: int | None = None) -> None:
    """For every row v: g_v = scale * sum_j P[v][j] xi_j; Gt[v] = g_v and/or X[v] -= h * g_v."""
    _require_cuda(P, X, Gt)
    ref = X if X is not None else Gt
    if ref is None:
        raise ValueError("one of X, Gt is required")
    for t_ in (P, X, Gt):
        if t_ is not None and (t_.dim() != 2 or t_.stride(1) != 1 or t_.dtype != torch.float32):
            raise ValueError("P, X, Gt must be 2-D float32 with unit stride along the last axis")
    if X is not None and Gt is not None and (X.stride(0) != Gt.stride(0) or X.shape != Gt.shape):
        raise ValueError("X and Gt must have the same shape and row stride")
    nb, m = P.shape
    if d is None:
        d = ref.shape[1]
    rc = load_library().core_reconstruct_update_batched(seed, rnd, d, m, nb, P.data_ptr(), P.stride(0), scale, h,
                                                        _ptr(X), _ptr(Gt), ref.stride(0), _stream())
    _check(rc, "core_reconstruct_update_batched")


def core_advance_round(round_dev: torch.Tensor) -> None:
    """Enqueue round_dev += 1 on the current stream."""
    _require_cuda(round_dev)
    if round_dev.dtype != torch.int64 or round_dev.numel() != 1:
        raise TypeError("round_dev must be a one-element int64 tensor")
    _check(load_library().core_advance_round(round_dev.data_ptr(), _stream()), "core_advance_round")


def core_debug_plan(d: int, m: int, n: int) -> dict:
    """The projection launch plan for these sizes (host arithmetic only)."""
    out = (ctypes.c_uint64 * 10)()
    rc = load_library().core_debug_plan(d, m, n, out)
    _check(rc, "core_debug_plan")
    keys = ("mode", "jtiles", "nchunks", "tiles_per_chunk", "slices", "blocks", "sub_tiles", "vectors_per_block",
            "narrow_tiles", "sub_tile_vectors")
    return dict(zip(keys, (int(v) for v in out)))


def core_xi_bytes(d: int, m: int) -> int:
    return int(load_library().core_xi_bytes(d, m))


def alloc_xi(d: int, m: int, device="cuda") -> torch.Tensor:
    """Buffer for the materialised-Xi comparison variant, viewed as [ceil(d/4), m, 4] fp32."""
    nbytes = core_xi_bytes(d, m)
    if nbytes == 0:
        raise CoreError(ERR_INVALID_ARGUMENT, "core_xi_bytes")
    return torch.empty((nbytes // (16 * m), m, 4), dtype=torch.float32, device=device)


def core_compress_batched_store_xi(seed: int, rnd: int, G: torch.Tensor, m: int, xi: torch.Tensor,
                                   d: int | None = None, ws: torch.Tensor | None = None,
                                   want_P: bool = True):
    """core_compress_batched that also writes the normals it generates into `xi`."""
    _require_cuda(G, xi, ws)
    if G.dim() != 2 or G.stride(1) != 1:
        raise ValueError("G must be 2-D with unit stride along the coordinate axis")
    n, ld = G.shape[0], G.stride(0)
    if d is None:
        d = G.shape[1]
    P = torch.empty((n, m), dtype=torch.float32, device=G.device) if want_P else None
    pbar = torch.empty(m, dtype=torch.float32, device=G.device)
    if ws is None:
        ws = alloc_workspace(d, m, n, G.device)
    rc = load_library().core_compress_batched_store_xi(
        seed, rnd, d, m, n, G.data_ptr(), _dtype_code(G), ld, P.data_ptr() if P is not None else None,
        pbar.data_ptr(), xi.data_ptr(), xi.numel() * 4, ws.data_ptr(), ws.numel(), _stream())
    _check(rc, "core_compress_batched_store_xi")
    return P, pbar


def core_reconstruct_from_xi(d: int, pbar: torch.Tensor, scale: float, xi: torch.Tensor,
                             gtilde: torch.Tensor | None = None) -> torch.Tensor:
    _require_cuda(pbar, xi, gtilde)
    m = pbar.numel()
    if gtilde is None:
        gtilde = torch.empty(d, dtype=torch.float32, device=pbar.device)
    rc = load_library().core_reconstruct_from_xi(d, m, pbar.data_ptr(), scale, xi.data_ptr(),
                                                 xi.numel() * 4, gtilde.data_ptr(), _stream())
    _check(rc, "core_reconstruct_from_xi")
    return gtilde


def core_round_materialized(seed: int, rnd: int, G: torch.Tensor, m: int, xi: torch.Tensor,
                            d: int | None = None, pbar: torch.Tensor | None = None,
                            gtilde: torch.Tensor | None = None, ws: torch.Tensor | None = None):
    """core_round that stores Xi while projecting and reads it back to reconstruct."""
    _require_cuda(G, xi, pbar, gtilde, ws)
    if G.dim() != 2 or G.stride(1) != 1:
        raise ValueError("G must be 2-D with unit stride along the coordinate axis")
    n, ld = G.shape[0], G.stride(0)
    if d is None:
        d = G.shape[1]
    if pbar is None:
        pbar = torch.empty(m, dtype=torch.float32, device=G.device)
    if gtilde is None:
        gtilde = torch.empty(d, dtype=torch.float32, device=G.device)
    if ws is None:
        ws = alloc_workspace(d, m, n, G.device)
    rc = load_library().core_round_materialized(
        seed, rnd, d, m, n, G.data_ptr(), _dtype_code(G), ld, pbar.data_ptr(), gtilde.data_ptr(),
        xi.data_ptr(), xi.numel() * 4, ws.data_ptr(), ws.numel(), _stream())
    _check(rc, "core_round_materialized")
    return pbar, gtilde


def core_debug_philox(seed: int, rnd: int, j: int, q0: int, nblocks: int, device="cuda") -> torch.Tensor:
    out = torch.empty((nblocks, 4), dtype=torch.int32, device=device)
    rc = load_library().core_debug_philox(seed, rnd, j, q0, nblocks, out.data_ptr(), _stream())
    _check(rc, "core_debug_philox")
    return out


PHILOX_LAYOUTS = {"scalar_keys": 0, "projection": 1, "reconstruction": 2, "debug_xi": 3, "projection_sub_tiles": 4}


def core_debug_philox_layout(layout: str | int, seed: int, rnd: int, j0: int, nj: int, q0: int, nq: int,
                             device="cuda") -> torch.Tensor:
    """Words [nj, nq, 4] of blocks q0.. of vectors j0.., generated the way one kernel family does."""
    code = PHILOX_LAYOUTS[layout] if isinstance(layout, str) else int(layout)
    out = torch.empty((nj, nq, 4), dtype=torch.int32, device=device)
    rc = load_library().core_debug_philox_layout(code, seed, rnd, j0, nj, q0, nq, out.data_ptr(), _stream())
    _check(rc, "core_debug_philox_layout")
    return out


PROJECTION_VARIANTS = {"default": 0, "valu": 1, "mfma": 2, "q": 3, "small": 4}


def core_debug_set_projection(variant: str | int) -> None:
    """Force the projection kernel for later calls ("default" hands the choice back)."""
    code = PROJECTION_VARIANTS[variant] if isinstance(variant, str) else int(variant)
    _check(load_library().core_debug_set_projection(code), "core_debug_set_projection")


def core_build_id() -> str:
    return load_library().core_build_id().decode()


def core_debug_xi(seed: int, rnd: int, j: int, i0: int, count: int, device="cuda") -> torch.Tensor:
    out = torch.empty(count, dtype=torch.float32, device=device)
    rc = load_library().core_debug_xi(seed, rnd, j, i0, count, out.data_ptr(), _stream())
    _check(rc, "core_debug_xi")
    return out
