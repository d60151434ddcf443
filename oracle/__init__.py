"""ctypes front end of the CPU oracle (``core_oracle.c``).

TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's
``cpu_baseline`` leg may import this package; the product package must not.

Every function here only marshals numpy arrays into the C routines; the
arithmetic of the method lives in ``core_oracle.c`` and is documented there
against Algorithm 1, Eq. (reconstruction), Eq. (tildefdef) and Algorithm 2 of
the paper.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "core_oracle.c")
_LIB = os.path.join(_HERE, "libcore_oracle.so")

F64, F32, BF16 = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, no fast-math, no contraction)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        subprocess.run(
            ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-Wall", "-Wextra",
             "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"],
            check=True,
        )
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        u32p = ctypes.POINTER(ctypes.c_uint32)
        f64p = ctypes.POINTER(ctypes.c_double)
        u64, u32, vp, i32, f64 = (ctypes.c_uint64, ctypes.c_uint32, ctypes.c_void_p,
                                  ctypes.c_int, ctypes.c_double)
        L.core_oracle_philox_round.argtypes = [u32p, u32p]
        L.core_oracle_philox_round.restype = None
        L.core_oracle_philox4x32_10.argtypes = [u32p, u32p, u32p]
        L.core_oracle_philox4x32_10.restype = None
        L.core_oracle_box_muller.argtypes = [u32, u32, f64p, f64p]
        L.core_oracle_box_muller.restype = None
        L.core_oracle_words.argtypes = [u64, u64, u32, u64, u32p]
        L.core_oracle_words.restype = None
        L.core_oracle_xi_block.argtypes = [u64, u64, u32, u64, f64p]
        L.core_oracle_xi_block.restype = None
        L.core_oracle_xi.argtypes = [u64, u64, u32, u64]
        L.core_oracle_xi.restype = f64
        L.core_oracle_xi_fill.argtypes = [u64, u64, u32, u64, u64, f64p]
        L.core_oracle_xi_fill.restype = None
        L.core_oracle_compress.argtypes = [u64, u64, u64, u32, vp, i32, u64, u32p, u64, f64p]
        L.core_oracle_compress.restype = i32
        L.core_oracle_client_mean.argtypes = [f64p, u32, u64, f64p]
        L.core_oracle_client_mean.restype = i32
        L.core_oracle_reconstruct.argtypes = [u64, u64, u32, f64p, f64, u64, u64, f64p]
        L.core_oracle_reconstruct.restype = i32
        L.core_oracle_round.argtypes = [u64, u64, u64, u32, u32, vp, i32, u64, u32p,
                                        f64p, f64p, f64p]
        L.core_oracle_round.restype = i32
        _lib = L
    return _lib


def _u32p(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint32))


def _f64p(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def philox_round(ctr, key) -> np.ndarray:
    """One Philox4x32 round applied to a 4-word counter with a 2-word round key."""
    c = np.array(ctr, dtype=np.uint32)
    k = np.array(key, dtype=np.uint32)
    lib().core_oracle_philox_round(_u32p(c), _u32p(k))
    return c


def philox4x32_10(ctr, key) -> np.ndarray:
    c = np.array(ctr, dtype=np.uint32)
    k = np.array(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().core_oracle_philox4x32_10(_u32p(c), _u32p(k), _u32p(out))
    return out


def box_muller(xa: int, xb: int):
    a, b = ctypes.c_double(), ctypes.c_double()
    lib().core_oracle_box_muller(xa, xb, ctypes.byref(a), ctypes.byref(b))
    return a.value, b.value


def words(seed: int, rnd: int, j: int, q: int) -> np.ndarray:
    out = np.zeros(4, dtype=np.uint32)
    lib().core_oracle_words(seed, rnd, j, q, _u32p(out))
    return out


def words_range(seed: int, rnd: int, j: int, q0: int, nblocks: int) -> np.ndarray:
    out = np.zeros((nblocks, 4), dtype=np.uint32)
    L = lib()
    for b in range(nblocks):
        L.core_oracle_words(seed, rnd, j, q0 + b, _u32p(out[b]))
    return out


def xi_block(seed: int, rnd: int, j: int, q: int) -> np.ndarray:
    out = np.zeros(4, dtype=np.float64)
    lib().core_oracle_xi_block(seed, rnd, j, q, _f64p(out))
    return out


def xi(seed: int, rnd: int, j: int, i: int) -> float:
    return lib().core_oracle_xi(seed, rnd, j, i)


def xi_range(seed: int, rnd: int, j: int, i0: int, count: int) -> np.ndarray:
    """xi_j[i0 : i0+count] as fp64."""
    out = np.zeros(count, dtype=np.float64)
    lib().core_oracle_xi_fill(seed, rnd, j, i0, count, _f64p(out))
    return out


def _as_stored(G):
    """Return (contiguous 2-D array, dtype code).  uint16 arrays are bf16 bit patterns."""
    G = np.asarray(G)
    if G.ndim == 1:
        G = G[None, :]
    if G.dtype == np.float64:
        code = F64
    elif G.dtype == np.float32:
        code = F32
    elif G.dtype == np.uint16:
        code = BF16
    else:
        raise TypeError(f"unsupported dtype {G.dtype}")
    return np.ascontiguousarray(G), code


def compress(seed: int, rnd: int, G, m: int | None = None, jidx=None) -> np.ndarray:
    """P[c, t] = <G[c], xi_{jidx[t]}> (fp64).  jidx defaults to 0..m-1."""
    G, code = _as_stored(G)
    n, d = G.shape
    if jidx is None:
        jidx = np.arange(m, dtype=np.uint32)
    jidx = np.ascontiguousarray(jidx, dtype=np.uint32)
    P = np.zeros((n, len(jidx)), dtype=np.float64)
    rc = lib().core_oracle_compress(seed, rnd, d, n, G.ctypes.data, code, d,
                                    _u32p(jidx), len(jidx), _f64p(P))
    if rc:
        raise ValueError("core_oracle_compress: bad argument")
    return P


def client_mean(P) -> np.ndarray:
    P = np.ascontiguousarray(P, dtype=np.float64)
    n, nj = P.shape
    pbar = np.zeros(nj, dtype=np.float64)
    if lib().core_oracle_client_mean(_f64p(P), n, nj, _f64p(pbar)):
        raise ValueError("core_oracle_client_mean: bad argument")
    return pbar


def reconstruct(seed: int, rnd: int, pbar, scale: float, i0: int, count: int) -> np.ndarray:
    """scale * sum_j pbar[j] xi_j[i0:i0+count] (fp64)."""
    pbar = np.ascontiguousarray(pbar, dtype=np.float64)
    out = np.zeros(count, dtype=np.float64)
    rc = lib().core_oracle_reconstruct(seed, rnd, len(pbar), _f64p(pbar), scale, i0, count,
                                       _f64p(out))
    if rc:
        raise ValueError("core_oracle_reconstruct: bad argument")
    return out


def core_round(seed: int, rnd: int, G, m: int):
    """Returns (P [n,m], pbar [m], gtilde [d]), all fp64."""
    G, code = _as_stored(G)
    n, d = G.shape
    allj = np.arange(m, dtype=np.uint32)
    P = np.zeros((n, m), dtype=np.float64)
    pbar = np.zeros(m, dtype=np.float64)
    gt = np.zeros(d, dtype=np.float64)
    rc = lib().core_oracle_round(seed, rnd, d, m, n, G.ctypes.data, code, d, _u32p(allj),
                                 _f64p(P), _f64p(pbar), _f64p(gt))
    if rc:
        raise ValueError("core_oracle_round: bad argument")
    return P, pbar, gt
