"""TEST INFRASTRUCTURE -- NOT PART OF THE PRODUCT PATH.

ctypes front end of ``ln_pegn_oracle.c``: the slow fp64 CPU definition of the
fused LayerNorm-backward + per-example-gradient-norm path (Appendix B, LayerNorm
algorithm; Section 2.1, Eq. 3-5).  Only tests, the smoke check and the
benchmark's ``cpu_baseline`` leg may import this package.  It imports nothing
from the HIP package and the HIP package imports nothing from here.

Every function takes and returns float64 numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ln_pegn_oracle.c")
_LIB = os.path.join(_HERE, "liblnpegn_oracle.so")
_lock = threading.Lock()
_lib = None

_dp = ctypes.POINTER(ctypes.c_double)


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (fp64, -O2, OpenMP over examples)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off",
               "-o", tmp, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


def _bind(lib):
    """Declare the argument types of every oracle entry point on a loaded library."""
    L, D_, I = ctypes.c_long, ctypes.c_double, ctypes.c_int
    lib.lnpegn_oracle_ln_stats.argtypes = [_dp, L, L, D_, _dp, _dp]
    lib.lnpegn_oracle_ln_fwd.argtypes = [_dp, _dp, _dp, L, L, D_, _dp]
    lib.lnpegn_oracle_ln_bwd_example.argtypes = [_dp, _dp, _dp, L, L, D_, _dp, _dp, _dp]
    lib.lnpegn_oracle_ln_bwd_pegn.argtypes = [_dp, _dp, _dp, L, L, L, D_] + [_dp] * 8 + [I]
    lib.lnpegn_oracle_gns_from_norms.argtypes = [D_, D_, D_, D_, _dp]
    lib.lnpegn_oracle_gns_estimate.argtypes = [_dp, _dp, L, L, D_, _dp]
    lib.lnpegn_oracle_max_threads.restype = I
    lib.lnpegn_oracle_rms_fwd.argtypes = [_dp, _dp, L, L, D_, _dp, _dp]
    lib.lnpegn_oracle_rms_bwd_example.argtypes = [_dp, _dp, _dp, L, L, D_, _dp, _dp]
    lib.lnpegn_oracle_rms_bwd_pegn.argtypes = [_dp, _dp, _dp, L, L, L, D_] + [_dp] * 5 + [I]
    for name in ("ln_stats", "ln_fwd", "ln_bwd_example", "ln_bwd_pegn", "gns_from_norms", "gns_estimate",
                 "rms_fwd", "rms_bwd_example", "rms_bwd_pegn"):
        getattr(lib, "lnpegn_oracle_" + name).restype = I
    return lib


def _load():
    global _lib
    with _lock:
        if _lib is None:
            build()
            _lib = _bind(ctypes.CDLL(_LIB))
    return _lib


def _c(a, shape=None):
    a = np.ascontiguousarray(a, dtype=np.float64)
    if shape is not None and a.shape != tuple(shape):
        raise ValueError(f"expected shape {tuple(shape)}, got {a.shape}")
    return a


def _p(a):
    return None if a is None else a.ctypes.data_as(_dp)


def max_threads() -> int:
    return int(_load().lnpegn_oracle_max_threads())


def ln_stats(x, eps):
    """mean[N], rstd[N] of x[..., D] (biased variance, eps inside the root)."""
    x = _c(x)
    D = x.shape[-1]
    N = x.size // D
    mean = np.empty(N)
    rstd = np.empty(N)
    rc = _load().lnpegn_oracle_ln_stats(_p(x), N, D, float(eps), _p(mean), _p(rstd))
    if rc:
        raise ValueError(f"oracle ln_stats rc={rc}")
    return mean.reshape(x.shape[:-1]), rstd.reshape(x.shape[:-1])


def ln_fwd(x, gamma, beta, eps):
    """y = gamma * xhat + beta over the last dimension."""
    x = _c(x)
    D = x.shape[-1]
    gamma, beta = _c(gamma, (D,)), _c(beta, (D,))
    y = np.empty_like(x)
    rc = _load().lnpegn_oracle_ln_fwd(_p(x), _p(gamma), _p(beta), x.size // D, D, float(eps), _p(y))
    if rc:
        raise ValueError(f"oracle ln_fwd rc={rc}")
    return y


def ln_bwd_example(x, dy, gamma, eps, want_dx=True):
    """Backward of ONE example x[T,D], dy[T,D] -> (dx[T,D] or None, g_gamma[D], g_beta[D])."""
    x = _c(x)
    if x.ndim != 2:
        raise ValueError("x must be [T,D]")
    T, D = x.shape
    dy, gamma = _c(dy, (T, D)), _c(gamma, (D,))
    dx = np.empty_like(x) if want_dx else None
    gg, gb = np.empty(D), np.empty(D)
    rc = _load().lnpegn_oracle_ln_bwd_example(_p(x), _p(dy), _p(gamma), T, D, float(eps), _p(dx),
                                              _p(gg), _p(gb))
    if rc:
        raise ValueError(f"oracle ln_bwd_example rc={rc}")
    return dx, gg, gb


def ln_bwd_pegn(x, dy, gamma, eps, want_dx=True, want_pe=True, nthreads=0):
    """Brute force over x[B,T,D], dy[B,T,D]: one separate backward per example.

    Returns a dict: dx [B,T,D] (or None), pe_gamma/pe_beta [B,D] (or None),
    dgamma/dbeta [D], s_gamma/s_beta [B] (raw, no B^2), big_sq [2].
    """
    x = _c(x)
    if x.ndim != 3:
        raise ValueError("x must be [B,T,D]")
    B, T, D = x.shape
    dy, gamma = _c(dy, (B, T, D)), _c(gamma, (D,))
    out = dict(
        dx=np.empty_like(x) if want_dx else None,
        pe_gamma=np.empty((B, D)) if want_pe else None,
        pe_beta=np.empty((B, D)) if want_pe else None,
        dgamma=np.empty(D), dbeta=np.empty(D),
        s_gamma=np.empty(B), s_beta=np.empty(B), big_sq=np.empty(2),
    )
    rc = _load().lnpegn_oracle_ln_bwd_pegn(
        _p(x), _p(dy), _p(gamma), B, T, D, float(eps), _p(out["dx"]), _p(out["pe_gamma"]),
        _p(out["pe_beta"]), _p(out["dgamma"]), _p(out["dbeta"]), _p(out["s_gamma"]),
        _p(out["s_beta"]), _p(out["big_sq"]), int(nthreads))
    if rc:
        raise ValueError(f"oracle ln_bwd_pegn rc={rc}")
    return out


def rms_fwd(x, gamma, eps):
    """RMSNorm forward -> (y, rstd): y = gamma * x * rstd, rstd = 1/sqrt(mean_d x^2 + eps)."""
    x = _c(x)
    D = x.shape[-1]
    gamma = _c(gamma, (D,))
    y = np.empty_like(x)
    rstd = np.empty(x.size // D)
    rc = _load().lnpegn_oracle_rms_fwd(_p(x), _p(gamma), x.size // D, D, float(eps), _p(y), _p(rstd))
    if rc:
        raise ValueError(f"oracle rms_fwd rc={rc}")
    return y, rstd.reshape(x.shape[:-1])


def rms_bwd_example(x, dy, gamma, eps, want_dx=True):
    """RMSNorm backward of ONE example x[T,D] -> (dx or None, g_gamma[D])."""
    x = _c(x)
    if x.ndim != 2:
        raise ValueError("x must be [T,D]")
    T, D = x.shape
    dy, gamma = _c(dy, (T, D)), _c(gamma, (D,))
    dx = np.empty_like(x) if want_dx else None
    gg = np.empty(D)
    rc = _load().lnpegn_oracle_rms_bwd_example(_p(x), _p(dy), _p(gamma), T, D, float(eps), _p(dx), _p(gg))
    if rc:
        raise ValueError(f"oracle rms_bwd_example rc={rc}")
    return dx, gg


def rms_bwd_pegn(x, dy, gamma, eps, want_dx=True, want_pe=True, nthreads=0):
    """RMSNorm brute force over [B,T,D] -> dict(dx, pe_gamma, dgamma, s_gamma, big_sq[1])."""
    x = _c(x)
    if x.ndim != 3:
        raise ValueError("x must be [B,T,D]")
    B, T, D = x.shape
    dy, gamma = _c(dy, (B, T, D)), _c(gamma, (D,))
    out = dict(dx=np.empty_like(x) if want_dx else None, pe_gamma=np.empty((B, D)) if want_pe else None,
               dgamma=np.empty(D), s_gamma=np.empty(B), big_sq=np.empty(1))
    rc = _load().lnpegn_oracle_rms_bwd_pegn(_p(x), _p(dy), _p(gamma), B, T, D, float(eps), _p(out["dx"]),
                                            _p(out["pe_gamma"]), _p(out["dgamma"]), _p(out["s_gamma"]),
                                            _p(out["big_sq"]), int(nthreads))
    if rc:
        raise ValueError(f"oracle rms_bwd_pegn rc={rc}")
    return out


def gns_from_norms(g_big_sq, g_small_sq, b_big, b_small):
    """Eq. 4, Eq. 5, Eq. 3 -> (G2, S, B_simple)."""
    out = np.empty(3)
    rc = _load().lnpegn_oracle_gns_from_norms(float(g_big_sq), float(g_small_sq), float(b_big),
                                              float(b_small), _p(out))
    if rc:
        raise ValueError(f"oracle gns_from_norms rc={rc}")
    return tuple(out.tolist())


def gns_estimate(pe_sq, big_sq, pe_scale):
    """pe_sq [n_groups,B] raw, big_sq [n_groups] -> dict(g_small_sq, g_big_sq, G2, S, B_simple)."""
    pe_sq = _c(pe_sq)
    if pe_sq.ndim == 1:
        pe_sq = pe_sq[None, :]
    n_groups, B = pe_sq.shape
    big_sq = _c(np.atleast_1d(big_sq), (n_groups,))
    out = np.empty(5)
    rc = _load().lnpegn_oracle_gns_estimate(_p(pe_sq), _p(big_sq), n_groups, B, float(pe_scale),
                                            _p(out))
    if rc:
        raise ValueError(f"oracle gns_estimate rc={rc}")
    keys = ("g_small_sq", "g_big_sq", "G2", "S", "B_simple")
    return dict(zip(keys, out.tolist()))
