"""CPU oracle (test infrastructure only) for the inverse convolution and its backward.

Thin ctypes wrapper around ``invconv_oracle.c``.  Inputs are promoted to
float64; every result is float64.  Only tests, the smoke check and the bench's
``cpu_baseline`` leg may import this package; the GPU library never does.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRCS = [os.path.join(_HERE, "invconv_oracle.c"), os.path.join(_HERE, "flowstep_oracle.c")]
_LIB = os.path.join(_HERE, "libinvconv_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, OpenMP over the batch)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < max(os.path.getmtime(f) for f in _SRCS):
        import shutil
        if shutil.which("gcc") is None:
            raise RuntimeError("the CPU oracle is plain C and needs gcc on PATH to build " + _LIB)
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp",
                               "-ffp-contract=off", "-o", _LIB, *_SRCS, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        dp = ctypes.POINTER(ctypes.c_double)
        ci = ctypes.c_int
        lib.oracle_conv.argtypes = [dp, dp, dp, ci, ci, ci, ci, ci, ci]
        lib.oracle_invconv_fwd.argtypes = [dp, dp, dp, ci, ci, ci, ci, ci, ci]
        lib.oracle_invconv_bwd_dy.argtypes = [dp, dp, dp, ci, ci, ci, ci, ci, ci]
        lib.oracle_invconv_bwd_dw.argtypes = [dp, dp, dp, ci, ci, ci, ci, ci, ci]
        lib.oracle_conv_bwd_dx.argtypes = [dp, dp, dp, ci, ci, ci, ci, ci, ci]
        lib.oracle_conv_bwd_dw.argtypes = [dp, dp, dp, ci, ci, ci, ci, ci, ci]
        lib.oracle_invconv_logdet.argtypes = [dp, ci, ci, ci, ci]
        lib.oracle_invconv_logdet.restype = ctypes.c_double
        lib.oracle_max_threads.restype = ci
        lib.oracle_actnorm_fwd.argtypes = [dp, dp, dp, dp, ci, ci, ci, ci]
        lib.oracle_actnorm_bwd.argtypes = [dp, dp, dp, dp, dp, dp, ci, ci, ci, ci]
        lib.oracle_conv1x1_fwd.argtypes = [dp, dp, dp, ci, ci, ci, ci]
        lib.oracle_conv1x1_bwd.argtypes = [dp, dp, dp, dp, dp, ci, ci, ci, ci]
        for f in (lib.oracle_actnorm_fwd, lib.oracle_actnorm_bwd, lib.oracle_conv1x1_fwd, lib.oracle_conv1x1_bwd):
            f.restype = None
        lib.oracle_actnorm_logdet.argtypes = [dp, ci, ci, ci]
        lib.oracle_actnorm_logdet.restype = ctypes.c_double
        lib.oracle_conv1x1_logdet.argtypes = [dp, ci, ci, ci]
        lib.oracle_conv1x1_logdet.restype = ctypes.c_double
        for f in (lib.oracle_conv, lib.oracle_invconv_fwd, lib.oracle_invconv_bwd_dy,
                  lib.oracle_invconv_bwd_dw, lib.oracle_conv_bwd_dx, lib.oracle_conv_bwd_dw):
            f.restype = None
        _lib = lib
    return _lib


def _d(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _dims(act: np.ndarray, w: np.ndarray):
    if act.ndim != 4 or w.ndim != 4:
        raise ValueError("activations must be [B,C,H,W] and kernels [C,C,k,k]")
    B, C, H, W = act.shape
    if w.shape[0] != C or w.shape[1] != C or w.shape[2] != w.shape[3]:
        raise ValueError(f"kernel shape {w.shape} does not match C={C}")
    return B, C, H, W, w.shape[2]


def max_threads() -> int:
    return int(_load().oracle_max_threads())


def conv(x, w, threads: int = 1) -> np.ndarray:
    """y = conv_w(x): masked causal convolution, Eq. 1."""
    x, w = _d(x), _d(w)
    B, C, H, W, k = _dims(x, w)
    y = np.empty_like(x)
    _load().oracle_conv(_p(x), _p(w), _p(y), B, C, H, W, k, threads)
    return y


def conv_bwd_dx(g, w, threads: int = 1) -> np.ndarray:
    """dL/dx = M^T dL/dy of y = conv_w(x)."""
    g, w = _d(g), _d(w)
    B, C, H, W, k = _dims(g, w)
    dx = np.empty_like(g)
    _load().oracle_conv_bwd_dx(_p(g), _p(w), _p(dx), B, C, H, W, k, threads)
    return dx


def conv_bwd_dw(x, g, k: int, threads: int = 1) -> np.ndarray:
    """dL/dw of y = conv_w(x): correlation of dL/dy with shifted x, summed over batch and pixels."""
    x, g = _d(x), _d(g)
    B, C, H, W = x.shape
    dw = np.empty((C, C, k, k), dtype=np.float64)
    _load().oracle_conv_bwd_dw(_p(x), _p(g), _p(dw), B, C, H, W, k, threads)
    return dw


def conv_bwd(x, w, g, threads: int = 1):
    """(dL/dx, dL/dw) of y = conv_w(x) given dL/dy."""
    w = _d(w)
    return conv_bwd_dx(g, w, threads), conv_bwd_dw(x, g, w.shape[2], threads)


def invconv_fwd(y, w, threads: int = 1) -> np.ndarray:
    """x with conv_w(x) = y, by forward substitution in row-major order."""
    y, w = _d(y), _d(w)
    B, C, H, W, k = _dims(y, w)
    x = np.empty_like(y)
    _load().oracle_invconv_fwd(_p(y), _p(w), _p(x), B, C, H, W, k, threads)
    return x


def invconv_bwd_dy(g, w, threads: int = 1) -> np.ndarray:
    """dL/dy = M^{-T} dL/dx (Eq. 2 / Theorem 1)."""
    g, w = _d(g), _d(w)
    B, C, H, W, k = _dims(g, w)
    v = np.empty_like(g)
    _load().oracle_invconv_bwd_dy(_p(g), _p(w), _p(v), B, C, H, W, k, threads)
    return v


def invconv_bwd_dw(x, v, k: int, threads: int = 1) -> np.ndarray:
    """dL/dW = -sum v (x) shifted x (Eq. 4 / Theorem 2), summed over batch and pixels."""
    x, v = _d(x), _d(v)
    B, C, H, W = x.shape
    dw = np.empty((C, C, k, k), dtype=np.float64)
    _load().oracle_invconv_bwd_dw(_p(x), _p(v), _p(dw), B, C, H, W, k, threads)
    return dw


def invconv_bwd(x, w, g, threads: int = 1):
    """(dL/dy, dL/dW) given the forward output x, the kernel and dL/dx."""
    w = _d(w)
    v = invconv_bwd_dy(g, w, threads)
    return v, invconv_bwd_dw(x, v, w.shape[2], threads)


def invconv_logdet(w, H: int, W: int) -> float:
    """log|det dx/dy| of the inverse convolution for one H x W image."""
    w = _d(w)
    C, k = w.shape[0], w.shape[2]
    return float(_load().oracle_invconv_logdet(_p(w), C, H, W, k))


# ---------------------------------------------------------------------------
# The neighbours of the inverse convolution inside a flow step (Section 4.1): Actnorm and the 1 x 1
# convolution, and the step composed of the three layers by the chain rule.
# ---------------------------------------------------------------------------
def actnorm_fwd(x, s, b) -> np.ndarray:
    """a = s[c] * x + b[c] per channel."""
    x, s, b = _d(x), _d(s), _d(b)
    B, C, H, W = x.shape
    a = np.empty_like(x)
    _load().oracle_actnorm_fwd(_p(x), _p(s), _p(b), _p(a), B, C, H, W)
    return a


def actnorm_bwd(x, s, ga):
    """(dL/dx, dL/ds, dL/db) given dL/da."""
    x, s, ga = _d(x), _d(s), _d(ga)
    B, C, H, W = x.shape
    gx, gs, gb = np.empty_like(x), np.empty(C), np.empty(C)
    _load().oracle_actnorm_bwd(_p(x), _p(s), _p(ga), _p(gx), _p(gs), _p(gb), B, C, H, W)
    return gx, gs, gb


def actnorm_logdet(s, H: int, W: int) -> float:
    s = _d(s)
    return float(_load().oracle_actnorm_logdet(_p(s), s.shape[0], H, W))


def conv1x1_fwd(a, Q) -> np.ndarray:
    """z[o] = sum_i Q[o][i] a[i] at every pixel."""
    a, Q = _d(a), _d(Q)
    B, C, H, W = a.shape
    z = np.empty_like(a)
    _load().oracle_conv1x1_fwd(_p(a), _p(Q), _p(z), B, C, H, W)
    return z


def conv1x1_bwd(a, Q, gz):
    """(dL/da, dL/dQ) given dL/dz."""
    a, Q, gz = _d(a), _d(Q), _d(gz)
    B, C, H, W = a.shape
    ga, gQ = np.empty_like(a), np.empty((C, C))
    _load().oracle_conv1x1_bwd(_p(a), _p(Q), _p(gz), _p(ga), _p(gQ), B, C, H, W)
    return ga, gQ


def conv1x1_logdet(Q, H: int, W: int) -> float:
    Q = _d(Q)
    return float(_load().oracle_conv1x1_logdet(_p(Q), Q.shape[0], H, W))


def flowstep_fwd(y, w, s, b, Q, threads: int = 1):
    """(x, z): x = invconv_w(y), z = Q (s * x + b) - the three layers of a flow step in order."""
    x = invconv_fwd(y, w, threads)
    return x, conv1x1_fwd(actnorm_fwd(x, s, b), Q)


def flowstep_bwd(x, w, s, b, Q, gz, threads: int = 1):
    """Chain rule through 1 x 1 convolution, Actnorm and inverse convolution, given x = invconv_w(y) and
    dL/dz.  Returns dict(dy, dw, ds, db, dQ)."""
    a = actnorm_fwd(x, s, b)
    ga, gQ = conv1x1_bwd(a, Q, gz)
    gx, gs, gb = actnorm_bwd(x, s, ga)
    dy, dw = invconv_bwd(x, w, gx, threads)
    return dict(dy=dy, dw=dw, ds=gs, db=gb, dQ=gQ)


def flowstep_logdet(w, s, Q, H: int, W: int) -> float:
    """log|det dz/dy| of the step for one image: the sum of the three layers' log-determinants."""
    return invconv_logdet(w, H, W) + actnorm_logdet(s, H, W) + conv1x1_logdet(Q, H, W)


def flowstep_logdet_grads(w, s, Q, H: int, W: int):
    """Gradients of flowstep_logdet with respect to the parameters (closed forms):
    d/dw[c][c][k-1][k-1] = -H W / w[c][c][k-1][k-1] (zero elsewhere), d/ds[c] = H W / s[c], d/dQ = H W Q^{-T}."""
    w, s, Q = _d(w), _d(s), _d(Q)
    C, k = w.shape[0], w.shape[2]
    gw = np.zeros_like(w)
    for c in range(C):
        gw[c, c, k - 1, k - 1] = -H * W / w[c, c, k - 1, k - 1]
    return gw, H * W / s, H * W * np.linalg.inv(Q).T
