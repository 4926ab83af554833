"""Seeded synthetic inputs for the inverse-convolution workloads.

This module only draws random numbers and shapes them; it contains none of the
method's arithmetic, so both the CPU oracle's tests and the HIP path's tests may
use it.  Everything is generated on the host with NumPy and returned as
contiguous float32 arrays; the same arrays are handed to both sides.

Workloads (shapes and value distributions stand in for the paper's MNIST /
CIFAR-10 / ablation tensors, Section 5 and the supplement's ablation tables;
the datasets themselves are not needed):

  id  B   C   H=W  k   y                          centre diagonal   other taps
  0   4   3   8    3   U(0,1)                     1.0               N(0, 0.05)
  1   16  3   32   3   (n + u)/256, n in 0..255   1.0               N(0, 0.05)
  2   64  12  16   3   N(0,1)                     U(0.5,1.5)        N(0, 0.03)
  3   32  3   64   5   (n + u)/256                1.0               N(0, 0.02)
  4   32  12  128  3   N(0,1), 8 stacked layers   U(0.5,1.5)        N(0, 0.03)

"N(0, s)" is read as standard deviation s.  Kernel layout is [C_out][C_in][k][k]
(Algorithm 1's K[c, k_c, ., .]); tap (k-1,k-1) multiplies the current pixel
(Eq. 1, bottom-right entry).  At that tap the channel mixing is lower
triangular; entries above the diagonal are generated as 0 (they are ignored by
the operator anyway).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

# tensor ids used in the seed sequence
_T_W_OFF, _T_W_CTR, _T_W_DIAG, _T_Y, _T_G = 0, 1, 2, 3, 4


@dataclass(frozen=True)
class Workload:
    cfg: int
    B: int
    C: int
    H: int
    W: int
    k: int
    layers: int
    y_kind: str       # "uniform" | "dequant" | "normal"
    diag_kind: str    # "one" | "uniform"
    tap_std: float

    @property
    def n_elems(self) -> int:
        return self.B * self.C * self.H * self.W


WORKLOADS = {
    0: Workload(0, 4, 3, 8, 8, 3, 1, "uniform", "one", 0.05),
    1: Workload(1, 16, 3, 32, 32, 3, 1, "dequant", "one", 0.05),
    2: Workload(2, 64, 12, 16, 16, 3, 1, "normal", "uniform", 0.03),
    3: Workload(3, 32, 3, 64, 64, 5, 1, "dequant", "one", 0.02),
    4: Workload(4, 32, 12, 128, 128, 3, 8, "normal", "uniform", 0.03),
}


def _rng(cfg: int, layer: int, tensor: int) -> np.random.Generator:
    return np.random.default_rng([0, cfg, layer, tensor])


def make_w(C: int, k: int, tap_std: float, diag_kind: str, *, cfg: int = 99,
           layer: int = 0) -> np.ndarray:
    """Kernel [C][C][k][k] float32: dense off-centre taps, lower-triangular centre tap."""
    w = _rng(cfg, layer, _T_W_OFF).normal(0.0, tap_std, size=(C, C, k, k))
    ctr = _rng(cfg, layer, _T_W_CTR).normal(0.0, tap_std, size=(C, C))
    ctr = np.tril(ctr, -1)
    if diag_kind == "one":
        diag = np.ones(C)
    elif diag_kind == "uniform":
        diag = _rng(cfg, layer, _T_W_DIAG).uniform(0.5, 1.5, size=C)
    else:
        raise ValueError(diag_kind)
    ctr[np.arange(C), np.arange(C)] = diag
    w[:, :, k - 1, k - 1] = ctr
    return np.ascontiguousarray(w, dtype=np.float32)


def make_act(kind: str, shape, *, cfg: int = 99, tensor: int = _T_Y) -> np.ndarray:
    rng = _rng(cfg, 0, tensor)
    if kind == "uniform":
        a = rng.uniform(0.0, 1.0, size=shape)
    elif kind == "dequant":
        n = rng.integers(0, 256, size=shape)
        a = (n + rng.uniform(0.0, 1.0, size=shape)) / 256.0
    elif kind == "normal":
        a = rng.normal(0.0, 1.0, size=shape)
    else:
        raise ValueError(kind)
    return np.ascontiguousarray(a, dtype=np.float32)


def make_workload(cfg: int, *, B: int | None = None, H: int | None = None,
                  W: int | None = None, layers: int | None = None) -> dict:
    """Arrays for workload `cfg`; B/H/W/layers may be overridden to shrink a case.

    Returns dict(B, C, H, W, k, layers, y, g, w) where w is a list with one
    kernel per layer, y the input of the first layer and g the upstream
    gradient dL/dx ~ N(0,1) (for the chain workload the harness replaces g by
    the last layer's output, as the chain loss prescribes).
    """
    wl = WORKLOADS[cfg]
    B = wl.B if B is None else B
    H = wl.H if H is None else H
    W = wl.W if W is None else W
    layers = wl.layers if layers is None else layers
    shape = (B, wl.C, H, W)
    y = make_act(wl.y_kind, shape, cfg=cfg, tensor=_T_Y)
    g = make_act("normal", shape, cfg=cfg, tensor=_T_G)
    w = [make_w(wl.C, wl.k, wl.tap_std, wl.diag_kind, cfg=cfg, layer=l) for l in range(layers)]
    return dict(cfg=cfg, B=B, C=wl.C, H=H, W=W, k=wl.k, layers=layers, y=y, g=g, w=w)


def make_case(B: int, C: int, H: int, W: int, k: int, *, seed: int = 0,
              tap_std: float = 0.05, diag_kind: str = "uniform",
              y_kind: str = "normal") -> dict:
    """Free-form seeded case for edge-shape tests (not one of the named workloads)."""
    cfg = 1000 + seed
    shape = (B, C, H, W)
    return dict(cfg=cfg, B=B, C=C, H=H, W=W, k=k, layers=1,
                y=make_act(y_kind, shape, cfg=cfg, tensor=_T_Y),
                g=make_act("normal", shape, cfg=cfg, tensor=_T_G),
                w=[make_w(C, k, tap_std, diag_kind, cfg=cfg, layer=0)])


_T_S, _T_B, _T_Q = 5, 6, 7


def make_flow_params(C: int, seed: int = 0, layer: int = 0) -> dict:
    """Seeded parameters of the two neighbours of the inverse convolution in a flow step (Section 4.1):
    Actnorm scale s ~ U(0.5, 1.5) and bias b ~ N(0, 0.5) per channel, and a 1 x 1 convolution Q that is a random
    rotation (the usual initialisation of that layer) plus N(0, 0.05) noise, so that it stays well conditioned."""
    cfg = 2000 + seed
    s = np.random.default_rng([0, cfg, layer, _T_S]).uniform(0.5, 1.5, size=C)
    b = np.random.default_rng([0, cfg, layer, _T_B]).normal(0.0, 0.5, size=C)
    rng = np.random.default_rng([0, cfg, layer, _T_Q])
    rot, _ = np.linalg.qr(rng.normal(size=(C, C)))
    Q = rot + rng.normal(0.0, 0.05, size=(C, C))
    return dict(s=s.astype(np.float32), b=b.astype(np.float32), Q=np.ascontiguousarray(Q, dtype=np.float32))
