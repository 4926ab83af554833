"""GPU parity of the masked causal convolution y = conv_w(x) (Eq. 1) against the fp64 oracle."""
import numpy as np
import pytest

import oracle
from paper_2410_14634_amd import binding as b
from paper_2410_14634_amd import inputs
from tests.util import THREADS, TOL_ACT, TOL_DW, dev, elementwise_ok, host, rel_err

pytestmark = pytest.mark.gpu

CONV_SHAPES = [  # (B, C, H, W, k)
    (1, 1, 1, 1, 1), (1, 1, 1, 1, 3), (2, 1, 5, 5, 2), (3, 2, 7, 13, 3), (2, 3, 13, 7, 3),
    (1, 4, 1, 40, 3), (1, 4, 40, 1, 3), (2, 3, 2, 2, 5), (1, 5, 9, 11, 4), (2, 16, 10, 10, 3),
    (1, 3, 70, 33, 3), (5, 2, 33, 70, 5), (1, 1, 100, 100, 7), (2, 7, 17, 19, 1),
    (1, 3, 5, 100, 5), (2, 12, 16, 16, 3), (1, 12, 33, 20, 3), (1, 16, 128, 40, 3),
    (2, 12, 40, 36, 5), (1, 16, 9, 12, 5), (1, 8, 20, 24, 4),
    (1, 3, 17, 1200, 3),                     # a row chunk of one row
    (1, 12, 4, 1400, 3),                     # many column tiles, ragged last one
    (1, 20, 6, 7, 2), (2, 18, 9, 5, 3),      # more than 16 channels: two blocks of output channels
    (1, 40, 5, 6, 7),                        # tile and tables exceed LDS: one-thread-per-output kernel
    (2, 8, 20, 70, 5), (1, 10, 9, 9, 7),     # contraction longer than one register chunk
]


# more tiles than the launch has workgroups: every workgroup walks several tiles (LDS reuse, XCD sweep)
MANY_TILE_SHAPES = [(300, 3, 64, 64, 3), (260, 12, 64, 64, 3), (1100, 2, 16, 40, 5)]


def check_conv(x, w):
    import torch
    y = b.invconv_conv_fwd(dev(x), dev(w))
    torch.cuda.synchronize()
    y = host(y)
    yr = oracle.conv(x, w, THREADS)
    e = rel_err(y, yr)
    assert e <= TOL_ACT and elementwise_ok(y, yr, TOL_ACT), f"conv rel err {e}"
    return y


def check_conv_bwd(x, w, g):
    import torch
    dx, dw = b.invconv_conv_bwd(dev(x), dev(w), dev(g))
    torch.cuda.synchronize()
    dx, dw = host(dx), host(dw)
    dxr, dwr = oracle.conv_bwd(x, w, g, THREADS)
    ex, ew = rel_err(dx, dxr), rel_err(dw, dwr)
    assert ex <= TOL_ACT and elementwise_ok(dx, dxr, TOL_ACT), f"conv dL/dx rel err {ex}"
    assert ew <= TOL_DW, f"conv dL/dw rel err {ew}"
    return dx, dw


@pytest.mark.parametrize("cfg", [0, 1, 2, 3])
def test_conv_bwd_workload_parity(cfg):
    wl = inputs.make_workload(cfg)
    print(f"conv bwd workload {cfg}", flush=True)
    check_conv_bwd(wl["y"], wl["w"][0], wl["g"])


def test_conv_bwd_workload4_reduced_batch_parity():
    wl = inputs.make_workload(4, B=4, layers=1)
    check_conv_bwd(wl["y"], wl["w"][0], wl["g"])


@pytest.mark.parametrize("shape", CONV_SHAPES)
def test_conv_bwd_edge_shapes(shape):
    B, C, H, W, k = shape
    print(f"conv bwd edge {shape}", flush=True)
    cs = inputs.make_case(B, C, H, W, k, seed=sum(shape) + 3, tap_std=0.05)
    check_conv_bwd(cs["y"], cs["w"][0], cs["g"])


@pytest.mark.parametrize("shape", MANY_TILE_SHAPES)
def test_conv_fwd_and_bwd_with_more_tiles_than_workgroups(shape):
    B, C, H, W, k = shape
    print(f"conv many tiles {shape}", flush=True)
    cs = inputs.make_case(B, C, H, W, k, seed=sum(shape) + 5, tap_std=0.05)
    check_conv(cs["y"], cs["w"][0])
    check_conv_bwd(cs["y"], cs["w"][0], cs["g"])


def test_conv_masked_garbage_at_twelve_channels():
    cs = inputs.make_case(3, 12, 40, 36, 3, seed=8, tap_std=0.05)
    w = cs["w"][0].copy()
    y0 = check_conv(cs["y"], w)
    dx0, dw0 = check_conv_bwd(cs["y"], w, cs["g"])
    iu = np.triu_indices(12, 1)
    w[:, :, 2, 2][iu] = 1e6
    y1 = check_conv(cs["y"], w)
    dx1, dw1 = check_conv_bwd(cs["y"], w, cs["g"])
    assert np.array_equal(y0, y1) and np.array_equal(dx0, dx1) and np.array_equal(dw0, dw1)
    assert np.all(dw1[:, :, 2, 2][iu] == 0.0)


def test_conv_bwd_masked_entries_get_zero_gradient_and_are_ignored():
    cs = inputs.make_case(2, 4, 9, 9, 3, seed=6, tap_std=0.05)
    w = cs["w"][0].copy()
    dx0, dw0 = check_conv_bwd(cs["y"], w, cs["g"])
    for o in range(4):
        for i in range(o + 1, 4):
            w[o, i, 2, 2] = 1e6
            assert dw0[o, i, 2, 2] == 0.0
    dx1, dw1 = check_conv_bwd(cs["y"], w, cs["g"])
    assert np.array_equal(dx0, dx1) and np.array_equal(dw0, dw1)


def test_conv_bwd_adjoint_identity_on_gpu():
    import torch
    wl = inputs.make_workload(1)
    xd, wd, gd = dev(wl["y"]), dev(wl["w"][0]), dev(wl["g"])
    y = b.invconv_conv_fwd(xd, wd)
    dx, _ = b.invconv_conv_bwd(xd, wd, gd)
    torch.cuda.synchronize()
    lhs = float((y.double() * gd.double()).sum())
    rhs = float((xd.double() * dx.double()).sum())
    assert abs(lhs - rhs) <= 1e-5 * max(abs(lhs), 1.0)


@pytest.mark.parametrize("cfg", [0, 1, 2, 3])
def test_conv_workload_parity(cfg):
    wl = inputs.make_workload(cfg)
    print(f"conv workload {cfg}", flush=True)
    check_conv(wl["y"], wl["w"][0])


def test_conv_workload4_reduced_batch_parity():
    wl = inputs.make_workload(4, B=4, layers=1)
    check_conv(wl["y"], wl["w"][0])


@pytest.mark.parametrize("shape", CONV_SHAPES)
def test_conv_edge_shapes(shape):
    B, C, H, W, k = shape
    print(f"conv edge {shape}", flush=True)
    cs = inputs.make_case(B, C, H, W, k, seed=sum(shape), tap_std=0.05)
    check_conv(cs["y"], cs["w"][0])


def test_conv_ignores_masked_entries():
    cs = inputs.make_case(2, 4, 9, 9, 3, seed=5, tap_std=0.05)
    w = cs["w"][0].copy()
    y0 = check_conv(cs["y"], w)
    for o in range(4):
        for i in range(o + 1, 4):
            w[o, i, 2, 2] = 1e6
    y1 = check_conv(cs["y"], w)
    assert np.array_equal(y0, y1)


@pytest.mark.parametrize("cfg", [1, 2])
def test_conv_undoes_invconv_fwd_on_device(cfg):
    import torch
    wl = inputs.make_workload(cfg)
    yd, wd = dev(wl["y"]), dev(wl["w"][0])
    x = b.invconv_fwd(yd, wd)
    y2 = b.invconv_conv_fwd(x, wd)
    torch.cuda.synchronize()
    assert rel_err(host(y2), wl["y"]) <= TOL_ACT


def test_conv_rejects_aliasing():
    cs = inputs.make_case(1, 3, 8, 8, 3, seed=1, tap_std=0.05)
    xd, wd = dev(cs["y"]), dev(cs["w"][0])
    with pytest.raises(b.InvconvError):
        b.invconv_conv_fwd(xd, wd, out=xd)
