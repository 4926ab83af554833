"""GPU parity of one flow step (inverse convolution + Actnorm + 1 x 1 convolution, Section 4.1) against the
fp64 oracle, element by element on the same seeded inputs; fused kernels (few channels) and separate passes."""
import numpy as np
import pytest

import oracle
from paper_2410_14634_amd import binding as b
from paper_2410_14634_amd import inputs
from tests.util import THREADS, TOL_ACT, TOL_DW, dev, elementwise_ok, host, rel_err

pytestmark = pytest.mark.gpu

FLOW_SHAPES = [  # (B, C, H, W, k)
    # fused: few channels, image in LDS, rows of whole 16-byte pieces
    (4, 3, 8, 8, 3), (16, 3, 32, 32, 3), (32, 3, 64, 64, 5), (3, 1, 28, 28, 3), (5, 2, 33, 20, 3), (2, 4, 64, 64, 3),
    (300, 3, 16, 16, 3), (2, 3, 1, 4, 3), (2, 3, 7, 12, 5),
    # few images of few channels: the split solve applies the map (forward); eight waves per image (backward, rows of
    # whole 16-pixel groups)
    (5, 1, 16, 48, 3), (7, 2, 24, 16, 3), (3, 4, 32, 32, 3), (9, 3, 20, 64, 3), (2, 3, 64, 32, 3), (200, 3, 16, 16, 3),
    (2, 3, 40, 36, 5),
    # separate passes: rows not a multiple of 4, tall or many-channel images, other kernel sizes
    (3, 3, 13, 7, 3), (2, 3, 130, 40, 3), (64, 12, 16, 16, 3), (2, 12, 128, 128, 3), (2, 8, 50, 17, 3),
    (1, 5, 9, 11, 4), (1, 20, 6, 7, 2), (2, 3, 32, 32, 7), (2, 16, 20, 24, 3), (1, 1, 1, 1, 1),
    # 5-16 channels on images of one band: the one-band kernel applies the map (forward)
    (64, 12, 16, 16, 3), (5, 8, 16, 20, 3), (3, 16, 7, 7, 3), (4, 6, 9, 33, 3), (2, 13, 16, 16, 3), (1, 12, 1, 1, 3),
    # more than 16 channels: set-up by sixteen waves, channel map in blocks of output channels, sums on the matrix cores
    (2, 48, 8, 8, 3), (3, 24, 16, 12, 3), (2, 33, 9, 5, 3), (1, 70, 4, 4, 3), (2, 17, 5, 8, 3),
    # 8-16 channels: the pipelined band kernel applies the map in its storers / folds it into its input weights
    (3, 12, 33, 20, 3), (1, 16, 64, 40, 3), (2, 8, 128, 8, 3), (26, 12, 100, 36, 3), (3, 12, 7, 5, 3), (2, 12, 20, 6, 3),
]


def flow_case(shape, seed):
    B, C, H, W, k = shape
    cs = inputs.make_case(B, C, H, W, k, seed=seed, tap_std=0.05 if k <= 5 else 0.15 / k)
    p = inputs.make_flow_params(C, seed)
    return cs["y"], cs["w"][0], p["s"], p["b"], p["Q"], cs["g"]


@pytest.mark.parametrize("shape", FLOW_SHAPES)
@pytest.mark.parametrize("form", [b.FLOW_FUSED, b.FLOW_AUTO])
def test_flowstep_parity(shape, form):
    import torch
    B, C, H, W, k = shape
    print(f"flow step {shape}", flush=True)
    y, w, s, bb, Q, gz = flow_case(shape, sum(shape))
    yd, wd, sd, bd, Qd, gd = (dev(t) for t in (y, w, s, bb, Q, gz))
    ws = b.new_workspace(b.flowstep_workspace_bytes(B, C, H, W, k))
    z, ld = b.invconv_flowstep_fwd(yd, wd, sd, bd, Qd, workspace=ws, form=form)
    lw = -0.25 * B
    grads = b.invconv_flowstep_bwd(z, wd, sd, bd, Qd, gd, logdet_weight=lw, workspace=ws, form=form)
    torch.cuda.synchronize()
    assert b.workspace_error(ws) == 0
    zh = host(z)
    xr, zr = oracle.flowstep_fwd(y, w, s, bb, Q, THREADS)
    e = rel_err(zh, zr)
    assert e <= TOL_ACT and elementwise_ok(zh, zr, TOL_ACT), f"z rel err {e}"
    ldr = oracle.flowstep_logdet(w, s, Q, H, W)
    assert abs(float(ld[0]) - ldr) <= 1e-5 * max(1.0, abs(ldr)), (float(ld[0]), ldr)
    # The backward pass starts from the GPU's own z, as in a training step; the oracle gets the x that this z
    # stands for (the neighbours undone in float64), so that both differentiate at the same point.
    s64, b64, Q64 = (np.asarray(t, dtype=np.float64) for t in (s, bb, Q))
    a64 = np.einsum("oi,nihw->nohw", np.linalg.inv(Q64), zh.astype(np.float64))
    x64 = (a64 - b64.reshape(1, C, 1, 1)) / s64.reshape(1, C, 1, 1)
    ref = oracle.flowstep_bwd(x64, w, s, bb, Q, gz, THREADS)
    gw, gs, gQ = oracle.flowstep_logdet_grads(w, s, Q, H, W)
    ref["dw"] = ref["dw"] + lw * gw
    ref["ds"] = ref["ds"] + lw * gs
    ref["dQ"] = ref["dQ"] + lw * gQ
    ev = rel_err(host(grads["dy"]), ref["dy"])
    assert ev <= TOL_ACT and elementwise_ok(host(grads["dy"]), ref["dy"], TOL_ACT), f"dL/dy rel err {ev}"
    for name in ("dw", "ds", "db", "dQ"):
        e = rel_err(host(grads[name]), ref[name])
        assert e <= TOL_DW, f"{name} rel err {e}"
    iu = np.triu_indices(C, 1)
    assert np.all(host(grads["dw"])[:, :, k - 1, k - 1][iu] == 0.0)


@pytest.mark.parametrize("shape", [(16, 3, 32, 32, 3), (32, 3, 64, 64, 5), (5, 2, 33, 20, 3), (700, 4, 16, 16, 3)])
def test_fused_and_separate_forms_agree(shape):
    """Where the fused kernels exist, the separate-pass form of the same step gives the same results to rounding."""
    import torch
    B, C, H, W, k = shape
    y, w, s, bb, Q, gz = flow_case(shape, sum(shape) + 1)
    yd, wd, sd, bd, Qd, gd = (dev(t) for t in (y, w, s, bb, Q, gz))
    z0, l0 = b.invconv_flowstep_fwd(yd, wd, sd, bd, Qd, form=b.FLOW_FUSED)
    z1, l1 = b.invconv_flowstep_fwd(yd, wd, sd, bd, Qd, form=b.FLOW_SEPARATE)
    g0 = b.invconv_flowstep_bwd(z0, wd, sd, bd, Qd, gd, logdet_weight=2.0, form=b.FLOW_FUSED)
    g1 = b.invconv_flowstep_bwd(z0, wd, sd, bd, Qd, gd, logdet_weight=2.0, form=b.FLOW_SEPARATE)
    torch.cuda.synchronize()
    assert rel_err(host(z0), host(z1)) <= 1e-5 and float(l0[0]) == float(l1[0])
    assert rel_err(host(g0["dy"]), host(g1["dy"])) <= 1e-5
    for name in ("dw", "ds", "db", "dQ"):
        assert rel_err(host(g0[name]), host(g1[name])) <= 1e-4, name


def test_flowstep_with_identity_neighbours_is_the_inverse_convolution():
    import torch
    wl = inputs.make_workload(1)
    C = wl["C"]
    yd, wd, gd = dev(wl["y"]), dev(wl["w"][0]), dev(wl["g"])
    one, zero, eye = dev(np.ones(C)), dev(np.zeros(C)), dev(np.eye(C))
    z, ld = b.invconv_flowstep_fwd(yd, wd, one, zero, eye)
    x = b.invconv_fwd(yd, wd)
    v, dw = b.invconv_bwd(x, wd, gd)
    grads = b.invconv_flowstep_bwd(z, wd, one, zero, eye, gd)
    torch.cuda.synchronize()
    assert rel_err(host(z), host(x)) <= 1e-6 and float(ld[0]) == 0.0
    assert rel_err(host(grads["dy"]), host(v)) <= 1e-5
    assert rel_err(host(grads["dw"]), host(dw)) <= 1e-4


def test_flowstep_is_bitwise_reproducible_and_rejects_bad_arguments():
    import torch
    shape = (16, 3, 32, 32, 3)
    y, w, s, bb, Q, gz = flow_case(shape, 5)
    yd, wd, sd, bd, Qd, gd = (dev(t) for t in (y, w, s, bb, Q, gz))
    z, _ = b.invconv_flowstep_fwd(yd, wd, sd, bd, Qd)
    first = b.invconv_flowstep_bwd(z, wd, sd, bd, Qd, gd, logdet_weight=1.5)
    for _ in range(3):
        again = b.invconv_flowstep_bwd(z, wd, sd, bd, Qd, gd, logdet_weight=1.5)
        torch.cuda.synchronize()
        for name in first:
            assert torch.equal(first[name], again[name]), name
    with pytest.raises(b.InvconvError) as ei:
        b.invconv_flowstep_fwd(yd, wd, sd, bd, Qd, out=yd)
    assert ei.value.status == b.ERR_ALIAS
    with pytest.raises(b.InvconvError) as ei:
        b.invconv_flowstep_fwd(yd, wd, sd, bd, Qd, workspace=b.new_workspace(256))
    assert ei.value.status == b.ERR_WORKSPACE
