"""GPU parity: the HIP library (through its C ABI) against the fp64 CPU oracle,
element by element on the same seeded inputs."""
import numpy as np
import pytest

import oracle
from paper_2410_14634_amd import binding as b
from paper_2410_14634_amd import inputs
from tests.util import THREADS, TOL_ACT, TOL_DW, dev, elementwise_ok, host, rel_err

pytestmark = pytest.mark.gpu

VARIANTS = [b.VARIANT_AUTO, b.VARIANT_BLOCK, b.VARIANT_DIAG_LAUNCH, b.VARIANT_WAVE, b.VARIANT_BAND,
            b.VARIANT_PERSISTENT, b.VARIANT_WAVE_SPLIT]
WAVE_OK = {0, 1, 3}     # workloads the wave-per-image variant covers (C <= 4, H <= 64)
BAND_OK = {2, 4}        # workloads the 16-row-band variant covers (C = 8, 12, 16; k = 3; H <= 128)


def run_layer(y, w, g, variant=b.VARIANT_AUTO):
    import torch
    yd, wd, gd = dev(y), dev(w), dev(g)
    x = b.invconv_fwd(yd, wd, variant=variant)
    v, dw = b.invconv_bwd(x, wd, gd, variant=variant)
    ld = b.invconv_logdet(wd, y.shape[2], y.shape[3])
    torch.cuda.synchronize()
    return host(x), host(v), host(dw), float(host(ld)[0])


def check_layer(y, w, g, variant=b.VARIANT_AUTO):
    x, v, dw, ld = run_layer(y, w, g, variant)
    xr = oracle.invconv_fwd(y, w, THREADS)
    # the backward is given the GPU's own fp32 x, as in a training step; the oracle gets the same x
    vr, dwr = oracle.invconv_bwd(x, w, g, THREADS)
    ldr = oracle.invconv_logdet(w, y.shape[2], y.shape[3])
    ex, ev, ew = rel_err(x, xr), rel_err(v, vr), rel_err(dw, dwr)
    assert ex <= TOL_ACT and elementwise_ok(x, xr, TOL_ACT), f"x rel err {ex}"
    assert ev <= TOL_ACT and elementwise_ok(v, vr, TOL_ACT), f"dL/dy rel err {ev}"
    assert ew <= TOL_DW, f"dL/dw rel err {ew}"
    assert abs(ld - ldr) <= 1e-5 * max(1.0, abs(ldr)), (ld, ldr)
    return ex, ev, ew


@pytest.mark.parametrize("cfg", [0, 1, 2, 3])
@pytest.mark.parametrize("variant", VARIANTS)
def test_workload_parity(cfg, variant):
    if (variant in (b.VARIANT_WAVE, b.VARIANT_WAVE_SPLIT) and cfg not in WAVE_OK) or \
            (variant == b.VARIANT_BAND and cfg not in BAND_OK):
        pytest.skip("variant does not cover this shape")
    wl = inputs.make_workload(cfg)
    print(f"cfg {cfg} variant {variant}", flush=True)
    print(check_layer(wl["y"], wl["w"][0], wl["g"], variant), flush=True)


def test_workload4_first_layer_parity():
    wl = inputs.make_workload(4, layers=1)
    print(check_layer(wl["y"], wl["w"][0], wl["g"]), flush=True)


EDGE_SHAPES = [  # (B, C, H, W, k)
    (1, 1, 1, 1, 1), (1, 1, 1, 1, 3), (2, 1, 5, 5, 2), (3, 2, 7, 13, 3), (2, 3, 13, 7, 3),
    (1, 4, 1, 40, 3), (1, 4, 40, 1, 3), (2, 3, 2, 2, 5), (1, 5, 9, 11, 4), (2, 16, 10, 10, 3),
    (1, 3, 70, 33, 3), (5, 2, 33, 70, 5), (1, 1, 100, 100, 7), (2, 7, 17, 19, 1),
    (2, 3, 64, 5, 3), (3, 1, 33, 20, 3), (1, 2, 64, 64, 3), (2, 4, 63, 9, 3), (1, 3, 5, 100, 5),
    (2, 12, 16, 16, 3), (1, 12, 33, 20, 3), (2, 8, 50, 17, 3), (1, 16, 128, 40, 3), (1, 12, 7, 100, 3),
    (3, 12, 1, 1, 3), (1, 8, 17, 2, 3), (1, 12, 129, 8, 3),
    (1, 20, 6, 7, 2), (2, 18, 9, 5, 3),      # more than 16 channels (k = 2: the LDS-window solve)
    (2, 48, 32, 32, 3), (1, 32, 40, 24, 3), (1, 24, 20, 12, 5), (1, 48, 60, 9, 3), (1, 40, 8, 8, 3),   # after two squeezes
    (2, 20, 17, 19, 3), (1, 28, 128, 8, 3), (3, 36, 7, 33, 3), (1, 44, 1, 1, 3), (2, 24, 50, 50, 3), (1, 32, 100, 12, 3),
    (1, 40, 64, 16, 3), (1, 32, 96, 20, 3), (2, 44, 33, 12, 3), (1, 48, 64, 24, 3),     # nine to twelve waves per image
    (1, 3, 17, 1200, 3), (1, 12, 4, 1400, 3),    # wide images: dL/dw row tiles beyond the preferred LDS budget
    # few channels, more than 64 rows: bands of 64 rows, one wave each
    (2, 3, 256, 256, 3), (1, 3, 130, 40, 5), (1, 4, 512, 16, 3), (1, 1, 65, 7, 3), (2, 3, 128, 200, 3),
    (1, 2, 191, 3, 3), (1, 3, 320, 70, 5),
    # three or more bands of wide images: one workgroup per band, logs handed over through global memory
    (1, 3, 512, 512, 3), (2, 3, 200, 130, 5), (3, 1, 300, 128, 3), (2, 4, 193, 160, 3), (5, 2, 257, 129, 3),
    (600, 3, 8, 8, 3), (520, 1, 64, 4, 3),     # large batches: the forward launch caps its waves per CU
    # large batches of small images: the image goes through LDS (forward and fused backward)
    (1400, 3, 16, 16, 3), (400, 3, 64, 24, 3), (2400, 1, 28, 28, 3), (700, 2, 50, 10, 3), (1500, 3, 15, 15, 3),
    (1200, 4, 16, 16, 3), (350, 3, 64, 32, 5), (3000, 3, 12, 8, 2),
    (701, 3, 32, 32, 3), (1367, 3, 16, 32, 3), (2401, 1, 28, 28, 3), (685, 3, 32, 20, 5), (1000, 2, 24, 40, 3),   # two images per wave
    (1401, 3, 32, 32, 3), (700, 3, 64, 32, 3), (1500, 3, 32, 28, 5),   # backward as separate launches (solve, then weight gradient)
    (4099, 3, 8, 8, 3), (2500, 3, 32, 32, 3), (2302, 1, 28, 28, 3),   # waves that walk over several pairs of images
    # 8 / 12 / 16 channels with the other kernel sizes of the kernel-size ablation (band kernel with k = 2, 5, 7)
    (2, 12, 16, 16, 5), (3, 8, 40, 24, 2), (2, 16, 33, 20, 5), (2, 12, 64, 24, 7), (1, 8, 16, 16, 7), (2, 16, 16, 16, 2),
    (2, 12, 20, 12, 2), (1, 16, 64, 9, 5), (3, 12, 7, 50, 5),
    # 8 / 12 / 16 channels with k = 9 and 11 (and 16 channels with k = 7): band kernel with its folded taps in LDS
    (3, 12, 16, 16, 9), (2, 12, 20, 12, 11), (2, 8, 33, 20, 9), (2, 16, 16, 16, 7), (1, 16, 40, 9, 9), (2, 16, 16, 16, 11),
    (1, 8, 64, 8, 11),
    # one band and k = 5 ... 11: the step split over four to seven waves by the age of its input
    (2, 12, 16, 16, 5), (2, 12, 7, 50, 5), (2, 8, 16, 20, 7), (1, 16, 9, 9, 9), (1, 8, 1, 8, 11), (2, 12, 16, 24, 11),
    (3, 12, 1, 1, 7), (2, 16, 13, 3, 5), (101, 12, 16, 16, 9),
    # channel counts between the band kernels' sizes (5-7, 9-11, 13-15): the next size up with the surplus slots off
    (3, 6, 16, 16, 3), (2, 5, 9, 11, 3), (2, 7, 33, 20, 3), (1, 10, 128, 40, 3), (2, 14, 40, 24, 3), (1, 15, 100, 8, 3),
    (2, 6, 20, 20, 2), (2, 10, 33, 16, 5), (1, 9, 40, 12, 7), (40, 6, 32, 32, 3), (2, 13, 16, 30, 3),
    # many channels, no multiple of 4 (17-47): the many-channel kernels with the surplus channels switched off
    (2, 17, 9, 11, 3), (1, 19, 40, 24, 3), (2, 23, 8, 8, 3), (1, 30, 96, 20, 3), (2, 33, 16, 16, 3), (1, 41, 64, 9, 3),
    (2, 45, 8, 8, 3), (3, 46, 8, 8, 3), (1, 37, 32, 32, 3),
    # shapes no on-chip kernel holds: one launch per anti-diagonal, a wave per pixel
    (5, 64, 4, 4, 3), (2, 96, 2, 2, 3), (1, 44, 70, 9, 3), (2, 128, 2, 3, 3), (1, 52, 5, 6, 2), (1, 64, 3, 3, 5),
    (2, 48, 8, 8, 5), (1, 48, 6, 5, 7), (1, 48, 4, 4, 11), (1, 64, 3, 3, 9),     # kernel rows of 1200 to 5808 entries
    # 8 / 12 channels, large batches or tall images: single-layer solves through the pipelined kernel
    (130, 12, 64, 64, 3), (26, 12, 100, 36, 3), (300, 8, 40, 24, 3), (40, 8, 128, 8, 3),
]


@pytest.mark.parametrize("shape", EDGE_SHAPES)
@pytest.mark.parametrize("variant", [b.VARIANT_AUTO, b.VARIANT_DIAG_LAUNCH, b.VARIANT_PERSISTENT])
def test_edge_shapes(shape, variant):
    B, C, H, W, k = shape
    print(f"edge {shape} variant {variant}", flush=True)
    cs = inputs.make_case(B, C, H, W, k, seed=sum(shape), tap_std=0.05)
    check_layer(cs["y"], cs["w"][0], cs["g"], variant)


WAVE_SPLIT_SHAPES = [  # (B, C, H, W, k): few channels, at most 64 rows
    (1, 1, 1, 1, 3), (3, 2, 7, 13, 3), (2, 3, 13, 7, 3), (1, 4, 1, 40, 3), (1, 4, 40, 1, 3), (2, 3, 2, 2, 5),
    (2, 3, 64, 5, 3), (3, 1, 33, 20, 3), (1, 2, 64, 64, 3), (2, 4, 63, 9, 3), (1, 3, 5, 100, 5), (1, 3, 64, 150, 3),
    (2, 3, 31, 33, 5), (1, 4, 64, 64, 3),
]


@pytest.mark.parametrize("shape", WAVE_SPLIT_SHAPES)
def test_wave_split_variant_edge_shapes(shape):
    B, C, H, W, k = shape
    print(f"wave split {shape}", flush=True)
    cs = inputs.make_case(B, C, H, W, k, seed=sum(shape) + 1, tap_std=0.05)
    check_layer(cs["y"], cs["w"][0], cs["g"], b.VARIANT_WAVE_SPLIT)


LARGE_K_SHAPES = [  # (B, C, H, W, k): the kernel sizes of the paper's kernel-size ablation, three channels
    (2, 3, 32, 32, 2), (2, 3, 32, 32, 7), (2, 3, 28, 28, 9), (1, 3, 32, 32, 11), (2, 3, 64, 40, 7), (2, 3, 20, 9, 11),
    (1, 3, 5, 50, 9), (3, 3, 64, 64, 11), (1, 3, 100, 20, 7), (2, 3, 7, 7, 2), (2, 3, 128, 64, 11), (1, 3, 256, 32, 9),
]


@pytest.mark.parametrize("shape", LARGE_K_SHAPES)
@pytest.mark.parametrize("variant", [b.VARIANT_AUTO, b.VARIANT_WAVE, b.VARIANT_WAVE_SPLIT])
def test_kernel_size_ablation_shapes(shape, variant):
    B, C, H, W, k = shape
    if variant == b.VARIANT_WAVE_SPLIT and (k < 3 or H > 64):
        pytest.skip("the four-wave split needs k >= 3 and at most 64 rows")
    if variant == b.VARIANT_WAVE and H > 64 and k > 5:
        pytest.skip("bands of 64 rows exist up to k = 5")
    print(f"kernel size {shape} variant {variant}", flush=True)
    cs = inputs.make_case(B, C, H, W, k, seed=sum(shape) + 2, tap_std=0.15 / k)
    check_layer(cs["y"], cs["w"][0], cs["g"], variant)


def test_bands_on_many_compute_units_at_full_occupancy():
    """512 band workgroups at once (128 images of 3 x 256 x 256, scratch from the caller): every image
    and dL/dw against the oracle, and the same results from the calls that take no workspace."""
    import torch
    B, C, H, W, k = 128, 3, 256, 256, 3
    cs = inputs.make_case(B, C, H, W, k, seed=77, tap_std=0.05)
    y, w, g = cs["y"], cs["w"][0], cs["g"]
    yd, wd, gd = dev(y), dev(w), dev(g)
    ws_f = b.new_workspace(b.fwd_workspace_bytes(B, C, H, W, k))
    ws_b = b.new_workspace(b.bwd_workspace_bytes(B, C, H, W, k))
    x = b.invconv_fwd(yd, wd, workspace=ws_f)
    v, dw = b.invconv_bwd(x, wd, gd, workspace=ws_b)
    x1 = b.invconv_fwd(yd, wd)                   # all bands of an image in one workgroup
    torch.cuda.synchronize()
    assert b.workspace_error(ws_f) == 0 and b.workspace_error(ws_b) == 0
    # (the kernel whose rows pass through LDS adds the terms of a pixel in another order: close, not equal)
    assert rel_err(host(x), host(x1)) <= 1e-5
    xh, vh = host(x), host(v)
    xr = oracle.invconv_fwd(y, w, THREADS)
    print("oracle fwd done", flush=True)
    vr, dwr = oracle.invconv_bwd(xh, w, g, THREADS)
    print("oracle bwd done", flush=True)
    for n in range(B):
        assert rel_err(xh[n], xr[n]) <= TOL_ACT, f"x of image {n}"
        assert rel_err(vh[n], vr[n]) <= TOL_ACT, f"dL/dy of image {n}"
    assert rel_err(host(dw), dwr) <= TOL_DW


TALL_SHAPES = [(2, 3, 256, 160, 3), (1, 3, 512, 512, 3), (5, 2, 257, 129, 3), (2, 3, 200, 130, 5), (1, 3, 130, 40, 5),
               # rows through the LDS ring (W a multiple of 4): ragged last chunk, ragged last band, every C, k = 2, 5
               (3, 3, 200, 132, 3), (2, 1, 193, 140, 3), (1, 4, 256, 128, 3), (2, 3, 192, 144, 5), (2, 2, 130, 128, 2),
               (1, 3, 129, 256, 3), (70, 3, 256, 128, 3)]


WIDE_K_SHAPES = [  # (B, C, H, W, k): many channels with the other kernel sizes of the kernel-size ablation
    (2, 48, 8, 8, 5), (2, 48, 8, 8, 2), (1, 48, 6, 5, 7), (1, 48, 4, 4, 11), (2, 24, 20, 12, 5), (1, 32, 32, 9, 2),
    (2, 20, 16, 16, 9), (1, 40, 9, 30, 7), (3, 28, 1, 1, 5), (1, 36, 13, 17, 11), (101, 48, 8, 8, 9),
]


@pytest.mark.parametrize("shape", WIDE_K_SHAPES)
def test_many_channels_other_kernel_sizes_with_workspace(shape):
    """With a workspace the folded weights of the call are streamed from it (one workgroup per image on the matrix
    cores); without one the same shapes take the per-diagonal fallback.  Both against the oracle."""
    import torch
    B, C, H, W, k = shape
    print(f"many channels, k != 3: {shape}", flush=True)
    cs = inputs.make_case(B, C, H, W, k, seed=sum(shape) + 11, tap_std=0.15 / k)
    yd, wd, gd = dev(cs["y"]), dev(cs["w"][0]), dev(cs["g"])
    assert b.fwd_workspace_bytes(B, C, H, W, k) > 256
    wsf = b.new_workspace(b.fwd_workspace_bytes(B, C, H, W, k))
    wsb = b.new_workspace(b.bwd_workspace_bytes(B, C, H, W, k))
    x = b.invconv_fwd(yd, wd, workspace=wsf)
    v, dw = b.invconv_bwd(x, wd, gd, workspace=wsb)
    torch.cuda.synchronize()
    xh = host(x)
    xr = oracle.invconv_fwd(cs["y"], cs["w"][0], THREADS)
    vr, dwr = oracle.invconv_bwd(xh, cs["w"][0], cs["g"], THREADS)
    assert rel_err(xh, xr) <= TOL_ACT and elementwise_ok(xh, xr, TOL_ACT)
    assert rel_err(host(v), vr) <= TOL_ACT and rel_err(host(dw), dwr) <= TOL_DW
    if B <= 3:
        x_plain = b.invconv_fwd(yd, wd)
        torch.cuda.synchronize()
        assert rel_err(host(x_plain), xr) <= TOL_ACT


MANY_SMALL_IMAGES = [  # (B, C, H, W, k): images of one row chunk in batches large enough for 2 .. 16 per workgroup
    (201, 48, 8, 8, 3), (1700, 12, 4, 4, 3), (331, 24, 8, 8, 5), (1537, 16, 8, 4, 3), (13000, 8, 2, 2, 3),
    (1030, 12, 16, 16, 3), (401, 24, 13, 16, 3), (513, 12, 10, 16, 7),      # 9 to 16 rows: one chunk of 16 rows
    (601, 12, 4, 8, 7),                                                      # fewer rows than the kernel's halo
]


@pytest.mark.parametrize("shape", MANY_SMALL_IMAGES)
def test_weight_gradient_of_many_small_images(shape):
    """Large batches of images that fit one row chunk: a workgroup of the weight-gradient kernel takes several
    images one after the other into the same accumulators (ragged last group included)."""
    import torch
    B, C, H, W, k = shape
    print(f"many small images: {shape}", flush=True)
    cs = inputs.make_case(B, C, H, W, k, seed=sum(shape) + 17, tap_std=0.15 / k)
    wd, gd = dev(cs["w"][0]), dev(cs["g"])
    xd = b.invconv_fwd(dev(cs["y"]), wd)
    ws = b.new_workspace(b.bwd_workspace_bytes(B, C, H, W, k))
    v, dw = b.invconv_bwd(xd, wd, gd, workspace=ws)
    torch.cuda.synchronize()
    vr, dwr = oracle.invconv_bwd(host(xd), cs["w"][0], cs["g"], THREADS)
    assert rel_err(host(v), vr) <= TOL_ACT and rel_err(host(dw), dwr) <= TOL_DW


WIDE_WS_SHAPES = [  # (B, C, H, W, k): many channels, 3 x 3, every group count C/4 = 5 .. 12, one to several bands
    (2, 48, 8, 8, 3), (3, 20, 5, 7, 3), (2, 24, 40, 9, 3), (1, 28, 33, 6, 3), (2, 32, 64, 5, 3), (1, 36, 17, 17, 3),
    (2, 40, 20, 9, 3), (1, 44, 16, 3, 3), (1, 48, 64, 4, 3), (101, 48, 8, 8, 3), (2, 22, 9, 9, 3),
]


@pytest.mark.parametrize("shape", WIDE_WS_SHAPES)
def test_many_channels_with_workspace_fold_the_weights_once(shape):
    """Many channels, 3 x 3: a call that brings a workspace folds the weights once, by a launch of its own, and
    its workgroups read them from there; a call without one folds them in every workgroup (and so does a channel
    count that is no multiple of 4, whose workspace is the header alone).  Both against the oracle."""
    import torch
    B, C, H, W, k = shape
    print(f"many channels, k = 3, workspace: {shape}", flush=True)
    cs = inputs.make_case(B, C, H, W, k, seed=sum(shape) + 13, tap_std=0.05)
    yd, wd, gd = dev(cs["y"]), dev(cs["w"][0]), dev(cs["g"])
    assert (b.fwd_workspace_bytes(B, C, H, W, k) > 256) == (C % 4 == 0)
    wsf = b.new_workspace(b.fwd_workspace_bytes(B, C, H, W, k))
    wsb = b.new_workspace(b.bwd_workspace_bytes(B, C, H, W, k))
    x = b.invconv_fwd(yd, wd, workspace=wsf)
    x_plain = b.invconv_fwd(yd, wd)
    v, dw = b.invconv_bwd(x, wd, gd, workspace=wsb)
    torch.cuda.synchronize()
    xh = host(x)
    xr = oracle.invconv_fwd(cs["y"], cs["w"][0], THREADS)
    vr, dwr = oracle.invconv_bwd(xh, cs["w"][0], cs["g"], THREADS)
    assert rel_err(xh, xr) <= TOL_ACT and elementwise_ok(xh, xr, TOL_ACT)
    assert rel_err(host(x_plain), xr) <= TOL_ACT and elementwise_ok(host(x_plain), xr, TOL_ACT)
    assert rel_err(host(v), vr) <= TOL_ACT and rel_err(host(dw), dwr) <= TOL_DW


@pytest.mark.parametrize("shape", TALL_SHAPES)
def test_tall_images_with_and_without_workspace_agree(shape):
    """invconv_fwd_ws / invconv_bwd spread the bands of an image over workgroups (logs in the caller's
    workspace); invconv_fwd keeps them in one workgroup (or, where the logs do not fit, uses the LDS-window
    kernel).  Same arithmetic per band: bit-identical where both run bands, and both match the oracle."""
    import torch
    B, C, H, W, k = shape
    print(f"tall {shape}", flush=True)
    cs = inputs.make_case(B, C, H, W, k, seed=sum(shape) + 9, tap_std=0.05)
    yd, wd = dev(cs["y"]), dev(cs["w"][0])
    ws = b.new_workspace(b.fwd_workspace_bytes(B, C, H, W, k))
    x_ws = b.invconv_fwd(yd, wd, workspace=ws)
    x_plain = b.invconv_fwd(yd, wd)
    torch.cuda.synchronize()
    assert b.workspace_error(ws) == 0
    xr = oracle.invconv_fwd(cs["y"], cs["w"][0], THREADS)
    assert rel_err(host(x_ws), xr) <= TOL_ACT and rel_err(host(x_plain), xr) <= TOL_ACT
    if H * W < 512 * 512:
        if W % 4 == 0 and W >= 64:      # rows through the LDS ring: the terms of a pixel are added in another order
            assert rel_err(host(x_ws), host(x_plain)) <= 1e-5
        else:
            assert torch.equal(x_ws, x_plain)
    # a workspace of the bare header is enough for any shape: it only changes which kernel runs
    tiny = b.new_workspace(0)
    if b.fwd_workspace_bytes(B, C, H, W, k) > 256:
        with pytest.raises(b.InvconvError) as ei:
            b.invconv_fwd(yd, wd, workspace=tiny)
        assert ei.value.status == b.ERR_WORKSPACE


@pytest.mark.parametrize("shape", [(2, 6, 16, 16, 3), (2, 10, 40, 24, 3), (3, 15, 20, 12, 5), (2, 22, 16, 12, 3),
                                   (1, 45, 8, 8, 3)])
def test_masked_garbage_with_surplus_channel_slots(shape):
    """Channel counts that run the band or many-channel kernels with surplus channel slots: entries above the
    diagonal of the current-pixel block are ignored and get zero gradient, and the surplus slots leak nothing into
    the results."""
    B, C, H, W, k = shape
    iu = np.triu_indices(C, 1)
    cs = inputs.make_case(B, C, H, W, k, seed=sum(shape) + 5, tap_std=0.1 / k)
    y, w, g = cs["y"], cs["w"][0].copy(), cs["g"]
    ref = run_layer(y, w, g)
    w[:, :, k - 1, k - 1][iu] = 1e6
    got = run_layer(y, w, g)
    for a, r in zip(got[:3], ref[:3]):
        np.testing.assert_array_equal(a, r)
    assert np.all(got[2][:, :, k - 1, k - 1][iu] == 0.0)
    xr = oracle.invconv_fwd(y, w, THREADS)
    assert rel_err(got[0], xr) <= TOL_ACT


def test_masked_garbage_at_twelve_channels():
    """Values above the diagonal of the current-pixel block are ignored by every kernel family that handles
    8-16 channels (band solve, pipelined solve, matrix-core dL/dw, chain calls) and get zero gradient."""
    import torch
    iu = np.triu_indices(12, 1)
    for shape in [(2, 12, 16, 16, 3), (24, 12, 96, 8, 3), (3, 12, 40, 24, 3)]:
        B, C, H, W, k = shape
        cs = inputs.make_case(B, C, H, W, k, seed=sum(shape) + 4, tap_std=0.03)
        y, w, g = cs["y"], cs["w"][0].copy(), cs["g"]
        ref = run_layer(y, w, g)
        w[:, :, 2, 2][iu] = 1e6
        got = run_layer(y, w, g)
        for a, r in zip(got[:3], ref[:3]):
            np.testing.assert_array_equal(a, r)
        assert np.all(got[2][:, :, 2, 2][iu] == 0.0)
        # and against the oracle, which masks by definition
        xr = oracle.invconv_fwd(y, w, THREADS)
        assert rel_err(got[0], xr) <= TOL_ACT
    # the chain calls
    L, B, C, H, W, k = 3, 2, 12, 33, 20, 3
    cases = [inputs.make_case(B, C, H, W, k, seed=300 + l, tap_std=0.03) for l in range(L)]
    ws_clean = [cs["w"][0] for cs in cases]
    ws_dirty = [w.copy() for w in ws_clean]
    for w in ws_dirty:
        w[:, :, 2, 2][iu] = -7e5
    outs = []
    for ws in (ws_clean, ws_dirty):
        wd = [dev(w) for w in ws]
        xs = b.invconv_chain_fwd(dev(cases[0]["y"]), wd)
        dy, dws = b.invconv_chain_bwd(xs, wd, dev(cases[0]["g"]))
        torch.cuda.synchronize()
        outs.append(([host(t) for t in xs], host(dy), [host(t) for t in dws]))
    for l in range(L):
        np.testing.assert_array_equal(outs[0][0][l], outs[1][0][l])
        np.testing.assert_array_equal(outs[0][2][l], outs[1][2][l])
        assert np.all(outs[1][2][l][:, :, 2, 2][iu] == 0.0)
    np.testing.assert_array_equal(outs[0][1], outs[1][1])


def test_gpu_properties_shift_invariance_and_batch_additivity():
    """Causal shift invariance of the solve and batch additivity of dL/dw, on the GPU's own outputs."""
    cs = inputs.make_case(4, 3, 24, 24, 3, seed=12, tap_std=0.05)
    y, w, g = cs["y"], cs["w"][0], cs["g"]
    x, v, dw, _ = run_layer(y, w, g)
    ys = np.zeros_like(y)
    ys[:, :, 3:, 5:] = y[:, :, :-3, :-5]           # shifted down 3, right 5, zero fill
    xs, _, _, _ = run_layer(ys, w, g)
    assert rel_err(xs[:, :, 3:, 5:], x[:, :, :-3, :-5]) <= 1e-5
    assert np.all(xs[:, :, :3, :] == 0.0) and np.all(xs[:, :, :, :5] == 0.0)
    parts = [run_layer(y[n:n + 1], w, g[n:n + 1])[2].astype(np.float64) for n in range(4)]
    assert rel_err(dw, sum(parts)) <= 1e-5


def test_masked_entries_are_ignored_and_get_zero_gradient():
    cs = inputs.make_case(2, 4, 9, 8, 3, seed=3)
    y, w, g = cs["y"], cs["w"][0].copy(), cs["g"]
    ref = run_layer(y, w, g)
    iu = np.triu_indices(4, 1)
    w[:, :, 2, 2][iu] = 1e6     # garbage above the diagonal of the current-pixel block
    got = run_layer(y, w, g)
    for a, r in zip(got[:3], ref[:3]):
        np.testing.assert_array_equal(a, r)
    assert np.all(got[2][:, :, 2, 2][iu] == 0.0)


FWD_LOGDET_SHAPES = [(4, 3, 8, 8, 3), (16, 3, 32, 32, 3), (32, 3, 64, 64, 5), (2, 1, 5, 5, 3), (700, 2, 50, 10, 3),
                     (64, 12, 16, 16, 3), (2, 3, 130, 40, 3), (1, 20, 6, 7, 2),
                     # band and many-channel kernels with the log-determinant formed by a spare wave
                     (2, 12, 40, 24, 3), (3, 8, 128, 8, 3), (2, 48, 32, 32, 3), (1, 28, 128, 8, 3), (1, 16, 16, 5, 3)]


@pytest.mark.parametrize("shape", FWD_LOGDET_SHAPES)
def test_fwd_logdet_matches_the_two_separate_calls_and_the_oracle(shape):
    """invconv_fwd_logdet = invconv_fwd + invconv_logdet (one launch for few-channel images)."""
    import torch
    B, C, H, W, k = shape
    cs = inputs.make_case(B, C, H, W, k, seed=sum(shape) + 13, tap_std=0.05)
    yd, wd = dev(cs["y"]), dev(cs["w"][0])
    x, ld = b.invconv_fwd_logdet(yd, wd)
    x2 = b.invconv_fwd(yd, wd)
    ld2 = b.invconv_logdet(wd, H, W)
    torch.cuda.synchronize()
    assert torch.equal(x, x2)
    ref = oracle.invconv_logdet(cs["w"][0], H, W)
    assert abs(float(ld[0]) - ref) <= 1e-5 * max(1.0, abs(ref))
    assert abs(float(ld[0]) - float(ld2[0])) <= 1e-6 * max(1.0, abs(ref))
    assert rel_err(host(x), oracle.invconv_fwd(cs["y"], cs["w"][0], THREADS)) <= TOL_ACT
    # the paper's unit diagonal: exactly 0
    w1 = cs["w"][0].copy()
    for c in range(C):
        w1[c, c, k - 1, k - 1] = 1.0
    _, ld1 = b.invconv_fwd_logdet(yd, dev(w1))
    assert float(ld1[0]) == 0.0


def test_dw_is_bitwise_reproducible():
    wl = inputs.make_workload(2)
    first = run_layer(wl["y"], wl["w"][0], wl["g"])
    for _ in range(5):
        again = run_layer(wl["y"], wl["w"][0], wl["g"])
        for a, r in zip(again[:3], first[:3]):
            np.testing.assert_array_equal(a, r)


def test_adjoint_identity_on_gpu():
    # <fwd(y), g> = <y, bwd_dy(g)> holds at any size; checked here in float64 on the GPU's outputs.
    wl = inputs.make_workload(3)
    x, v, _, _ = run_layer(wl["y"], wl["w"][0], wl["g"])
    lhs = np.sum(x.astype(np.float64) * wl["g"])
    rhs = np.sum(wl["y"].astype(np.float64) * v)
    assert lhs == pytest.approx(rhs, rel=1e-4)


def test_binding_error_paths_on_gpu():
    import torch
    y = torch.zeros(1, 2, 4, 4, device="cuda")
    w = torch.zeros(2, 2, 3, 3, device="cuda")
    with pytest.raises(b.InvconvError) as ei:
        b.invconv_fwd(y, w, out=y)
    assert ei.value.status == b.ERR_ALIAS
    with pytest.raises(b.InvconvError) as ei:
        b.invconv_bwd(y, w, torch.zeros_like(y), workspace=torch.empty(16, dtype=torch.uint8, device="cuda"))
    assert ei.value.status == b.ERR_WORKSPACE


def test_chain_workload_parity():
    """Training-step chain: 8 stacked layers forward, loss 0.5*sum(x^2), then backward through all 8."""
    import torch
    wl = inputs.make_workload(4)
    H, W = wl["H"], wl["W"]
    ws = [dev(w) for w in wl["w"]]
    acts = [dev(wl["y"])]
    for wd in ws:
        acts.append(b.invconv_fwd(acts[-1], wd))
    g = acts[-1]
    dws = [None] * len(ws)
    for l in reversed(range(len(ws))):
        g, dws[l] = b.invconv_bwd(acts[l + 1], ws[l], g)
    lds = [b.invconv_logdet(wd, H, W) for wd in ws]
    torch.cuda.synchronize()
    # oracle chain in fp64 from the same fp32 inputs
    xr = [wl["y"].astype(np.float64)]
    for w in wl["w"]:
        xr.append(oracle.invconv_fwd(xr[-1], w, THREADS))
        print("oracle fwd layer done", flush=True)
    gr = xr[-1]
    for l in reversed(range(len(ws))):
        assert rel_err(host(acts[l + 1]), xr[l + 1]) <= TOL_ACT
        gr, dwr = oracle.invconv_bwd(xr[l + 1], wl["w"][l], gr, THREADS)
        print("oracle bwd layer done", l, flush=True)
        assert rel_err(host(dws[l]), dwr) <= TOL_DW
        assert float(host(lds[l])[0]) == pytest.approx(oracle.invconv_logdet(wl["w"][l], H, W), rel=1e-5)
    assert rel_err(host(g), gr) <= TOL_ACT


CHAIN_SHAPES = [  # (L, B, C, H, W, k)
    (1, 2, 12, 16, 16, 3), (3, 2, 12, 16, 20, 3), (2, 3, 12, 40, 9, 3), (4, 1, 8, 33, 31, 3),
    (2, 2, 16, 128, 12, 3), (3, 2, 12, 7, 5, 3), (2, 2, 12, 20, 3, 3), (2, 2, 16, 64, 16, 3), (3, 1, 8, 128, 4, 3),
    (2, 2, 3, 10, 10, 3),          # not covered by the pipelined kernel: falls back to per-layer launches
    # more (layer, image) workgroups than the device holds at once: several launches of whole layers
    (3, 100, 12, 128, 8, 3), (8, 40, 12, 128, 16, 3), (2, 300, 8, 128, 4, 3),
]


def oracle_chain(y, ws, g_last):
    xs = [np.asarray(y, dtype=np.float64)]
    for w in ws:
        xs.append(oracle.invconv_fwd(xs[-1], w, THREADS))
    return xs[1:]


@pytest.mark.parametrize("shape", CHAIN_SHAPES)
def test_chain_calls_match_oracle(shape):
    import torch
    L, B, C, H, W, k = shape
    print(f"chain {shape}", flush=True)
    cases = [inputs.make_case(B, C, H, W, k, seed=100 + l, tap_std=0.03) for l in range(L)]
    ws = [cs["w"][0] for cs in cases]
    y, g_last = cases[0]["y"], cases[0]["g"]
    wd = [dev(w) for w in ws]
    xs = b.invconv_chain_fwd(dev(y), wd)
    dy, dws = b.invconv_chain_bwd(xs, wd, dev(g_last))
    torch.cuda.synchronize()
    xr = oracle_chain(y, ws, g_last)
    lds = host(b.invconv_chain_logdet(wd, H, W))
    for l in range(L):
        assert rel_err(host(xs[l]), xr[l]) <= TOL_ACT, f"x of layer {l}"
        assert float(lds[l]) == pytest.approx(oracle.invconv_logdet(ws[l], H, W), rel=1e-5, abs=1e-5)
    # backward oracle on the GPU's own activations
    gr = g_last.astype(np.float64)
    for l in reversed(range(L)):
        gr, dwr = oracle.invconv_bwd(host(xs[l]), ws[l], gr, THREADS)
        assert rel_err(host(dws[l]), dwr) <= TOL_DW, f"dw of layer {l}"
    assert rel_err(host(dy), gr) <= TOL_ACT


def test_chain_workload4_matches_per_layer_calls_and_oracle():
    import torch
    wl = inputs.make_workload(4)
    H, W = wl["H"], wl["W"]
    wd = [dev(w) for w in wl["w"]]
    yd = dev(wl["y"])
    xs = b.invconv_chain_fwd(yd, wd)
    dy, dws = b.invconv_chain_bwd(xs, wd, xs[-1])
    torch.cuda.synchronize()
    # per-layer calls of the plain API
    acts = [yd]
    for w in wd:
        acts.append(b.invconv_fwd(acts[-1], w))
    g = acts[-1]
    dws2 = [None] * len(wd)
    for l in reversed(range(len(wd))):
        g, dws2[l] = b.invconv_bwd(acts[l + 1], wd[l], g)
    torch.cuda.synchronize()
    for l in range(len(wd)):
        assert rel_err(host(xs[l]), host(acts[l + 1])) <= 1e-5
        assert rel_err(host(dws[l]), host(dws2[l])) <= 1e-4
    assert rel_err(host(dy), host(g)) <= 1e-5
    # and the oracle for the forward chain (the backward chain is covered by test_chain_workload_parity)
    xr = wl["y"].astype(np.float64)
    for l, w in enumerate(wl["w"]):
        xr = oracle.invconv_fwd(xr, w, THREADS)
        assert rel_err(host(xs[l]), xr) <= TOL_ACT


def test_hip_graph_replays_match_eager():
    """A captured step (fwd + bwd + logdet) replayed several times, with eager work in between,
    gives the eager results every time (the library records kernel nodes only)."""
    import torch
    wl = inputs.make_workload(1)
    y, w, g = dev(wl["y"]), dev(wl["w"][0]), dev(wl["g"])
    x, v, dw = torch.empty_like(y), torch.empty_like(y), torch.empty_like(w)
    ld = torch.empty(1, device="cuda")
    wsp = b.new_workspace(b.bwd_workspace_bytes(16, 3, 32, 32, 3))

    def step():
        b.invconv_fwd(y, w, out=x)
        b.invconv_bwd(x, w, g, out=(v, dw), workspace=wsp)
        b.invconv_logdet(w, 32, 32, out=ld)

    step()
    torch.cuda.synchronize()
    ref = [t.clone() for t in (x, v, dw, ld)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(4):
        for t in (x, v, dw, ld):
            t.fill_(float("nan"))             # eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for t, r in zip((x, v, dw, ld), ref):
            assert torch.equal(t, r), f"replay {rep}"


def test_hip_graph_of_a_tall_image_solve_matches_eager():
    """Tall few-channel images with scratch from the caller: the bands of an image run on different compute
    units, eagerly and when captured into a graph alike (the library allocates nothing)."""
    import torch
    cs = inputs.make_case(2, 3, 256, 160, 3, seed=31, tap_std=0.05)
    y, w = dev(cs["y"]), dev(cs["w"][0])
    ws = b.new_workspace(b.fwd_workspace_bytes(2, 3, 256, 160, 3))
    x = torch.empty_like(y)
    b.invconv_fwd(y, w, out=x, workspace=ws)
    torch.cuda.synchronize()
    ref = x.clone()
    assert rel_err(host(ref), oracle.invconv_fwd(cs["y"], cs["w"][0], THREADS)) <= TOL_ACT
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        b.invconv_fwd(y, w, out=x, workspace=ws)
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        b.invconv_fwd(y, w, out=x, workspace=ws)
    for rep in range(3):
        x.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(x, ref), f"replay {rep}"
    assert b.workspace_error(ws) == 0


def test_error_word_stays_clear_and_is_set_when_a_wait_gives_up():
    """Bounded waits: in normal operation none runs out (error word stays 0).  With the wait budget cut to
    one poll from the host, the waits of the multi-workgroup kernels run out at once: every kernel still
    ends, the error word is 1 and the outputs that lost their input are NaN, never plausible numbers."""
    import torch
    L, B, C, H, W, k = 4, 3, 12, 48, 40, 3
    cases = [inputs.make_case(B, C, H, W, k, seed=200 + l, tap_std=0.03) for l in range(L)]
    wd = [dev(cs["w"][0]) for cs in cases]
    yd = dev(cases[0]["y"])
    need = b.chain_workspace_bytes(L, B, C, H, W, k)
    # tall images: rows of 158 floats are read by the solving wave itself, rows of 160 pass through the LDS
    # ring that a second wave fills (so there even the top band has somebody to wait for)
    talls = []
    for TW in (158, 160):
        tall = inputs.make_case(2, 3, 256, TW, 3, seed=41, tap_std=0.05)
        talls.append((dev(tall["y"]), dev(tall["w"][0]), b.fwd_workspace_bytes(2, 3, 256, TW, 3)))
    # normal operation
    wsp = b.new_workspace(need)
    xs = b.invconv_chain_fwd(yd, wd, workspace=wsp)
    txs = []
    for ty, tw, tneed in talls:
        tws = b.new_workspace(tneed)
        txs.append(b.invconv_fwd(ty, tw, workspace=tws))
        torch.cuda.synchronize()
        assert b.workspace_error(tws) == 0
    assert b.workspace_error(wsp) == 0
    try:
        b.set_wait_budget(1)
        wsp2 = b.new_workspace(need)
        xs2 = b.invconv_chain_fwd(yd, wd, workspace=wsp2)
        lost = []
        for ty, tw, tneed in talls:
            tws2 = b.new_workspace(tneed)
            tx2 = b.invconv_fwd(ty, tw, workspace=tws2)
            tx3 = b.invconv_fwd(ty, tw)             # no workspace: no error word, but NaN all the same
            lost.append((tws2, tx2, tx3))
        torch.cuda.synchronize()
    finally:
        b.set_wait_budget(0)
    assert b.workspace_error(wsp2) == 1
    assert torch.equal(xs2[0], xs[0])               # the first layer waits for nobody
    assert bool(torch.isnan(xs2[-1]).any())
    for i, (tws2, tx2, tx3) in enumerate(lost):
        assert b.workspace_error(tws2) == 1
        assert bool(torch.isnan(tx2[:, :, 64:]).any()) and bool(torch.isnan(tx3[:, :, 64:]).any())
        ok = ~torch.isnan(tx2)                      # whatever is not NaN is the right number
        assert torch.equal(tx2[ok], txs[i][ok])
    assert torch.equal(lost[0][1][:, :, :64], txs[0][:, :, :64])     # W = 158: the top band waits for nobody
    # the word is sticky until the caller clears the header; a fresh run on a cleared header is clean
    wsp2[:256].zero_()
    xs3 = b.invconv_chain_fwd(yd, wd, workspace=wsp2)
    torch.cuda.synchronize()
    assert b.workspace_error(wsp2) == 0
    for a, r in zip(xs3, xs):
        assert torch.equal(a, r)
