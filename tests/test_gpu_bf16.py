"""GPU parity of the bf16-storage variant (activations as bf16 in memory, fp32 arithmetic) against the fp64 oracle
on the same bf16-exact inputs.  Tolerance: a stored result is the fp32 result rounded to bf16 (8 significant bits,
round to nearest even), i.e. within 2^-8 relative of it, on top of the fp32 path's own 1e-4 of the largest value;
dL/dw is fp32 and is formed from the unrounded dL/dy, so it keeps the 1e-3 gate."""
import numpy as np
import pytest

import oracle
from paper_2410_14634_amd import binding as b
from paper_2410_14634_amd import inputs
from tests.util import THREADS, TOL_DW, host, rel_err

pytestmark = pytest.mark.gpu

RTOL_BF16 = 2.0 ** -8
BF16_SHAPES = [  # (B, C, H, W, k)
    # on-chip form: few channels, image in LDS
    (16, 3, 32, 32, 3), (32, 3, 64, 64, 5), (5, 2, 33, 20, 3), (3, 1, 28, 28, 3), (300, 4, 16, 16, 3), (2, 3, 1, 4, 3),
    # conversion passes around the fp32 kernels
    (2, 12, 16, 16, 3), (2, 3, 130, 40, 3), (3, 3, 13, 7, 3), (1, 20, 6, 7, 2), (2, 3, 32, 32, 7),
]


def bf16_ok(a, ref) -> bool:
    a, ref = np.asarray(a, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    return bool(np.all(np.abs(a - ref) <= RTOL_BF16 * np.abs(ref) + 1e-4 * np.abs(ref).max()))


@pytest.mark.parametrize("shape", BF16_SHAPES)
def test_bf16_storage_parity(shape):
    import torch
    B, C, H, W, k = shape
    print(f"bf16 {shape}", flush=True)
    cs = inputs.make_case(B, C, H, W, k, seed=sum(shape) + 21, tap_std=0.05 if k <= 5 else 0.15 / k)
    w = cs["w"][0]
    wd = torch.from_numpy(w).cuda()
    y16 = torch.from_numpy(cs["y"]).cuda().to(torch.bfloat16)
    g16 = torch.from_numpy(cs["g"]).cuda().to(torch.bfloat16)
    ws = b.new_workspace(b.bf16_workspace_bytes(B, C, H, W, k))
    x16 = b.invconv_fwd_bf16(y16, wd, workspace=ws)
    v16, dw = b.invconv_bwd_bf16(x16, wd, g16, workspace=ws)
    torch.cuda.synchronize()
    assert b.workspace_error(ws) == 0
    y_exact, g_exact = host(y16.float()), host(g16.float())        # what the kernels read, exactly
    xr = oracle.invconv_fwd(y_exact, w, THREADS)
    xg = host(x16.float())
    assert bf16_ok(xg, xr), f"x rel err {rel_err(xg, xr)}"
    vr, dwr = oracle.invconv_bwd(xg, w, g_exact, THREADS)          # the backward pass is given the stored (bf16) x
    vg = host(v16.float())
    assert bf16_ok(vg, vr), f"dL/dy rel err {rel_err(vg, vr)}"
    assert rel_err(host(dw), dwr) <= TOL_DW
    # the fp32 calls on the same inputs, rounded afterwards, give the same stored values up to one bf16 step
    x32 = b.invconv_fwd(y16.float(), wd)
    torch.cuda.synchronize()
    assert bf16_ok(xg, host(x32))


def test_bf16_rejects_bad_arguments():
    import torch
    y16 = torch.zeros(1, 3, 8, 8, device="cuda", dtype=torch.bfloat16)
    w = torch.zeros(3, 3, 3, 3, device="cuda")
    with pytest.raises(b.InvconvError) as ei:
        b.invconv_fwd_bf16(y16, w, out=y16)
    assert ei.value.status == b.ERR_ALIAS
    with pytest.raises(b.InvconvError) as ei:
        b.invconv_fwd_bf16(y16, w, workspace=b.new_workspace(256))
    assert ei.value.status == b.ERR_WORKSPACE
    with pytest.raises(TypeError):
        b.invconv_fwd_bf16(y16.float(), w)
