"""The entry point that allocates nothing (invconv_bwd_static: the library's own static scratch) against
invconv_bwd with a caller workspace: same kernels, so the results are bit-identical, and both match the
oracle.  Two calls in a row, the second on a smaller input."""
import numpy as np
import pytest

import oracle
from paper_2410_14634_amd import binding as b
from paper_2410_14634_amd import inputs
from tests.util import THREADS, TOL_ACT, TOL_DW, dev, host, rel_err

pytestmark = pytest.mark.gpu


def _one(shape, seed):
    import torch
    B, C, H, W, k = shape
    cs = inputs.make_case(B, C, H, W, k, seed=seed, tap_std=0.04)
    wd, gd = dev(cs["w"][0]), dev(cs["g"])
    x = b.invconv_fwd(dev(cs["y"]), wd)
    v_ref, dw_ref = b.invconv_bwd(x, wd, gd)
    torch.cuda.synchronize()
    v, dw = torch.full_like(x, float("nan")), torch.full_like(wd, float("nan"))
    torch.cuda.synchronize()
    st = b.lib().invconv_bwd_static(x.data_ptr(), wd.data_ptr(), gd.data_ptr(), v.data_ptr(), dw.data_ptr(),
                                    B, C, H, W, k, torch.cuda.current_stream().cuda_stream)
    assert st == 0, b.status_string(st)
    torch.cuda.synchronize()
    assert torch.equal(v, v_ref) and torch.equal(dw, dw_ref)
    vr, dwr = oracle.invconv_bwd(host(x), cs["w"][0], cs["g"], THREADS)
    assert rel_err(host(v), vr) <= TOL_ACT and rel_err(host(dw), dwr) <= TOL_DW
    # the binding's wrapper hands back the tensors it was given
    v2, dw2 = b.invconv_bwd_static(x, wd, gd, out=(torch.empty_like(x), torch.empty_like(wd)))
    torch.cuda.synchronize()
    assert torch.equal(v2, v_ref) and torch.equal(dw2, dw_ref)


@pytest.mark.parametrize("first,second", [
    ((16, 3, 32, 32, 3), (5, 3, 20, 12, 3)),          # fused few-channel backward: one partial row per image
    ((8, 12, 64, 48, 3), (2, 12, 16, 16, 3)),         # band solve + matrix-core dL/dw partial rows
    ((3, 3, 256, 160, 3), (1, 3, 130, 40, 5)),        # tall images: band logs and counters in the scratch too
    ((2, 20, 9, 11, 3), (1, 5, 7, 7, 2)),             # generic kernels
])
def test_static_scratch_backward_matches_workspace_backward(first, second):
    print(f"no-alloc {first} then {second}", flush=True)
    _one(first, 11)
    _one(second, 12)


def test_static_scratch_backward_refuses_what_does_not_fit():
    import torch
    B, C, H, W, k = 4096, 12, 128, 128, 3          # needs more scratch than the library holds
    assert b.bwd_workspace_bytes(B, C, H, W, k) > 8 << 20
    t = torch.zeros(4, device="cuda")               # never touched: the call fails validation
    st = b.lib().invconv_bwd_static(t.data_ptr(), t.data_ptr(), t.data_ptr(), t.data_ptr(), t.data_ptr(),
                                    B, C, H, W, k, None)
    assert st == b.ERR_WORKSPACE
