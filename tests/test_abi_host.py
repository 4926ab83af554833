"""Host-only checks of the C ABI: the library loads, exports what the header declares,
and rejects bad arguments before touching the GPU."""
import ctypes
import os
import re

import pytest

from paper_2410_14634_amd import binding as b

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = [0x10000 * (i + 1) for i in range(8)]   # never dereferenced: every call below must fail validation


def declared_functions():
    import glob
    names = set()
    for path in glob.glob(os.path.join(ROOT, "include", "*.h")):
        text = re.sub(r"/\*.*?\*/", "", open(path).read(), flags=re.S)
        names.update(re.findall(r"\b(invconv_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    L = b.lib()
    names = declared_functions()
    assert set(names) == set(b.EXPORTS)
    for name in names:
        assert getattr(L, name) is not None
    assert b.version() >= 100


def test_status_strings():
    seen = {b.status_string(s) for s in range(0, -8, -1)}
    assert len(seen) == 8 and b.status_string(-99) == "unknown status"


def test_fwd_rejects_bad_arguments():
    L = b.lib()
    y, w, x = FAKE[:3]
    assert L.invconv_fwd(None, w, x, 1, 1, 4, 4, 3, None) == b.ERR_NULL
    assert L.invconv_fwd(y, None, x, 1, 1, 4, 4, 3, None) == b.ERR_NULL
    assert L.invconv_fwd(y, w, None, 1, 1, 4, 4, 3, None) == b.ERR_NULL
    for bad in [(0, 1, 4, 4, 3), (1, 0, 4, 4, 3), (1, 1, 0, 4, 3), (1, 1, 4, 0, 3), (1, 1, 4, 4, 0),
                (-1, 1, 4, 4, 3), (2 ** 20, 64, 64, 64, 3),
                (1, 1, 32768, 16384, 3)]:      # one image of 2^29 elements: past the 32-bit byte offsets
        assert L.invconv_fwd(y, w, x, *bad, None) == b.ERR_SHAPE
    assert L.invconv_fwd(y, w, y, 1, 1, 4, 4, 3, None) == b.ERR_ALIAS
    assert L.invconv_fwd_ex(y, w, x, 1, 1, 4, 4, 3, None, 99) == b.ERR_VARIANT
    # on-chip buffers too small for this shape: the LDS-window variant asked for by name refuses, and so does the
    # default path when even its last resort (a wave per pixel, one launch per anti-diagonal) cannot hold a row of
    # the kernel (more than 8192 entries per output channel)
    assert L.invconv_fwd_ex(y, w, x, 1, 64, 2048, 1024, 11, None, b.VARIANT_BLOCK) == b.ERR_UNSUPPORTED
    assert L.invconv_fwd(y, w, x, 1, 80, 2048, 1024, 11, None) == b.ERR_UNSUPPORTED


def test_conv_rejects_bad_arguments():
    L = b.lib()
    x, w, y = FAKE[:3]
    assert L.invconv_conv_fwd(None, w, y, 1, 1, 4, 4, 3, None) == b.ERR_NULL
    assert L.invconv_conv_fwd(x, None, y, 1, 1, 4, 4, 3, None) == b.ERR_NULL
    assert L.invconv_conv_fwd(x, w, None, 1, 1, 4, 4, 3, None) == b.ERR_NULL
    assert L.invconv_conv_fwd(x, w, y, 1, 1, 0, 4, 3, None) == b.ERR_SHAPE
    assert L.invconv_conv_fwd(x, w, x, 1, 1, 4, 4, 3, None) == b.ERR_ALIAS


def test_conv_bwd_rejects_bad_arguments():
    L = b.lib()
    x, w, g, dx, dw, ws = FAKE[:6]
    need = L.invconv_bwd_workspace_bytes(2, 3, 8, 8, 3)
    assert L.invconv_conv_bwd(None, w, g, dx, dw, 2, 3, 8, 8, 3, ws, need, None) == b.ERR_NULL
    assert L.invconv_conv_bwd(x, w, g, None, dw, 2, 3, 8, 8, 3, ws, need, None) == b.ERR_NULL
    assert L.invconv_conv_bwd(x, w, g, dx, dw, 2, 3, 8, 0, 3, ws, need, None) == b.ERR_SHAPE
    assert L.invconv_conv_bwd(x, w, g, g, dw, 2, 3, 8, 8, 3, ws, need, None) == b.ERR_ALIAS
    assert L.invconv_conv_bwd(x, w, g, dx, dw, 2, 3, 8, 8, 3, None, need, None) == b.ERR_WORKSPACE
    assert L.invconv_conv_bwd(x, w, g, dx, dw, 2, 3, 8, 8, 3, ws, need - 1, None) == b.ERR_WORKSPACE


def test_bwd_rejects_bad_arguments():
    L = b.lib()
    x, w, g, v, dw, ws = FAKE[:6]
    shape = (2, 3, 8, 8, 3)
    need = b.bwd_workspace_bytes(*shape)
    assert need > 0 and need % 256 == 0
    assert L.invconv_bwd(None, w, g, v, dw, *shape, ws, need, None) == b.ERR_NULL
    assert L.invconv_bwd(x, w, g, None, dw, *shape, ws, need, None) == b.ERR_NULL
    assert L.invconv_bwd(x, w, g, v, None, *shape, ws, need, None) == b.ERR_NULL
    assert L.invconv_bwd(x, w, g, v, dw, 2, 3, 8, 8, 0, ws, need, None) == b.ERR_SHAPE
    assert L.invconv_bwd(x, w, g, g, dw, *shape, ws, need, None) == b.ERR_ALIAS
    assert L.invconv_bwd(x, w, g, x, dw, *shape, ws, need, None) == b.ERR_ALIAS
    assert L.invconv_bwd(x, w, g, v, dw, *shape, None, need, None) == b.ERR_WORKSPACE
    assert L.invconv_bwd(x, w, g, v, dw, *shape, ws, need - 1, None) == b.ERR_WORKSPACE
    assert L.invconv_bwd_ex(x, w, g, v, dw, *shape, ws, need, None, -1) == b.ERR_VARIANT
    assert b.bwd_workspace_bytes(0, 3, 8, 8, 3) == 0


def test_workspace_taking_calls_reject_bad_workspaces():
    L = b.lib()
    y, w, x, g, v, dw, ws = FAKE[:7]
    shape = (2, 3, 256, 256, 3)             # tall few-channel images: the solve can use scratch
    need = b.fwd_workspace_bytes(*shape)
    assert need > 256 and need % 256 == 0
    assert b.fwd_workspace_bytes(2, 3, 8, 8, 3) == 256          # header only
    assert b.fwd_workspace_bytes(2, 3, 8, 0, 3) == 0
    assert b.bwd_workspace_bytes(*shape) > need                  # the solve's share plus the dL/dw partial sums
    assert L.invconv_fwd_ws(y, w, x, *shape, None, need, None) == b.ERR_WORKSPACE
    assert L.invconv_fwd_ws(y, w, x, *shape, ws, need - 1, None) == b.ERR_WORKSPACE
    assert L.invconv_fwd_ws(y, w, x, *shape, ws + 16, need, None) == b.ERR_WORKSPACE     # not 256-byte aligned
    assert L.invconv_fwd_ws(None, w, x, *shape, ws, need, None) == b.ERR_NULL
    assert L.invconv_fwd_ws(y, w, y, *shape, ws, need, None) == b.ERR_ALIAS
    assert L.invconv_bwd(x, w, g, v, dw, 2, 3, 8, 8, 3, ws + 16, 1 << 20, None) == b.ERR_WORKSPACE
    assert L.invconv_workspace_error(None, None, None) == b.ERR_NULL


def test_backward_workspace_covers_every_block_of_a_blocked_weight_gradient():
    """More than 16 channels, or more columns C k k than a wave has accumulators: dL/dw is formed in blocks of
    channels that share one launch, each block with partial rows of its own - the workspace grows with the
    number of blocks, stays a multiple of 256 bytes, and every shape with a solve has one."""
    one = b.bwd_workspace_bytes(8, 16, 32, 32, 3)                 # one GEMM
    nine = b.bwd_workspace_bytes(8, 48, 32, 32, 3)                # 3 x 3 blocks of 16 x 16 channels
    assert nine % 256 == 0 and nine > 8 * one
    k3 = b.bwd_workspace_bytes(8, 12, 16, 16, 3)                  # 108 columns: one GEMM
    k5 = b.bwd_workspace_bytes(8, 12, 16, 16, 5)                  # 300 columns: two blocks of 6 input channels
    assert k5 % 256 == 0 and k5 > k3
    for shape in [(2, 64, 4, 4, 3), (1, 96, 2, 2, 3), (3, 12, 16, 16, 7), (2, 3, 32, 32, 11), (1, 44, 95, 20, 3)]:
        assert b.bwd_workspace_bytes(*shape) > 256, shape         # (the solve of such shapes is the last-resort path)


def test_static_scratch_call_rejects_bad_arguments_and_oversized_shapes():
    L = b.lib()
    x, w, g, v, dw = FAKE[:5]
    assert L.invconv_bwd_static(None, w, g, v, dw, 2, 3, 8, 8, 3, None) == b.ERR_NULL
    assert L.invconv_bwd_static(x, w, g, v, dw, 2, 3, 8, 0, 3, None) == b.ERR_SHAPE
    big = (4096, 12, 128, 128, 3)
    assert b.bwd_workspace_bytes(*big) > 8 << 20
    assert L.invconv_bwd_static(x, w, g, v, dw, *big, None) == b.ERR_WORKSPACE


def test_logdet_rejects_bad_arguments():
    L = b.lib()
    assert L.invconv_logdet(None, 3, 8, 8, 3, FAKE[0], None) == b.ERR_NULL
    assert L.invconv_logdet(FAKE[0], 3, 8, 8, 3, None, None) == b.ERR_NULL
    assert L.invconv_logdet(FAKE[0], 0, 8, 8, 3, FAKE[1], None) == b.ERR_SHAPE


def test_binding_refuses_cpu_tensors():
    import torch
    with pytest.raises(TypeError):
        b.invconv_fwd(torch.zeros(1, 1, 4, 4), torch.zeros(1, 1, 3, 3))


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU: bench.py --gpus N with N > 1 exits with a message that says so."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr or "one GPU" in r.stderr
    assert r.stdout.strip() == ""
