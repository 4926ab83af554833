"""Thin ctypes binding over libinvconv.so: argument marshalling only.

PyTorch is used for device memory and the current HIP stream; every step of
the computation runs in the library's kernels.  There is no CPU fallback: if
the shared library has not been built this module raises at import of the
first symbol.
"""
from __future__ import annotations

import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libinvconv.so")

OK = 0
ERR_NULL, ERR_SHAPE, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_ALIAS, ERR_LAUNCH, ERR_VARIANT = range(-1, -8, -1)
VARIANT_AUTO, VARIANT_BLOCK, VARIANT_DIAG_LAUNCH, VARIANT_WAVE, VARIANT_BAND, VARIANT_PERSISTENT, VARIANT_WAVE_SPLIT = \
    0, 1, 2, 3, 4, 5, 6

EXPORTS = (
    "invconv_fwd", "invconv_bwd", "invconv_bwd_workspace_bytes", "invconv_logdet",
    "invconv_fwd_ex", "invconv_bwd_ex", "invconv_status_string", "invconv_version",
    "invconv_probe_step_sync", "invconv_chain_fwd", "invconv_chain_bwd", "invconv_chain_workspace_bytes",
    "invconv_chain_logdet", "invconv_conv_fwd", "invconv_conv_bwd",
    "invconv_fwd_logdet", "invconv_fwd_ws", "invconv_fwd_workspace_bytes", "invconv_workspace_error", "invconv_set_wait_budget",
    "invconv_bwd_static",
    "invconv_flowstep_fwd", "invconv_flowstep_bwd", "invconv_flowstep_workspace_bytes",
    "invconv_flowstep_fwd_ex", "invconv_flowstep_bwd_ex",
    "invconv_fwd_bf16", "invconv_bwd_bf16", "invconv_bf16_workspace_bytes",
)
FLOW_AUTO, FLOW_SEPARATE, FLOW_FUSED = 0, 1, 2
WS_HEADER_BYTES = 256

_lib = None


class InvconvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


def lib() -> ctypes.CDLL:
    """Load the HIP library; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2410_14634_amd.build` "
                "(or __graft_entry__.build()); there is no CPU fallback")
        L = ctypes.CDLL(LIB_PATH)
        vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
        L.invconv_fwd.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, vp]
        L.invconv_fwd_ex.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, vp, ci]
        L.invconv_bwd.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, vp, sz, vp]
        L.invconv_bwd_ex.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, vp, sz, vp, ci]
        L.invconv_bwd_workspace_bytes.argtypes = [ci, ci, ci, ci, ci]
        L.invconv_bwd_workspace_bytes.restype = sz
        L.invconv_logdet.argtypes = [vp, ci, ci, ci, ci, vp, vp]
        L.invconv_probe_step_sync.argtypes = [ci, ci, ci, vp]
        L.invconv_probe_step_sync.restype = ci
        L.invconv_chain_workspace_bytes.argtypes = [ci, ci, ci, ci, ci, ci]
        L.invconv_chain_workspace_bytes.restype = sz
        L.invconv_chain_fwd.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, ci, vp, sz, vp]
        L.invconv_chain_fwd.restype = ci
        L.invconv_chain_bwd.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, vp, sz, vp]
        L.invconv_chain_bwd.restype = ci
        L.invconv_chain_logdet.argtypes = [vp, ci, ci, ci, ci, ci, vp, vp]
        L.invconv_chain_logdet.restype = ci
        L.invconv_conv_fwd.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, vp]
        L.invconv_conv_fwd.restype = ci
        L.invconv_conv_bwd.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, vp, ctypes.c_size_t, vp]
        L.invconv_conv_bwd.restype = ci
        L.invconv_fwd_logdet.argtypes = [vp, vp, vp, vp, ci, ci, ci, ci, ci, vp]
        L.invconv_fwd_logdet.restype = ci
        L.invconv_fwd_ws.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, vp, sz, vp]
        L.invconv_fwd_ws.restype = ci
        L.invconv_fwd_workspace_bytes.argtypes = [ci, ci, ci, ci, ci]
        L.invconv_fwd_workspace_bytes.restype = sz
        L.invconv_workspace_error.argtypes = [vp, vp, ctypes.POINTER(ci)]
        L.invconv_workspace_error.restype = ci
        L.invconv_set_wait_budget.argtypes = [ci]
        L.invconv_set_wait_budget.restype = None
        L.invconv_bwd_static.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, vp]
        L.invconv_bwd_static.restype = ci
        L.invconv_flowstep_fwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, vp, sz, vp]
        L.invconv_flowstep_fwd.restype = ci
        L.invconv_flowstep_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_float,
                                           ci, ci, ci, ci, ci, vp, sz, vp]
        L.invconv_flowstep_bwd.restype = ci
        L.invconv_flowstep_fwd_ex.argtypes = L.invconv_flowstep_fwd.argtypes + [ci]
        L.invconv_flowstep_fwd_ex.restype = ci
        L.invconv_flowstep_bwd_ex.argtypes = L.invconv_flowstep_bwd.argtypes + [ci]
        L.invconv_flowstep_bwd_ex.restype = ci
        L.invconv_flowstep_workspace_bytes.argtypes = [ci, ci, ci, ci, ci]
        L.invconv_flowstep_workspace_bytes.restype = sz
        L.invconv_fwd_bf16.argtypes = [vp, vp, vp, ci, ci, ci, ci, ci, vp, sz, vp]
        L.invconv_fwd_bf16.restype = ci
        L.invconv_bwd_bf16.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, vp, sz, vp]
        L.invconv_bwd_bf16.restype = ci
        L.invconv_bf16_workspace_bytes.argtypes = [ci, ci, ci, ci, ci]
        L.invconv_bf16_workspace_bytes.restype = sz
        L.invconv_status_string.argtypes = [ci]
        L.invconv_status_string.restype = ctypes.c_char_p
        L.invconv_version.restype = ci
        for name in ("invconv_fwd", "invconv_fwd_ex", "invconv_bwd", "invconv_bwd_ex", "invconv_logdet"):
            getattr(L, name).restype = ci
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().invconv_status_string(status).decode()


def version() -> int:
    return int(lib().invconv_version())


def _check(t: torch.Tensor, name: str, shape=None) -> torch.Tensor:
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()):
        raise TypeError(f"{name} must be a contiguous float32 CUDA tensor")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} has shape {tuple(t.shape)}, expected {tuple(shape)}")
    return t


def _dims(act: torch.Tensor, w: torch.Tensor):
    if act.dim() != 4 or w.dim() != 4:
        raise ValueError("activations must be [B,C,H,W] and kernels [C,C,k,k]")
    B, C, H, W = act.shape
    if w.shape[0] != C or w.shape[1] != C or w.shape[2] != w.shape[3]:
        raise ValueError(f"kernel shape {tuple(w.shape)} does not match C={C}")
    return B, C, H, W, w.shape[2]


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def bwd_workspace_bytes(B: int, C: int, H: int, W: int, k: int) -> int:
    return int(lib().invconv_bwd_workspace_bytes(B, C, H, W, k))


def fwd_workspace_bytes(B: int, C: int, H: int, W: int, k: int) -> int:
    return int(lib().invconv_fwd_workspace_bytes(B, C, H, W, k))


def new_workspace(nbytes: int, device="cuda") -> torch.Tensor:
    """Device scratch of at least `nbytes` bytes with a zeroed header (the error word starts clear)."""
    ws = torch.empty(max(int(nbytes), WS_HEADER_BYTES), dtype=torch.uint8, device=device)
    ws[:WS_HEADER_BYTES].zero_()
    return ws


def workspace_error(workspace: torch.Tensor) -> int:
    """The workspace's error word (waits for the current stream): non-zero after a bounded wait ran out."""
    word = ctypes.c_int(-1)
    st = lib().invconv_workspace_error(workspace.data_ptr(), _stream(), ctypes.byref(word))
    if st != OK:
        raise InvconvError(st, "invconv_workspace_error")
    return int(word.value)


def set_wait_budget(polls: int) -> None:
    """Test hook: polls a bounded wait makes before it gives up (0 = built-in budgets)."""
    lib().invconv_set_wait_budget(int(polls))


def invconv_fwd(y: torch.Tensor, w: torch.Tensor, out: torch.Tensor | None = None,
                variant: int = VARIANT_AUTO, workspace: torch.Tensor | None = None) -> torch.Tensor:
    """x with conv_w(x) = y (inverse of the masked causal convolution).  With `workspace` the call goes
    through invconv_fwd_ws (scratch from the caller), otherwise through invconv_fwd."""
    _check(y, "y"), _check(w, "w")
    B, C, H, W, k = _dims(y, w)
    x = torch.empty_like(y) if out is None else _check(out, "out", y.shape)
    if workspace is not None:
        if variant != VARIANT_AUTO:
            raise ValueError("a workspace goes with the automatic kernel choice only")
        st = lib().invconv_fwd_ws(y.data_ptr(), w.data_ptr(), x.data_ptr(), B, C, H, W, k,
                                  workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream())
    else:
        st = lib().invconv_fwd_ex(y.data_ptr(), w.data_ptr(), x.data_ptr(), B, C, H, W, k, _stream(), variant)
    if st != OK:
        raise InvconvError(st, "invconv_fwd")
    return x


def invconv_fwd_logdet(y: torch.Tensor, w: torch.Tensor, out: tuple[torch.Tensor, torch.Tensor] | None = None):
    """(x, log|det dx/dy| of one image): forward pass and log-determinant in one call."""
    _check(y, "y"), _check(w, "w")
    B, C, H, W, k = _dims(y, w)
    if out is None:
        x, ld = torch.empty_like(y), torch.empty(1, dtype=torch.float32, device=y.device)
    else:
        x, ld = _check(out[0], "out[0]", y.shape), _check(out[1], "out[1]", (1,))
    st = lib().invconv_fwd_logdet(y.data_ptr(), w.data_ptr(), x.data_ptr(), ld.data_ptr(), B, C, H, W, k, _stream())
    if st != OK:
        raise InvconvError(st, "invconv_fwd_logdet")
    return x, ld


def invconv_bwd_static(x: torch.Tensor, w: torch.Tensor, dLdx: torch.Tensor,
                       out: tuple[torch.Tensor, torch.Tensor]):
    """invconv_bwd on the library's own scratch: allocates nothing (outputs must be passed in)."""
    _check(x, "x"), _check(w, "w"), _check(dLdx, "dLdx", x.shape)
    B, C, H, W, k = _dims(x, w)
    dLdy, dLdw = _check(out[0], "out[0]", x.shape), _check(out[1], "out[1]", w.shape)
    st = lib().invconv_bwd_static(x.data_ptr(), w.data_ptr(), dLdx.data_ptr(), dLdy.data_ptr(), dLdw.data_ptr(),
                                  B, C, H, W, k, _stream())
    if st != OK:
        raise InvconvError(st, "invconv_bwd_static")
    return dLdy, dLdw


def invconv_bwd(x: torch.Tensor, w: torch.Tensor, dLdx: torch.Tensor,
                out: tuple[torch.Tensor, torch.Tensor] | None = None,
                workspace: torch.Tensor | None = None, variant: int = VARIANT_AUTO):
    """(dL/dy, dL/dw) from the forward output x, the kernel and dL/dx."""
    _check(x, "x"), _check(w, "w"), _check(dLdx, "dLdx", x.shape)
    B, C, H, W, k = _dims(x, w)
    if out is None:
        dLdy, dLdw = torch.empty_like(x), torch.empty_like(w)
    else:
        dLdy, dLdw = _check(out[0], "out[0]", x.shape), _check(out[1], "out[1]", w.shape)
    need = bwd_workspace_bytes(B, C, H, W, k)
    if workspace is None:
        workspace = new_workspace(need, x.device)
    ws_bytes = workspace.numel() * workspace.element_size()
    st = lib().invconv_bwd_ex(x.data_ptr(), w.data_ptr(), dLdx.data_ptr(), dLdy.data_ptr(), dLdw.data_ptr(),
                              B, C, H, W, k, workspace.data_ptr(), ws_bytes, _stream(), variant)
    if st != OK:
        raise InvconvError(st, "invconv_bwd")
    return dLdy, dLdw


def invconv_logdet(w: torch.Tensor, H: int, W: int, out: torch.Tensor | None = None) -> torch.Tensor:
    """log|det dx/dy| of the inverse convolution for one H x W image (a 1-element tensor)."""
    _check(w, "w")
    if w.dim() != 4 or w.shape[0] != w.shape[1] or w.shape[2] != w.shape[3]:
        raise ValueError("kernel must be [C,C,k,k]")
    res = torch.empty(1, dtype=torch.float32, device=w.device) if out is None else _check(out, "out", (1,))
    st = lib().invconv_logdet(w.data_ptr(), w.shape[0], H, W, w.shape[2], res.data_ptr(), _stream())
    if st != OK:
        raise InvconvError(st, "invconv_logdet")
    return res


def _ptr_array(tensors):
    return (ctypes.c_void_p * len(tensors))(*[t.data_ptr() for t in tensors])


def chain_workspace_bytes(L: int, B: int, C: int, H: int, W: int, k: int) -> int:
    return int(lib().invconv_chain_workspace_bytes(L, B, C, H, W, k))


def invconv_chain_fwd(y: torch.Tensor, ws: list, out: list | None = None, workspace: torch.Tensor | None = None):
    """x[0] = invconv(y; ws[0]), x[l] = invconv(x[l-1]; ws[l]); returns the list of all x[l]."""
    _check(y, "y")
    for i, w in enumerate(ws):
        _check(w, f"ws[{i}]", ws[0].shape)
    B, C, H, W, k = _dims(y, ws[0])
    L = len(ws)
    xs = [torch.empty_like(y) for _ in range(L)] if out is None else [_check(t, "out", y.shape) for t in out]
    need = chain_workspace_bytes(L, B, C, H, W, k)
    if workspace is None:
        workspace = new_workspace(need, y.device)
    st = lib().invconv_chain_fwd(y.data_ptr(), _ptr_array(ws), _ptr_array(xs), L, B, C, H, W, k,
                                 workspace.data_ptr(), workspace.numel(), _stream())
    if st != OK:
        raise InvconvError(st, "invconv_chain_fwd")
    return xs


def invconv_chain_bwd(xs: list, ws: list, dLdx_last: torch.Tensor, workspace: torch.Tensor | None = None):
    """(dL/dy of layer 0, [dL/dw of every layer]) for the stack evaluated by invconv_chain_fwd."""
    _check(dLdx_last, "dLdx_last")
    for i, (x, w) in enumerate(zip(xs, ws)):
        _check(x, f"xs[{i}]", dLdx_last.shape), _check(w, f"ws[{i}]", ws[0].shape)
    B, C, H, W, k = _dims(dLdx_last, ws[0])
    L = len(ws)
    dy = torch.empty_like(dLdx_last)
    dws = [torch.empty_like(w) for w in ws]
    need = chain_workspace_bytes(L, B, C, H, W, k)
    if workspace is None:
        workspace = new_workspace(need, dy.device)
    st = lib().invconv_chain_bwd(_ptr_array(xs), _ptr_array(ws), dLdx_last.data_ptr(), dy.data_ptr(),
                                 _ptr_array(dws), L, B, C, H, W, k, workspace.data_ptr(), workspace.numel(),
                                 _stream())
    if st != OK:
        raise InvconvError(st, "invconv_chain_bwd")
    return dy, dws


def invconv_chain_logdet(ws: list, H: int, W: int) -> torch.Tensor:
    """log|det dx/dy| of every layer of a stack (tensor of len(ws) floats)."""
    for i, w in enumerate(ws):
        _check(w, f"ws[{i}]", ws[0].shape)
    res = torch.empty(len(ws), dtype=torch.float32, device=ws[0].device)
    st = lib().invconv_chain_logdet(_ptr_array(ws), len(ws), ws[0].shape[0], H, W, ws[0].shape[2],
                                    res.data_ptr(), _stream())
    if st != OK:
        raise InvconvError(st, "invconv_chain_logdet")
    return res


def invconv_conv_fwd(x: torch.Tensor, w: torch.Tensor, out: torch.Tensor | None = None) -> torch.Tensor:
    """y = conv_w(x): the masked causal convolution (the inverse of invconv_fwd)."""
    _check(x, "x"), _check(w, "w")
    B, C, H, W, k = _dims(x, w)
    y = torch.empty_like(x) if out is None else _check(out, "out", x.shape)
    st = lib().invconv_conv_fwd(x.data_ptr(), w.data_ptr(), y.data_ptr(), B, C, H, W, k, _stream())
    if st != OK:
        raise InvconvError(st, "invconv_conv_fwd")
    return y


def invconv_conv_bwd(x: torch.Tensor, w: torch.Tensor, dLdy: torch.Tensor,
                     out: tuple[torch.Tensor, torch.Tensor] | None = None,
                     workspace: torch.Tensor | None = None):
    """(dL/dx, dL/dw) of y = conv_w(x) given dL/dy."""
    _check(x, "x"), _check(w, "w"), _check(dLdy, "dLdy", x.shape)
    B, C, H, W, k = _dims(x, w)
    if out is None:
        dLdx, dLdw = torch.empty_like(x), torch.empty_like(w)
    else:
        dLdx, dLdw = _check(out[0], "out[0]", x.shape), _check(out[1], "out[1]", w.shape)
    need = bwd_workspace_bytes(B, C, H, W, k)
    if workspace is None:
        workspace = new_workspace(need, x.device)
    ws_bytes = workspace.numel() * workspace.element_size()
    st = lib().invconv_conv_bwd(x.data_ptr(), w.data_ptr(), dLdy.data_ptr(), dLdx.data_ptr(), dLdw.data_ptr(),
                                B, C, H, W, k, workspace.data_ptr(), ws_bytes, _stream())
    if st != OK:
        raise InvconvError(st, "invconv_conv_bwd")
    return dLdx, dLdw


def flowstep_workspace_bytes(B: int, C: int, H: int, W: int, k: int) -> int:
    return int(lib().invconv_flowstep_workspace_bytes(B, C, H, W, k))


def _flow_params(w, s, b, Q):
    C = w.shape[0]
    _check(s, "s", (C,)), _check(b, "b", (C,)), _check(Q, "Q", (C, C))


def invconv_flowstep_fwd(y: torch.Tensor, w: torch.Tensor, s: torch.Tensor, b: torch.Tensor, Q: torch.Tensor,
                         out: torch.Tensor | None = None, workspace: torch.Tensor | None = None,
                         form: int = FLOW_AUTO):
    """(z, logdet) of one flow step: z = Q (s * invconv_w(y) + b); logdet = log|det dz/dy| of one image."""
    _check(y, "y"), _check(w, "w")
    B, C, H, W, k = _dims(y, w)
    _flow_params(w, s, b, Q)
    z = torch.empty_like(y) if out is None else _check(out, "out", y.shape)
    ld = torch.empty(1, dtype=torch.float32, device=y.device)
    if workspace is None:
        workspace = new_workspace(flowstep_workspace_bytes(B, C, H, W, k), y.device)
    st = lib().invconv_flowstep_fwd_ex(y.data_ptr(), w.data_ptr(), s.data_ptr(), b.data_ptr(), Q.data_ptr(),
                                       z.data_ptr(), ld.data_ptr(), B, C, H, W, k, workspace.data_ptr(),
                                       workspace.numel(), _stream(), form)
    if st != OK:
        raise InvconvError(st, "invconv_flowstep_fwd")
    return z, ld


def invconv_flowstep_bwd(z: torch.Tensor, w: torch.Tensor, s: torch.Tensor, b: torch.Tensor, Q: torch.Tensor,
                         dLdz: torch.Tensor, logdet_weight: float = 0.0, workspace: torch.Tensor | None = None,
                         form: int = FLOW_AUTO, out: dict | None = None):
    """dict(dy, dw, ds, db, dQ) of one flow step from its output z and dL/dz."""
    _check(z, "z"), _check(w, "w"), _check(dLdz, "dLdz", z.shape)
    B, C, H, W, k = _dims(z, w)
    _flow_params(w, s, b, Q)
    if out is None:
        dy, dw = torch.empty_like(z), torch.empty_like(w)
        ds, db, dQ = torch.empty_like(s), torch.empty_like(b), torch.empty_like(Q)
    else:
        dy, dw, ds, db, dQ = (out[n] for n in ("dy", "dw", "ds", "db", "dQ"))
    if workspace is None:
        workspace = new_workspace(flowstep_workspace_bytes(B, C, H, W, k), z.device)
    st = lib().invconv_flowstep_bwd_ex(z.data_ptr(), w.data_ptr(), s.data_ptr(), b.data_ptr(), Q.data_ptr(),
                                       dLdz.data_ptr(), dy.data_ptr(), dw.data_ptr(), ds.data_ptr(), db.data_ptr(),
                                       dQ.data_ptr(), float(logdet_weight), B, C, H, W, k, workspace.data_ptr(),
                                       workspace.numel(), _stream(), form)
    if st != OK:
        raise InvconvError(st, "invconv_flowstep_bwd")
    return dict(dy=dy, dw=dw, ds=ds, db=db, dQ=dQ)


def _check16(t: torch.Tensor, name: str, shape=None) -> torch.Tensor:
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.bfloat16 and t.is_contiguous()):
        raise TypeError(f"{name} must be a contiguous bfloat16 CUDA tensor")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} has shape {tuple(t.shape)}, expected {tuple(shape)}")
    return t


def bf16_workspace_bytes(B: int, C: int, H: int, W: int, k: int) -> int:
    return int(lib().invconv_bf16_workspace_bytes(B, C, H, W, k))


def invconv_fwd_bf16(y: torch.Tensor, w: torch.Tensor, out: torch.Tensor | None = None,
                     workspace: torch.Tensor | None = None) -> torch.Tensor:
    """invconv_fwd with bf16 activations in memory (fp32 kernel, fp32 arithmetic)."""
    _check16(y, "y"), _check(w, "w")
    B, C, H, W, k = _dims(y, w)
    x = torch.empty_like(y) if out is None else _check16(out, "out", y.shape)
    if workspace is None:
        workspace = new_workspace(bf16_workspace_bytes(B, C, H, W, k), y.device)
    st = lib().invconv_fwd_bf16(y.data_ptr(), w.data_ptr(), x.data_ptr(), B, C, H, W, k, workspace.data_ptr(),
                                workspace.numel(), _stream())
    if st != OK:
        raise InvconvError(st, "invconv_fwd_bf16")
    return x


def invconv_bwd_bf16(x: torch.Tensor, w: torch.Tensor, dLdx: torch.Tensor, workspace: torch.Tensor | None = None,
                     out: tuple[torch.Tensor, torch.Tensor] | None = None):
    """(dL/dy as bf16, dL/dw as fp32) with bf16 activations in memory."""
    _check16(x, "x"), _check(w, "w"), _check16(dLdx, "dLdx", x.shape)
    B, C, H, W, k = _dims(x, w)
    if out is None:
        dLdy, dLdw = torch.empty_like(x), torch.empty_like(w)
    else:
        dLdy, dLdw = _check16(out[0], "out[0]", x.shape), _check(out[1], "out[1]", w.shape)
    if workspace is None:
        workspace = new_workspace(bf16_workspace_bytes(B, C, H, W, k), x.device)
    st = lib().invconv_bwd_bf16(x.data_ptr(), w.data_ptr(), dLdx.data_ptr(), dLdy.data_ptr(), dLdw.data_ptr(),
                                B, C, H, W, k, workspace.data_ptr(), workspace.numel(), _stream())
    if st != OK:
        raise InvconvError(st, "invconv_bwd_bf16")
    return dLdy, dLdw
