"""Thin Python binding of libssmscan.so: argument marshalling only.

Every function has the name of the C entry point it calls (include/ssm.h).  Tensors are torch
tensors that live on the GPU; torch is used for device memory and for the current stream and for
nothing else -- all arithmetic of the layer runs in the HIP kernels of the library.  There is no
CPU fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libssmscan.so")

SSM_OK = 0
SSM_ERR_INVALID_ARG = 1
SSM_ERR_WORKSPACE = 2
SSM_ERR_UNSUPPORTED = 3
SSM_ERR_HIP = 4
SSM_ERR_SCAN_TIMEOUT = 5
SSM_ERR_SCRATCH_LIMIT = 6
SSM_NOALLOC_SCRATCH_BYTES = 8 << 20
SSM_FWD_STAGES = 4
SSM_BWD_STAGES = 6
FWD_STAGE_NAMES = ("discretize_pack", "project_in", "scan", "project_out")
BWD_STAGE_NAMES = ("discretize_pack_dD", "gx", "reverse_scan", "du_dBbar_dC_partials", "sum_du_halves",
                   "param_epilogue")

EXPORTS = ("ssm_strerror", "ssm_version", "ssm_workspace_bytes", "ssm_discretize", "ssm_scan_fwd",
           "ssm_scan_bwd", "ssm_scan_states", "ssm_scan_states_reverse", "ssm_scan_fwd_profiled",
           "ssm_scan_bwd_profiled", "ssm_workspace_status", "ssm_step_plan_bytes", "ssm_step_prepare", "ssm_step",
           "ssm_step_bwd", "ssm_lambda_return", "ssm_lambda_return_bwd", "ssm_half_glu_workspace_bytes", "ssm_half_glu_fwd",
           "ssm_half_glu_bwd", "ssm_block_workspace_bytes", "ssm_block_fwd", "ssm_block_bwd", "ssm_set_spin_limit",
           "ssm_scan_states_noalloc", "ssm_scan_states_noalloc_status", "ssm_plan_describe")

_lib = None
_vp, _i64, _sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_size_t


class SsmError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__("%s: %s (status %d)" % (where, strerror(code), code))


def lib():
    """The loaded C-ABI library.  Raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libssmscan.so is not built: run `python -c \"import __graft_entry__ as g; "
                              "g.build()\"` or `python paper_2502_20168_amd/build.py` first")
        # torch first: it brings its own copy of the HIP runtime, and the library must bind to that one.  Loaded
        # before torch, the library would pull in the system's copy, torch a second one afterwards, and
        # every launch on torch's memory and streams would fail (status SSM_ERR_HIP)
        _torch()
        L = ctypes.CDLL(LIB_PATH)
        L.ssm_strerror.restype = ctypes.c_char_p
        L.ssm_strerror.argtypes = [ctypes.c_int]
        L.ssm_version.restype = ctypes.c_int
        L.ssm_workspace_bytes.restype = _sz
        L.ssm_workspace_bytes.argtypes = [_i64, _i64, _i64, _i64, ctypes.c_int]
        L.ssm_discretize.restype = ctypes.c_int
        L.ssm_discretize.argtypes = [_vp, _vp, _vp, _i64, _i64, _vp, _vp, _vp]
        fwd = [_vp] * 8 + [_i64] * 4 + [_vp] * 3 + [_vp, _sz, _vp]
        bwd = [_vp] * 8 + [_i64] * 4 + [_vp] * 2 + [_vp] * 7 + [_vp, _sz, _vp]
        L.ssm_scan_fwd.restype = ctypes.c_int
        L.ssm_scan_fwd.argtypes = fwd
        L.ssm_scan_bwd.restype = ctypes.c_int
        L.ssm_scan_bwd.argtypes = bwd
        L.ssm_scan_fwd_profiled.restype = ctypes.c_int
        L.ssm_scan_fwd_profiled.argtypes = fwd + [_vp]
        L.ssm_scan_bwd_profiled.restype = ctypes.c_int
        L.ssm_scan_bwd_profiled.argtypes = bwd + [_vp]
        L.ssm_scan_states.restype = ctypes.c_int
        L.ssm_scan_states.argtypes = [_vp, _vp, _vp, _vp, _i64, _i64, _i64, _vp, _vp, _sz, _vp]
        L.ssm_scan_states_reverse.restype = ctypes.c_int
        L.ssm_scan_states_reverse.argtypes = [_vp] * 5 + [_i64] * 3 + [_vp, _vp, _vp, _sz, _vp]
        L.ssm_workspace_status.restype = ctypes.c_int
        L.ssm_workspace_status.argtypes = [_vp, _vp]
        L.ssm_step_plan_bytes.restype = _sz
        L.ssm_step_plan_bytes.argtypes = [_i64, _i64]
        L.ssm_step_prepare.restype = ctypes.c_int
        L.ssm_step_prepare.argtypes = [_vp, _vp, _vp, _vp, _i64, _i64, _vp, _sz, _vp]
        L.ssm_step.restype = ctypes.c_int
        L.ssm_step.argtypes = [_vp, _sz, _vp, _vp, _vp, _vp, _i64, _i64, _i64, _vp, _vp, _vp]
        L.ssm_step_bwd.restype = ctypes.c_int
        L.ssm_step_bwd.argtypes = [_vp, _sz, _vp, _vp, _vp, _vp, _i64, _i64, _i64, _vp, _vp, _vp, _vp]
        _f = ctypes.c_float
        L.ssm_lambda_return.restype = ctypes.c_int
        L.ssm_lambda_return.argtypes = [_vp, _vp, _vp, _f, _f, _i64, _i64, _vp, _vp]
        L.ssm_lambda_return_bwd.restype = ctypes.c_int
        L.ssm_lambda_return_bwd.argtypes = [_vp, _vp, _vp, _vp, _f, _f, _i64, _i64, _vp, _vp, _vp, _vp]
        L.ssm_half_glu_workspace_bytes.restype = _sz
        L.ssm_half_glu_workspace_bytes.argtypes = [_i64, _i64, ctypes.c_int]
        L.ssm_half_glu_fwd.restype = ctypes.c_int
        L.ssm_half_glu_fwd.argtypes = [_vp, _vp, _i64, _i64, _vp, _vp, _vp, _sz, _vp]
        L.ssm_half_glu_bwd.restype = ctypes.c_int
        L.ssm_half_glu_bwd.argtypes = [_vp, _vp, _vp, _vp, _i64, _i64, _vp, _vp, _vp, _sz, _vp]
        L.ssm_scan_states_noalloc.restype = ctypes.c_int
        L.ssm_scan_states_noalloc.argtypes = [_vp, _vp, _vp, _vp, _i64, _i64, _i64, _vp, _vp]
        L.ssm_scan_states_noalloc_status.restype = ctypes.c_int
        L.ssm_scan_states_noalloc_status.argtypes = [_vp]
        L.ssm_set_spin_limit.restype = ctypes.c_uint32
        L.ssm_set_spin_limit.argtypes = [ctypes.c_uint32]
        L.ssm_block_workspace_bytes.restype = _sz
        L.ssm_block_workspace_bytes.argtypes = [_i64, _i64, _i64, _i64, ctypes.c_int]
        L.ssm_block_fwd.restype = ctypes.c_int
        L.ssm_block_fwd.argtypes = [_vp] * 9 + [_i64] * 4 + [_vp] * 5 + [_vp, _sz, _vp]
        L.ssm_block_bwd.restype = ctypes.c_int
        L.ssm_block_bwd.argtypes = [_vp] * 9 + [_i64] * 4 + [_vp] * 4 + [_vp] * 8 + [_vp, _sz, _vp]
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().ssm_strerror(int(code)).decode()


def ssm_version() -> int:
    return int(lib().ssm_version())


def ssm_workspace_bytes(Bt: int, L: int, H: int, P: int, want_bwd: bool) -> int:
    return int(lib().ssm_workspace_bytes(Bt, L, H, P, 1 if want_bwd else 0))


# ------------------------------------------------------------------ torch marshalling
def _torch():
    import torch
    return torch


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    torch = _torch()
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _chk(t, dtype, shape, name):
    torch = _torch()
    if t is None:
        return
    if not t.is_cuda or t.dtype != dtype or tuple(t.shape) != tuple(shape) or not t.is_contiguous():
        raise ValueError("%s must be a contiguous cuda tensor of dtype %s and shape %s, got %s %s on %s"
                         % (name, dtype, tuple(shape), t.dtype, tuple(t.shape), t.device))


def alloc_workspace(Bt, L, H, P, want_bwd, device="cuda"):
    torch = _torch()
    n = ssm_workspace_bytes(Bt, L, H, P, want_bwd)
    if n == 0:
        raise SsmError(SSM_ERR_UNSUPPORTED, "ssm_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def _own_workspace(ws, stream):
    """A workspace this module allocated for one call is dropped when the call returns, while its
    kernels are still queued: tell the caching allocator which stream they run on, so that the block is
    not handed out again before they finish (the allocation itself happened on the current stream)."""
    if stream is not None:
        ws.record_stream(stream)
    return ws


def _check_inputs(Lambda, B, C, D, log_delta, u, is_first, x0):
    torch = _torch()
    if u.dim() != 3 or Lambda.dim() != 1:
        raise ValueError("u must be [Bt,L,H] and Lambda [P]")
    Bt, L, H = u.shape
    P = Lambda.shape[0]
    _chk(Lambda, torch.complex64, (P,), "Lambda")
    _chk(B, torch.complex64, (P, H), "B")
    _chk(C, torch.complex64, (H, P), "C")
    _chk(D, torch.float32, (H,), "D")
    _chk(log_delta, torch.float32, (P,), "log_delta")
    _chk(u, torch.float32, (Bt, L, H), "u")
    _chk(is_first, torch.uint8, (Bt, L), "is_first")
    _chk(x0, torch.complex64, (Bt, P), "x0")
    return Bt, L, H, P


def ssm_discretize(Lambda, B, log_delta, stream=None):
    """Returns (A_bar [P], B_bar [P,H]); B may be None (then B_bar is None)."""
    torch = _torch()
    P = Lambda.shape[0]
    _chk(Lambda, torch.complex64, (P,), "Lambda")
    _chk(log_delta, torch.float32, (P,), "log_delta")
    H = 1 if B is None else B.shape[1]
    _chk(B, torch.complex64, (P, H), "B")
    A_bar = torch.empty_like(Lambda)
    B_bar = None if B is None else torch.empty_like(B)
    rc = lib().ssm_discretize(_ptr(Lambda), _ptr(B), _ptr(log_delta), P, H, _ptr(A_bar), _ptr(B_bar),
                              _stream(stream))
    if rc != SSM_OK:
        raise SsmError(rc, "ssm_discretize")
    return A_bar, B_bar


def ssm_scan_fwd(Lambda, B, C, D, log_delta, u, is_first=None, x0=None, *, want_x=True,
                 want_x_last=True, workspace=None, stream=None, out=None,
                 profile=False) -> Dict[str, object]:
    """Forward pass.  Returns dict(y, x or None, x_last or None[, stage_ms])."""
    torch = _torch()
    Bt, L, H, P = _check_inputs(Lambda, B, C, D, log_delta, u, is_first, x0)
    out = out or {}
    y = out.get("y") if out.get("y") is not None else torch.empty_like(u)
    x = out.get("x") if out.get("x") is not None else (
        torch.empty((Bt, L, P), dtype=torch.complex64, device=u.device) if want_x else None)
    x_last = out.get("x_last") if out.get("x_last") is not None else (
        torch.empty((Bt, P), dtype=torch.complex64, device=u.device) if want_x_last else None)
    ws = workspace if workspace is not None else _own_workspace(alloc_workspace(Bt, L, H, P, False, u.device), stream)
    args = [_ptr(Lambda), _ptr(B), _ptr(C), _ptr(D), _ptr(log_delta), _ptr(u), _ptr(is_first), _ptr(x0),
            Bt, L, H, P, _ptr(y), _ptr(x), _ptr(x_last), _ptr(ws), ws.numel(), _stream(stream)]
    res = {"y": y, "x": x, "x_last": x_last}
    if profile:
        ms = (ctypes.c_float * SSM_FWD_STAGES)()
        rc = lib().ssm_scan_fwd_profiled(*args, ctypes.cast(ms, ctypes.c_void_p))
        res["stage_ms"] = list(ms)
    else:
        rc = lib().ssm_scan_fwd(*args)
    if rc != SSM_OK:
        raise SsmError(rc, "ssm_scan_fwd")
    return res


def ssm_scan_bwd(Lambda, B, C, D, log_delta, u, is_first, x0, x, dy, *, want_dx0=True,
                 workspace=None, stream=None, out=None, profile=False) -> Dict[str, object]:
    """Gradient pass.  Returns dict(du, dLambda, dB, dC, dD, dlog_delta, dx0 or None[, stage_ms])."""
    torch = _torch()
    Bt, L, H, P = _check_inputs(Lambda, B, C, D, log_delta, u, is_first, x0)
    _chk(x, torch.complex64, (Bt, L, P), "x")
    _chk(dy, torch.float32, (Bt, L, H), "dy")
    out = out or {}

    def get(name, like=None, shape=None, dtype=None):
        if out.get(name) is not None:
            return out[name]
        return torch.empty_like(like) if like is not None else torch.empty(shape, dtype=dtype, device=u.device)

    res = {
        "du": get("du", like=u), "dLambda": get("dLambda", like=Lambda), "dB": get("dB", like=B),
        "dC": get("dC", like=C), "dD": get("dD", like=D), "dlog_delta": get("dlog_delta", like=log_delta),
        "dx0": get("dx0", shape=(Bt, P), dtype=torch.complex64) if want_dx0 else None,
    }
    ws = workspace if workspace is not None else _own_workspace(alloc_workspace(Bt, L, H, P, True, u.device), stream)
    args = [_ptr(Lambda), _ptr(B), _ptr(C), _ptr(D), _ptr(log_delta), _ptr(u), _ptr(is_first), _ptr(x0),
            Bt, L, H, P, _ptr(x), _ptr(dy), _ptr(res["du"]), _ptr(res["dLambda"]), _ptr(res["dB"]),
            _ptr(res["dC"]), _ptr(res["dD"]), _ptr(res["dlog_delta"]), _ptr(res["dx0"]),
            _ptr(ws), ws.numel(), _stream(stream)]
    if profile:
        ms = (ctypes.c_float * SSM_BWD_STAGES)()
        rc = lib().ssm_scan_bwd_profiled(*args, ctypes.cast(ms, ctypes.c_void_p))
        res["stage_ms"] = list(ms)
    else:
        rc = lib().ssm_scan_bwd(*args)
    if rc != SSM_OK:
        raise SsmError(rc, "ssm_scan_bwd")
    return res


def ssm_scan_states(A_bar, v, is_first=None, x0=None, *, want_x_last=True, workspace=None, stream=None):
    """In-place resettable scan of v [Bt,L,P] (becomes x).  Returns (v, x_last or None)."""
    torch = _torch()
    Bt, L, P = v.shape
    _chk(A_bar, torch.complex64, (P,), "A_bar")
    _chk(v, torch.complex64, (Bt, L, P), "v")
    _chk(is_first, torch.uint8, (Bt, L), "is_first")
    _chk(x0, torch.complex64, (Bt, P), "x0")
    x_last = torch.empty((Bt, P), dtype=torch.complex64, device=v.device) if want_x_last else None
    ws = workspace if workspace is not None else _own_workspace(alloc_workspace(Bt, L, 1, P, False, v.device), stream)
    rc = lib().ssm_scan_states(_ptr(A_bar), _ptr(v), _ptr(is_first), _ptr(x0), Bt, L, P, _ptr(x_last),
                               _ptr(ws), ws.numel(), _stream(stream))
    if rc != SSM_OK:
        raise SsmError(rc, "ssm_scan_states")
    return v, x_last


def ssm_scan_states_noalloc(A_bar, v, is_first=None, x0=None, *, x_last=None, stream=None):
    """ssm_scan_states on the library's built-in scratch: no workspace, and nothing is allocated here
    either (x_last, when wanted, is the caller's tensor).  Returns v."""
    torch = _torch()
    Bt, L, P = v.shape
    _chk(A_bar, torch.complex64, (P,), "A_bar")
    _chk(v, torch.complex64, (Bt, L, P), "v")
    _chk(is_first, torch.uint8, (Bt, L), "is_first")
    _chk(x0, torch.complex64, (Bt, P), "x0")
    _chk(x_last, torch.complex64, (Bt, P), "x_last")
    rc = lib().ssm_scan_states_noalloc(_ptr(A_bar), _ptr(v), _ptr(is_first), _ptr(x0), Bt, L, P, _ptr(x_last),
                                       _stream(stream))
    if rc != SSM_OK:
        raise SsmError(rc, "ssm_scan_states_noalloc")
    return v


def ssm_scan_states_noalloc_status(stream=None) -> int:
    return int(lib().ssm_scan_states_noalloc_status(_stream(stream)))


def ssm_scan_states_reverse(A_bar, gx, x, is_first=None, x0=None, *, want_dx0=True, workspace=None,
                            stream=None):
    """In-place reverse scan of gx [Bt,L,P] (becomes chi).  Returns (gx, dA_bar, dx0 or None)."""
    torch = _torch()
    Bt, L, P = gx.shape
    _chk(A_bar, torch.complex64, (P,), "A_bar")
    _chk(gx, torch.complex64, (Bt, L, P), "gx")
    _chk(x, torch.complex64, (Bt, L, P), "x")
    _chk(is_first, torch.uint8, (Bt, L), "is_first")
    _chk(x0, torch.complex64, (Bt, P), "x0")
    dA = torch.empty_like(A_bar)
    dx0 = torch.empty((Bt, P), dtype=torch.complex64, device=gx.device) if want_dx0 else None
    ws = workspace if workspace is not None else _own_workspace(alloc_workspace(Bt, L, 1, P, True, gx.device), stream)
    rc = lib().ssm_scan_states_reverse(_ptr(A_bar), _ptr(gx), _ptr(x), _ptr(is_first), _ptr(x0), Bt, L, P,
                                       _ptr(dA), _ptr(dx0), _ptr(ws), ws.numel(), _stream(stream))
    if rc != SSM_OK:
        raise SsmError(rc, "ssm_scan_states_reverse")
    return gx, dA, dx0


def ssm_step_plan_bytes(H: int, P: int) -> int:
    return int(lib().ssm_step_plan_bytes(H, P))


def ssm_step_prepare(Lambda, B, C, log_delta, stream=None):
    """Discretise and pack the parameters once per roll-out.  Returns the plan (a cuda byte tensor)."""
    torch = _torch()
    P, H = B.shape
    _chk(Lambda, torch.complex64, (P,), "Lambda")
    _chk(B, torch.complex64, (P, H), "B")
    _chk(C, torch.complex64, (H, P), "C")
    _chk(log_delta, torch.float32, (P,), "log_delta")
    plan = torch.empty(ssm_step_plan_bytes(H, P), dtype=torch.uint8, device=B.device)
    rc = lib().ssm_step_prepare(_ptr(Lambda), _ptr(B), _ptr(C), _ptr(log_delta), H, P, _ptr(plan), plan.numel(),
                                _stream(stream))
    if rc != SSM_OK:
        raise SsmError(rc, "ssm_step_prepare")
    return plan


def ssm_step(plan, D, u, x_prev=None, is_first=None, *, P=None, x=None, y=None, stream=None):
    """One transition.  u [Bt,H], x_prev [Bt,P] or None, is_first [Bt] u8 or None.  Returns (x, y)."""
    torch = _torch()
    Bt, H = u.shape
    if P is None:
        P = x_prev.shape[1] if x_prev is not None else x.shape[1]
    _chk(D, torch.float32, (H,), "D")
    _chk(u, torch.float32, (Bt, H), "u")
    _chk(x_prev, torch.complex64, (Bt, P), "x_prev")
    _chk(is_first, torch.uint8, (Bt,), "is_first")
    x = x if x is not None else torch.empty((Bt, P), dtype=torch.complex64, device=u.device)
    y = y if y is not None else torch.empty_like(u)
    rc = lib().ssm_step(_ptr(plan), plan.numel(), _ptr(D), _ptr(u), _ptr(x_prev), _ptr(is_first), Bt, H, P,
                        _ptr(x), _ptr(y), _stream(stream))
    if rc != SSM_OK:
        raise SsmError(rc, "ssm_step")
    return x, y


def ssm_step_bwd(plan, D, dy, dx=None, is_first=None, *, P, want_dx_prev=True, stream=None):
    """Adjoint of one transition.  dy [Bt,H], dx [Bt,P] or None.  Returns (gx, du, dx_prev)."""
    torch = _torch()
    Bt, H = dy.shape
    _chk(D, torch.float32, (H,), "D")
    _chk(dy, torch.float32, (Bt, H), "dy")
    _chk(dx, torch.complex64, (Bt, P), "dx")
    _chk(is_first, torch.uint8, (Bt,), "is_first")
    gx = torch.empty((Bt, P), dtype=torch.complex64, device=dy.device)
    du = torch.empty_like(dy)
    dx_prev = torch.empty_like(gx) if want_dx_prev else None
    rc = lib().ssm_step_bwd(_ptr(plan), plan.numel(), _ptr(D), _ptr(dy), _ptr(dx), _ptr(is_first), Bt, H, P,
                            _ptr(gx), _ptr(du), _ptr(dx_prev), _stream(stream))
    if rc != SSM_OK:
        raise SsmError(rc, "ssm_step_bwd")
    return gx, du, dx_prev


def ssm_lambda_return(reward, cont, value, gamma: float, lam: float, *, ret=None, stream=None):
    """Time-major [T, N] float32 tensors.  Returns ret [T, N]."""
    torch = _torch()
    T, N = reward.shape
    for name, t in (("reward", reward), ("cont", cont), ("value", value), ("ret", ret)):
        _chk(t, torch.float32, (T, N), name)
    ret = ret if ret is not None else torch.empty_like(reward)
    rc = lib().ssm_lambda_return(_ptr(reward), _ptr(cont), _ptr(value), gamma, lam, T, N, _ptr(ret), _stream(stream))
    if rc != SSM_OK:
        raise SsmError(rc, "ssm_lambda_return")
    return ret


def ssm_lambda_return_bwd(cont, value, ret, dret, gamma: float, lam: float, *, stream=None):
    """Returns (dreward, dcont, dvalue), each [T, N]."""
    torch = _torch()
    T, N = cont.shape
    for name, t in (("cont", cont), ("value", value), ("ret", ret), ("dret", dret)):
        _chk(t, torch.float32, (T, N), name)
    dr, dc, dv = torch.empty_like(cont), torch.empty_like(cont), torch.empty_like(cont)
    rc = lib().ssm_lambda_return_bwd(_ptr(cont), _ptr(value), _ptr(ret), _ptr(dret), gamma, lam, T, N,
                                     _ptr(dr), _ptr(dc), _ptr(dv), _stream(stream))
    if rc != SSM_OK:
        raise SsmError(rc, "ssm_lambda_return_bwd")
    return dr, dc, dv


def ssm_set_spin_limit(polls: int) -> int:
    """Test hook: bound on the polls of a cross-workgroup wait.  Returns the previous bound."""
    return int(lib().ssm_set_spin_limit(int(polls)))


def ssm_half_glu_workspace_bytes(T: int, H: int, want_bwd: bool) -> int:
    return int(lib().ssm_half_glu_workspace_bytes(T, H, 1 if want_bwd else 0))


def _glu_workspace(T, H, want_bwd, device):
    torch = _torch()
    n = ssm_half_glu_workspace_bytes(T, H, want_bwd)
    if n == 0:
        raise SsmError(SSM_ERR_UNSUPPORTED, "ssm_half_glu_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def ssm_half_glu_fwd(u, W, *, want_gate=True, workspace=None, y=None, gate=None, stream=None):
    """u [T, H], W [H, H] float32.  Returns (y, gate); gate is None unless asked for."""
    torch = _torch()
    T, H = u.shape
    _chk(u, torch.float32, (T, H), "u")
    _chk(W, torch.float32, (H, H), "W")
    _chk(y, torch.float32, (T, H), "y")
    _chk(gate, torch.float32, (T, H), "gate")
    ws = workspace if workspace is not None else _own_workspace(_glu_workspace(T, H, False, u.device), stream)
    y = y if y is not None else torch.empty_like(u)
    if gate is None and want_gate:
        gate = torch.empty_like(u)
    rc = lib().ssm_half_glu_fwd(_ptr(u), _ptr(W), T, H, _ptr(y), _ptr(gate), _ptr(ws), ws.numel(), _stream(stream))
    if rc != SSM_OK:
        raise SsmError(rc, "ssm_half_glu_fwd")
    return y, gate


def ssm_half_glu_bwd(u, W, gate, dy, *, workspace=None, du=None, dW=None, stream=None):
    """Returns (du [T, H], dW [H, H])."""
    torch = _torch()
    T, H = u.shape
    for name, t in (("u", u), ("gate", gate), ("dy", dy), ("du", du)):
        _chk(t, torch.float32, (T, H), name)
    _chk(W, torch.float32, (H, H), "W")
    _chk(dW, torch.float32, (H, H), "dW")
    ws = workspace if workspace is not None else _own_workspace(_glu_workspace(T, H, True, u.device), stream)
    du = du if du is not None else torch.empty_like(u)
    dW = dW if dW is not None else torch.empty_like(W)
    rc = lib().ssm_half_glu_bwd(_ptr(u), _ptr(W), _ptr(gate), _ptr(dy), T, H, _ptr(du), _ptr(dW), _ptr(ws), ws.numel(),
                                _stream(stream))
    if rc != SSM_OK:
        raise SsmError(rc, "ssm_half_glu_bwd")
    return du, dW


def ssm_block_workspace_bytes(Bt: int, L: int, H: int, P: int, want_bwd: bool) -> int:
    return int(lib().ssm_block_workspace_bytes(Bt, L, H, P, 1 if want_bwd else 0))


def _block_workspace(Bt, L, H, P, want_bwd, device):
    torch = _torch()
    n = ssm_block_workspace_bytes(Bt, L, H, P, want_bwd)
    if n == 0:
        raise SsmError(SSM_ERR_UNSUPPORTED, "ssm_block_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def ssm_block_fwd(Lambda, B, C, D, log_delta, W, u, is_first=None, x0=None, *, want_gate=True, workspace=None,
                  stream=None):
    """SSM layer followed by the half-GLU gate.  Returns dict(y, out, gate, x, x_last)."""
    torch = _torch()
    Bt, L, H = u.shape
    P = Lambda.shape[0]
    _chk(Lambda, torch.complex64, (P,), "Lambda")
    _chk(B, torch.complex64, (P, H), "B")
    _chk(C, torch.complex64, (H, P), "C")
    _chk(D, torch.float32, (H,), "D")
    _chk(log_delta, torch.float32, (P,), "log_delta")
    _chk(W, torch.float32, (H, H), "W")
    _chk(u, torch.float32, (Bt, L, H), "u")
    _chk(is_first, torch.uint8, (Bt, L), "is_first")
    _chk(x0, torch.complex64, (Bt, P), "x0")
    ws = workspace if workspace is not None else _own_workspace(_block_workspace(Bt, L, H, P, False, u.device), stream)
    y, out = torch.empty_like(u), torch.empty_like(u)
    gate = torch.empty_like(u) if want_gate else None
    x = torch.empty((Bt, L, P), dtype=torch.complex64, device=u.device)
    x_last = torch.empty((Bt, P), dtype=torch.complex64, device=u.device)
    rc = lib().ssm_block_fwd(_ptr(Lambda), _ptr(B), _ptr(C), _ptr(D), _ptr(log_delta), _ptr(W), _ptr(u), _ptr(is_first),
                             _ptr(x0), Bt, L, H, P, _ptr(y), _ptr(out), _ptr(gate), _ptr(x), _ptr(x_last),
                             _ptr(ws), ws.numel(), _stream(stream))
    if rc != SSM_OK:
        raise SsmError(rc, "ssm_block_fwd")
    return {"y": y, "out": out, "gate": gate, "x": x, "x_last": x_last}


def ssm_block_bwd(Lambda, B, C, D, log_delta, W, u, is_first, x0, x, y, gate, dout, *, workspace=None, stream=None):
    """Gradient pass of ssm_block_fwd.  Returns dict(du, dLambda, dB, dC, dD, dlog_delta, dx0, dW)."""
    torch = _torch()
    Bt, L, H = u.shape
    P = Lambda.shape[0]
    for name, t in (("u", u), ("y", y), ("gate", gate), ("dout", dout)):
        _chk(t, torch.float32, (Bt, L, H), name)
    _chk(x, torch.complex64, (Bt, L, P), "x")
    _chk(W, torch.float32, (H, H), "W")
    ws = workspace if workspace is not None else _own_workspace(_block_workspace(Bt, L, H, P, True, u.device), stream)
    o = {"du": torch.empty_like(u), "dLambda": torch.empty_like(Lambda), "dB": torch.empty_like(B),
         "dC": torch.empty_like(C), "dD": torch.empty_like(D), "dlog_delta": torch.empty_like(log_delta),
         "dx0": torch.empty((Bt, P), dtype=torch.complex64, device=u.device), "dW": torch.empty_like(W)}
    rc = lib().ssm_block_bwd(_ptr(Lambda), _ptr(B), _ptr(C), _ptr(D), _ptr(log_delta), _ptr(W), _ptr(u), _ptr(is_first),
                             _ptr(x0), Bt, L, H, P, _ptr(x), _ptr(y), _ptr(gate), _ptr(dout),
                             _ptr(o["du"]), _ptr(o["dLambda"]), _ptr(o["dB"]), _ptr(o["dC"]), _ptr(o["dD"]),
                             _ptr(o["dlog_delta"]), _ptr(o["dx0"]), _ptr(o["dW"]), _ptr(ws), ws.numel(), _stream(stream))
    if rc != SSM_OK:
        raise SsmError(rc, "ssm_block_bwd")
    return o


SSM_PLAN_FIELDS = 12
PLAN_FIELD_NAMES = ("scans_in_projections", "planes", "slabs_dC", "slabs_dBbar", "products_per_gradient_launch",
                    "slabs_first", "dC_first", "dBbar_first", "du_as_two_k_halves", "tier_in", "tier_out", "scan_time_blocks")


def ssm_plan_describe(Bt: int, L: int, H: int, P: int) -> Dict[str, int]:
    """What ssm_scan_fwd / ssm_scan_bwd would launch for a shape (host logic only, needs no GPU)."""
    out = (ctypes.c_int32 * SSM_PLAN_FIELDS)()
    fn = lib().ssm_plan_describe
    fn.restype = ctypes.c_int
    fn.argtypes = [_i64, _i64, _i64, _i64, ctypes.POINTER(ctypes.c_int32)]
    rc = fn(Bt, L, H, P, out)
    if rc != SSM_OK:
        raise SsmError(rc, "ssm_plan_describe")
    return dict(zip(PLAN_FIELD_NAMES, [int(v) for v in out]))


def ssm_workspace_status(workspace, stream=None) -> int:
    return int(lib().ssm_workspace_status(_ptr(workspace), _stream(stream)))


# ------------------------------------------------------------------ convenience for tests/bench
def to_device(inp: Dict[str, Optional[object]], device="cuda") -> Dict[str, Optional[object]]:
    """numpy dict from the workload generator -> dict of cuda tensors (None stays None)."""
    torch = _torch()
    return {k: (None if v is None else torch.from_numpy(v).to(device)) for k, v in inp.items()}
