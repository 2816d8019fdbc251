"""ctypes front-end of the float64 CPU oracle (ssm_oracle.c) plus a finite-difference checker.

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
CPU-baseline leg.  Nothing here imports, links or calls the HIP library, and the HIP package
never imports this module.

All functions take numpy arrays; inputs are up-cast to float64 / complex128 (the callers pass
the fp32-rounded synthetic values so both sides see identical numbers).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ssm_oracle.c")
_LIB = os.path.join(_HERE, "libssm_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile ssm_oracle.c with gcc (plain -O2, OpenMP over sequences only)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fcx-limited-range", "-shared", "-fPIC",
                               _SRC, "-o", tmp, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.ssm_oracle_fwd.restype = ctypes.c_int
        _lib.ssm_oracle_bwd.restype = ctypes.c_int
        _lib.ssm_oracle_max_threads.restype = ctypes.c_int
    return _lib


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _c128(a):
    return np.ascontiguousarray(a, dtype=np.complex128)


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def max_threads() -> int:
    return int(_load().ssm_oracle_max_threads())


def discretize(Lambda, log_delta):
    """ZOH: returns (Abar [P], g [P]) with Bbar = g[:, None] * B."""
    lib = _load()
    Lambda, log_delta = _c128(Lambda), _f64(log_delta)
    P = Lambda.shape[0]
    Abar = np.empty(P, np.complex128)
    g = np.empty(P, np.complex128)
    lib.ssm_oracle_discretize(_ptr(Lambda), _ptr(log_delta), ctypes.c_long(P), _ptr(Abar), _ptr(g))
    return Abar, g


def scan(Abar, v, is_first=None, x0=None):
    """Resettable diagonal recurrence on projected inputs v [Bt,L,P]."""
    lib = _load()
    Abar, v = _c128(Abar), _c128(v)
    Bt, L, P = v.shape
    fl = None if is_first is None else np.ascontiguousarray(is_first, dtype=np.uint8)
    x0c = None if x0 is None else _c128(x0)
    x = np.empty_like(v)
    lib.ssm_oracle_scan(_ptr(Abar), _ptr(v), _ptr(fl), _ptr(x0c), ctypes.c_long(Bt),
                        ctypes.c_long(L), ctypes.c_long(P), _ptr(x))
    return x


def forward(Lambda, B, C, D, log_delta, u, is_first=None, x0=None, nthreads: int = 1):
    """Returns dict(y [Bt,L,H] f64, x [Bt,L,P] c128, x_last [Bt,P] c128)."""
    lib = _load()
    Lambda, B, C = _c128(Lambda), _c128(B), _c128(C)
    D, log_delta, u = _f64(D), _f64(log_delta), _f64(u)
    Bt, L, H = u.shape
    P = Lambda.shape[0]
    assert B.shape == (P, H) and C.shape == (H, P) and D.shape == (H,) and log_delta.shape == (P,)
    fl = None if is_first is None else np.ascontiguousarray(is_first, dtype=np.uint8)
    x0c = None if x0 is None else _c128(x0)
    if fl is not None:
        assert fl.shape == (Bt, L)
    if x0c is not None:
        assert x0c.shape == (Bt, P)
    y = np.empty((Bt, L, H), np.float64)
    x = np.empty((Bt, L, P), np.complex128)
    x_last = np.empty((Bt, P), np.complex128)
    rc = lib.ssm_oracle_fwd(_ptr(Lambda), _ptr(B), _ptr(C), _ptr(D), _ptr(log_delta), _ptr(u),
                            _ptr(fl), _ptr(x0c), ctypes.c_long(Bt), ctypes.c_long(L),
                            ctypes.c_long(H), ctypes.c_long(P), _ptr(y), _ptr(x), _ptr(x_last),
                            ctypes.c_int(nthreads))
    if rc != 0:
        raise MemoryError("ssm_oracle_fwd failed")
    return {"y": y, "x": x, "x_last": x_last}


def backward(Lambda, B, C, D, log_delta, u, is_first, x0, x, dy, nthreads: int = 1):
    """Gradients of l = sum(dy * y).  Returns dict(du, dLambda, dB, dC, dD, dlog_delta, dx0)."""
    lib = _load()
    Lambda, B, C = _c128(Lambda), _c128(B), _c128(C)
    D, log_delta, u, dy = _f64(D), _f64(log_delta), _f64(u), _f64(dy)
    x = _c128(x)
    Bt, L, H = u.shape
    P = Lambda.shape[0]
    fl = None if is_first is None else np.ascontiguousarray(is_first, dtype=np.uint8)
    x0c = None if x0 is None else _c128(x0)
    out = {
        "du": np.empty((Bt, L, H), np.float64),
        "dLambda": np.empty(P, np.complex128),
        "dB": np.empty((P, H), np.complex128),
        "dC": np.empty((H, P), np.complex128),
        "dD": np.empty(H, np.float64),
        "dlog_delta": np.empty(P, np.float64),
        "dx0": np.empty((Bt, P), np.complex128),
    }
    rc = lib.ssm_oracle_bwd(_ptr(Lambda), _ptr(B), _ptr(C), _ptr(D), _ptr(log_delta), _ptr(u),
                            _ptr(fl), _ptr(x0c), ctypes.c_long(Bt), ctypes.c_long(L),
                            ctypes.c_long(H), ctypes.c_long(P), _ptr(x), _ptr(dy),
                            _ptr(out["du"]), _ptr(out["dLambda"]), _ptr(out["dB"]),
                            _ptr(out["dC"]), _ptr(out["dD"]), _ptr(out["dlog_delta"]),
                            _ptr(out["dx0"]), ctypes.c_int(nthreads))
    if rc != 0:
        raise MemoryError("ssm_oracle_bwd failed")
    return out


def run_workload(inp: Dict[str, Optional[np.ndarray]], backward_pass: bool, nthreads: int = 1):
    """Forward (and gradient pass) on a dict produced by the synthetic-workload generator."""
    fwd = forward(inp["Lambda"], inp["B"], inp["C"], inp["D"], inp["log_delta"], inp["u"],
                  inp["is_first"], inp["x0"], nthreads)
    if backward_pass:
        fwd.update(backward(inp["Lambda"], inp["B"], inp["C"], inp["D"], inp["log_delta"],
                            inp["u"], inp["is_first"], inp["x0"], fwd["x"], inp["dy"], nthreads))
    return fwd


# ---------------------------------------------------------------------------------------------
# Finite-difference checker: perturbs every real degree of freedom of every input of the
# float64 forward (real and imaginary parts separately) and differences l = sum(dy * y).
# It never looks at the analytic gradient code.
# ---------------------------------------------------------------------------------------------
_GRAD_OF = {"u": "du", "Lambda": "dLambda", "B": "dB", "C": "dC", "D": "dD",
            "log_delta": "dlog_delta", "x0": "dx0"}


def _loss(params, is_first, dy):
    out = forward(params["Lambda"], params["B"], params["C"], params["D"], params["log_delta"],
                  params["u"], is_first, params.get("x0"))
    return float(np.sum(dy * out["y"]))


def fd_gradients(Lambda, B, C, D, log_delta, u, is_first, x0, dy, eps: float = 1e-6):
    """Central differences of l = sum(dy*y) w.r.t. every input; complex inputs get
    dl/dRe + i dl/dIm.  O(#dof) forward passes: tiny shapes only."""
    params = {"Lambda": _c128(Lambda).copy(), "B": _c128(B).copy(), "C": _c128(C).copy(),
              "D": _f64(D).copy(), "log_delta": _f64(log_delta).copy(), "u": _f64(u).copy()}
    if x0 is not None:
        params["x0"] = _c128(x0).copy()
    dy = _f64(dy)
    grads = {}
    for name, arr in params.items():
        gout = np.zeros_like(arr)
        flat = arr.reshape(-1)
        gflat = gout.reshape(-1)
        for i in range(flat.size):
            base = flat[i]
            parts = (1.0, 1j) if np.iscomplexobj(arr) else (1.0,)
            val = 0.0
            for unit in parts:
                flat[i] = base + eps * unit
                lp = _loss(params, is_first, dy)
                flat[i] = base - eps * unit
                lm = _loss(params, is_first, dy)
                flat[i] = base
                val = val + unit * (lp - lm) / (2.0 * eps)
            gflat[i] = val
        grads[_GRAD_OF[name]] = gout
    return grads


def fd_directional(inp, direction, dy, eps: float = 1e-6, nthreads: int = 1):
    """(l(theta + eps d) - l(theta - eps d)) / (2 eps) for one direction d over all inputs
    (dict with the same keys as the inputs it perturbs).  Two forward passes: usable at full size."""
    def shifted(sign):
        q = {}
        for k in ("Lambda", "B", "C", "D", "log_delta", "u", "x0"):
            a = inp.get(k)
            if a is None:
                q[k] = None
                continue
            a = _c128(a) if np.iscomplexobj(a) else _f64(a)
            q[k] = a + sign * eps * direction[k] if k in direction else a
        out = forward(q["Lambda"], q["B"], q["C"], q["D"], q["log_delta"], q["u"],
                      inp.get("is_first"), q["x0"], nthreads)
        return float(np.sum(_f64(dy) * out["y"]))
    return (shifted(+1.0) - shifted(-1.0)) / (2.0 * eps)
