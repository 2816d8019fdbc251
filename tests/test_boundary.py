"""Host-side contract of the C-ABI library: it loads without a GPU, exports every symbol the
header declares, and every argument error is reported before any launch."""
import ctypes
import os
import re

import pytest

from paper_2502_20168_amd import binding as ssm
from paper_2502_20168_amd import build as ssm_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if ssm_build.is_stale():
        ssm_build.build()
    return ssm.lib()


def test_every_declared_symbol_is_exported(lib):
    header = "".join(open(os.path.join(ROOT, "include", h)).read() for h in ("ssm.h", "ssm_measure.h"))
    declared = set(re.findall(r"\b(ssm_[a-z0-9_]+)\s*\(", header))
    assert declared == set(ssm.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_strerror_covers_every_code(lib):
    texts = {ssm.strerror(c) for c in range(7)}
    assert len(texts) == 7 and all(texts)
    assert ssm.strerror(99) == "unknown status"
    assert ssm.ssm_version() >= 100


def test_workspace_bytes(lib):
    assert ssm.ssm_workspace_bytes(16, 256, 512, 512, False) > 16 * 256 * 512 * 8
    assert ssm.ssm_workspace_bytes(16, 256, 512, 512, True) > ssm.ssm_workspace_bytes(16, 256, 512, 512, False)
    assert ssm.ssm_workspace_bytes(4, 4096, 1, 256, True) <= ssm.ssm_workspace_bytes(4, 4096, 256, 256, True)
    for bad in [(0, 1, 1, 1), (1, 0, 1, 1), (1, 1, 0, 1), (1, 1, 1, 0), (-3, 8, 8, 8),
                (1, 1, 65537, 1), (1, 1, 1, 65537), (1 << 20, 1 << 20, 8, 8)]:
        assert ssm.ssm_workspace_bytes(*bad, False) == 0


FAKE = 0x10000  # never dereferenced: every check below fails before a launch


def _fwd_args(**over):
    a = dict(Lambda=FAKE, B=FAKE, C=FAKE, D=FAKE, log_delta=FAKE, u=FAKE, is_first=None, x0=None,
             Bt=2, L=8, H=4, P=4, y=FAKE, x=FAKE, x_last=None, ws=FAKE, ws_bytes=1 << 30, stream=None)
    a.update(over)
    return [a[k] for k in ("Lambda", "B", "C", "D", "log_delta", "u", "is_first", "x0", "Bt", "L", "H",
                           "P", "y", "x", "x_last", "ws", "ws_bytes", "stream")]


def _bwd_args(**over):
    a = dict(Lambda=FAKE, B=FAKE, C=FAKE, D=FAKE, log_delta=FAKE, u=FAKE, is_first=None, x0=None,
             Bt=2, L=8, H=4, P=4, x=FAKE, dy=FAKE, du=FAKE, dLambda=FAKE, dB=FAKE, dC=FAKE, dD=FAKE,
             dlog_delta=FAKE, dx0=None, ws=FAKE, ws_bytes=1 << 30, stream=None)
    a.update(over)
    return [a[k] for k in ("Lambda", "B", "C", "D", "log_delta", "u", "is_first", "x0", "Bt", "L", "H",
                           "P", "x", "dy", "du", "dLambda", "dB", "dC", "dD", "dlog_delta", "dx0", "ws",
                           "ws_bytes", "stream")]


def test_forward_argument_errors_need_no_gpu(lib):
    for name in ("Lambda", "B", "C", "D", "log_delta", "u", "y"):
        assert lib.ssm_scan_fwd(*_fwd_args(**{name: None})) == ssm.SSM_ERR_INVALID_ARG, name
    for dim in ("Bt", "L", "H", "P"):
        assert lib.ssm_scan_fwd(*_fwd_args(**{dim: 0})) == ssm.SSM_ERR_INVALID_ARG
        assert lib.ssm_scan_fwd(*_fwd_args(**{dim: -1})) == ssm.SSM_ERR_INVALID_ARG
    assert lib.ssm_scan_fwd(*_fwd_args(H=1 << 17)) == ssm.SSM_ERR_UNSUPPORTED
    assert lib.ssm_scan_fwd(*_fwd_args(Bt=1 << 31, L=2)) == ssm.SSM_ERR_UNSUPPORTED
    assert lib.ssm_scan_fwd(*_fwd_args(Lambda=FAKE + 4)) == ssm.SSM_ERR_INVALID_ARG      # misaligned
    assert lib.ssm_scan_fwd(*_fwd_args(u=FAKE + 2)) == ssm.SSM_ERR_INVALID_ARG
    assert lib.ssm_scan_fwd(*_fwd_args(ws=None)) == ssm.SSM_ERR_WORKSPACE
    assert lib.ssm_scan_fwd(*_fwd_args(ws=FAKE + 64)) == ssm.SSM_ERR_WORKSPACE
    need = ssm.ssm_workspace_bytes(2, 8, 4, 4, False)
    assert lib.ssm_scan_fwd(*_fwd_args(ws_bytes=need - 1)) == ssm.SSM_ERR_WORKSPACE
    ms = (ctypes.c_float * 4)()
    assert lib.ssm_scan_fwd_profiled(*_fwd_args(u=None), ctypes.cast(ms, ctypes.c_void_p)) == ssm.SSM_ERR_INVALID_ARG
    assert lib.ssm_scan_fwd_profiled(*_fwd_args(), None) == ssm.SSM_ERR_INVALID_ARG


def test_backward_argument_errors_need_no_gpu(lib):
    for name in ("Lambda", "B", "C", "D", "log_delta", "u", "x", "dy", "du", "dLambda", "dB", "dC", "dD",
                 "dlog_delta"):
        assert lib.ssm_scan_bwd(*_bwd_args(**{name: None})) == ssm.SSM_ERR_INVALID_ARG, name
    assert lib.ssm_scan_bwd(*_bwd_args(P=0)) == ssm.SSM_ERR_INVALID_ARG
    assert lib.ssm_scan_bwd(*_bwd_args(P=1 << 17)) == ssm.SSM_ERR_UNSUPPORTED
    need = ssm.ssm_workspace_bytes(2, 8, 4, 4, True)
    assert need > ssm.ssm_workspace_bytes(2, 8, 4, 4, False)
    assert lib.ssm_scan_bwd(*_bwd_args(ws_bytes=need - 1)) == ssm.SSM_ERR_WORKSPACE
    assert lib.ssm_scan_bwd(*_bwd_args(dx0=FAKE + 4)) == ssm.SSM_ERR_INVALID_ARG


def test_other_entry_points_argument_errors(lib):
    assert lib.ssm_discretize(None, FAKE, FAKE, 4, 4, FAKE, FAKE, None) == ssm.SSM_ERR_INVALID_ARG
    assert lib.ssm_discretize(FAKE, None, FAKE, 4, 4, FAKE, FAKE, None) == ssm.SSM_ERR_INVALID_ARG
    assert lib.ssm_discretize(FAKE, FAKE, FAKE, 0, 4, FAKE, FAKE, None) == ssm.SSM_ERR_INVALID_ARG
    assert lib.ssm_discretize(FAKE, FAKE, FAKE, 1 << 17, 4, FAKE, FAKE, None) == ssm.SSM_ERR_UNSUPPORTED
    assert lib.ssm_scan_states(None, FAKE, None, None, 2, 8, 4, None, FAKE, 1 << 20, None) == ssm.SSM_ERR_INVALID_ARG
    assert lib.ssm_scan_states(FAKE, FAKE, None, None, 2, 0, 4, None, FAKE, 1 << 20, None) == ssm.SSM_ERR_INVALID_ARG
    assert lib.ssm_scan_states(FAKE, FAKE, None, None, 2, 8, 4, None, FAKE, 16, None) == ssm.SSM_ERR_WORKSPACE
    assert lib.ssm_scan_states_reverse(FAKE, FAKE, None, None, None, 2, 8, 4, FAKE, None, FAKE, 1 << 20,
                                       None) == ssm.SSM_ERR_INVALID_ARG
    assert lib.ssm_scan_states_reverse(FAKE, FAKE, FAKE, None, None, 2, 8, 4, FAKE, None, FAKE, 16,
                                       None) == ssm.SSM_ERR_WORKSPACE
    assert lib.ssm_workspace_status(None, None) == ssm.SSM_ERR_WORKSPACE
    # step mode
    need = ssm.ssm_step_plan_bytes(4, 4)
    assert need > 0 and ssm.ssm_step_plan_bytes(0, 4) == 0 and ssm.ssm_step_plan_bytes(4, 1 << 17) == 0
    assert lib.ssm_step_prepare(None, FAKE, FAKE, FAKE, 4, 4, FAKE, need, None) == ssm.SSM_ERR_INVALID_ARG
    assert lib.ssm_step_prepare(FAKE, FAKE, FAKE, FAKE, 4, 4, FAKE, need - 1, None) == ssm.SSM_ERR_WORKSPACE
    assert lib.ssm_step_prepare(FAKE, FAKE, FAKE, FAKE, 4, 4, None, need, None) == ssm.SSM_ERR_WORKSPACE
    assert lib.ssm_step(FAKE, need, None, FAKE, None, None, 2, 4, 4, FAKE, FAKE, None) == ssm.SSM_ERR_INVALID_ARG
    assert lib.ssm_step(FAKE, need, FAKE, FAKE, None, None, 0, 4, 4, FAKE, FAKE, None) == ssm.SSM_ERR_INVALID_ARG
    assert lib.ssm_step(FAKE, need - 1, FAKE, FAKE, None, None, 2, 4, 4, FAKE, FAKE, None) == ssm.SSM_ERR_WORKSPACE
    assert lib.ssm_step(FAKE, need, FAKE, FAKE, FAKE + 512, None, 2, 4, 4, FAKE + 512, FAKE, None) == ssm.SSM_ERR_INVALID_ARG
    G = FAKE + 4096
    assert lib.ssm_step_bwd(FAKE, need, FAKE, None, None, None, 2, 4, 4, G, FAKE, None, None) == ssm.SSM_ERR_INVALID_ARG
    assert lib.ssm_step_bwd(FAKE, need, FAKE, FAKE, None, None, 2, 4, 4, None, FAKE, None, None) == ssm.SSM_ERR_INVALID_ARG
    assert lib.ssm_step_bwd(FAKE, need, FAKE, FAKE, None, None, 2, 0, 4, G, FAKE, None, None) == ssm.SSM_ERR_INVALID_ARG
    assert lib.ssm_step_bwd(FAKE, need - 1, FAKE, FAKE, None, None, 2, 4, 4, G, FAKE, None, None) == ssm.SSM_ERR_WORKSPACE
    assert lib.ssm_step_bwd(FAKE, need, FAKE, FAKE, G, None, 2, 4, 4, G, FAKE, None, None) == ssm.SSM_ERR_INVALID_ARG
    assert lib.ssm_step_bwd(FAKE, need, FAKE, FAKE, None, None, 2, 4, 4, G, FAKE, G, None) == ssm.SSM_ERR_INVALID_ARG


def test_block_entry_points_argument_errors(lib):
    # lambda-return: no workspace, errors before any launch
    assert lib.ssm_lambda_return(None, FAKE, FAKE, 0.9, 0.9, 4, 8, FAKE, None) == ssm.SSM_ERR_INVALID_ARG
    assert lib.ssm_lambda_return(FAKE, FAKE, FAKE, 0.9, 0.9, 0, 8, FAKE, None) == ssm.SSM_ERR_INVALID_ARG
    assert lib.ssm_lambda_return(FAKE, FAKE, FAKE, 0.9, 0.9, 4, 8, None, None) == ssm.SSM_ERR_INVALID_ARG
    assert lib.ssm_lambda_return(FAKE, FAKE + 2, FAKE, 0.9, 0.9, 4, 8, FAKE, None) == ssm.SSM_ERR_INVALID_ARG
    assert lib.ssm_lambda_return(FAKE, FAKE, FAKE, 0.9, 0.9, 1 << 31, 8, FAKE, None) == ssm.SSM_ERR_UNSUPPORTED
    assert lib.ssm_lambda_return_bwd(FAKE, FAKE, FAKE, None, 0.9, 0.9, 4, 8, FAKE, FAKE, FAKE,
                                     None) == ssm.SSM_ERR_INVALID_ARG
    assert lib.ssm_lambda_return_bwd(FAKE, FAKE, FAKE, FAKE, 0.9, 0.9, 4, -1, FAKE, FAKE, FAKE,
                                     None) == ssm.SSM_ERR_INVALID_ARG
    # half-GLU
    need_f, need_b = ssm.ssm_half_glu_workspace_bytes(64, 32, False), ssm.ssm_half_glu_workspace_bytes(64, 32, True)
    assert 64 * 32 * 4 <= need_f < need_b
    assert ssm.ssm_half_glu_workspace_bytes(0, 32, False) == 0 and ssm.ssm_half_glu_workspace_bytes(64, 1 << 17, True) == 0
    assert lib.ssm_half_glu_fwd(None, FAKE, 64, 32, FAKE, None, FAKE, need_f, None) == ssm.SSM_ERR_INVALID_ARG
    assert lib.ssm_half_glu_fwd(FAKE, FAKE, 64, 0, FAKE, None, FAKE, need_f, None) == ssm.SSM_ERR_INVALID_ARG
    assert lib.ssm_half_glu_fwd(FAKE + 4, FAKE, 64, 32, FAKE, None, FAKE, need_f, None) == ssm.SSM_ERR_INVALID_ARG
    assert lib.ssm_half_glu_fwd(FAKE, FAKE, 64, 32, FAKE, None, FAKE, need_f - 1, None) == ssm.SSM_ERR_WORKSPACE
    assert lib.ssm_half_glu_fwd(FAKE, FAKE, 64, 32, FAKE, None, None, need_f, None) == ssm.SSM_ERR_WORKSPACE
    assert lib.ssm_half_glu_fwd(FAKE, FAKE, 64, 1 << 17, FAKE, None, FAKE, need_f, None) == ssm.SSM_ERR_UNSUPPORTED
    assert lib.ssm_half_glu_bwd(FAKE, FAKE, None, FAKE, 64, 32, FAKE, FAKE, FAKE, need_b, None) == ssm.SSM_ERR_INVALID_ARG
    assert lib.ssm_half_glu_bwd(FAKE, FAKE, FAKE, FAKE, 64, 32, FAKE, FAKE, FAKE, need_f, None) == ssm.SSM_ERR_WORKSPACE
    assert lib.ssm_half_glu_bwd(FAKE, FAKE, FAKE, FAKE + 8, 64, 32, FAKE, FAKE, FAKE, need_b,
                                None) == ssm.SSM_ERR_INVALID_ARG


def test_s5_block_argument_errors(lib):
    need_f, need_b = ssm.ssm_block_workspace_bytes(2, 8, 4, 4, False), ssm.ssm_block_workspace_bytes(2, 8, 4, 4, True)
    assert need_f > ssm.ssm_workspace_bytes(2, 8, 4, 4, False) and need_b > ssm.ssm_workspace_bytes(2, 8, 4, 4, True)
    assert ssm.ssm_block_workspace_bytes(2, 0, 4, 4, False) == 0
    F = [FAKE] * 9
    assert lib.ssm_block_fwd(*F, 2, 8, 4, 4, FAKE, None, None, FAKE, None, FAKE, need_f, None) == ssm.SSM_ERR_INVALID_ARG
    assert lib.ssm_block_fwd(*F, 2, 8, 4, 4, None, FAKE, None, FAKE, None, FAKE, need_f, None) == ssm.SSM_ERR_INVALID_ARG
    assert lib.ssm_block_fwd(*F, 2, 8, 4, 4, FAKE, FAKE, None, FAKE, None, FAKE, need_f - 1, None) == ssm.SSM_ERR_WORKSPACE
    assert lib.ssm_block_fwd(*F, 2, 8, 0, 4, FAKE, FAKE, None, FAKE, None, FAKE, need_f, None) == ssm.SSM_ERR_INVALID_ARG
    Gd = [FAKE] * 8
    assert lib.ssm_block_bwd(*F, 2, 8, 4, 4, FAKE, FAKE, FAKE, None, *Gd, FAKE, need_b, None) == ssm.SSM_ERR_INVALID_ARG
    assert lib.ssm_block_bwd(*F, 2, 8, 4, 4, FAKE, FAKE, FAKE, FAKE, *Gd, FAKE, need_b - 1, None) == ssm.SSM_ERR_WORKSPACE


def test_no_allocation_entry_point_argument_errors(lib):
    """Errors of ssm_scan_states_noalloc come before any launch (and before the scratch is looked up)."""
    f = lib.ssm_scan_states_noalloc
    assert f(None, FAKE, None, None, 2, 8, 4, None, None) == ssm.SSM_ERR_INVALID_ARG
    assert f(FAKE, None, None, None, 2, 8, 4, None, None) == ssm.SSM_ERR_INVALID_ARG
    assert f(FAKE, FAKE, None, None, 2, 0, 4, None, None) == ssm.SSM_ERR_INVALID_ARG
    assert f(FAKE, FAKE, None, None, 2, 8, 1 << 17, None, None) == ssm.SSM_ERR_UNSUPPORTED
    # 64 sequences of 8192 steps with 256 states need 16 MiB of look-back descriptors: beyond the built-in 8 MiB
    assert ssm.ssm_workspace_bytes(64, 8192, 1, 256, False) > ssm.SSM_NOALLOC_SCRATCH_BYTES
    assert f(FAKE, FAKE, None, None, 64, 8192, 256, None, None) == ssm.SSM_ERR_SCRATCH_LIMIT
    assert "scratch" in ssm.strerror(ssm.SSM_ERR_SCRATCH_LIMIT)


def test_spin_limit_hook_returns_the_previous_bound(lib):
    old = ssm.ssm_set_spin_limit(7)
    assert ssm.ssm_set_spin_limit(old) == 7
    assert ssm.ssm_set_spin_limit(old) == old


def test_binding_refuses_cpu_tensors(lib):
    import numpy as np
    import torch
    z = torch.zeros(4, dtype=torch.complex64)
    with pytest.raises(ValueError):
        ssm.ssm_scan_fwd(z, torch.zeros(4, 3, dtype=torch.complex64), torch.zeros(3, 4, dtype=torch.complex64),
                         torch.zeros(3), torch.zeros(4), torch.zeros(1, 5, 3))
