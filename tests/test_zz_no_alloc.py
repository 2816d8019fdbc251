"""ssm_scan_states_noalloc (the entry point for callers that cannot allocate: built-in device scratch
instead of a workspace) against ssm_scan_states, through the C ABI: the same kernels on different
scratch memory must give the same bits.  Two calls in a row, the second on a smaller input, so that
what the first call left in the shared scratch (ticket counters, look-back descriptors) is seen to be
cleared; both shapes split their sequences over several workgroups along time, i.e. really use it."""
import numpy as np
import pytest

from oracle import ssm_oracle as orc
from paper_2502_20168_amd import binding as ssm
from tests.parity_util import TOL_FWD, assert_close

pytestmark = pytest.mark.gpu


def _case(Bt, L, P, seed):
    rng = np.random.default_rng(seed)
    Abar = (rng.uniform(0.9, 1.0, P) * np.exp(1j * rng.uniform(0, np.pi, P))).astype(np.complex64)
    v = (rng.normal(size=(Bt, L, P)) + 1j * rng.normal(size=(Bt, L, P))).astype(np.complex64)
    x0 = (rng.normal(size=(Bt, P)) + 1j * rng.normal(size=(Bt, P))).astype(np.complex64)
    fl = (rng.random((Bt, L)) < 0.003).astype(np.uint8)
    return Abar, v, fl, x0


def test_no_allocation_entry_point_equals_the_workspace_one_on_two_calls_in_a_row():
    import torch
    assert torch.cuda.is_available()
    for Bt, L, P, seed in ((3, 3000, 40, 1), (2, 700, 24, 2)):          # the second call is the smaller one
        print("no-alloc scan", Bt, L, P, flush=True)
        Abar, v, fl, x0 = _case(Bt, L, P, seed)
        assert 256 < ssm.ssm_workspace_bytes(Bt, L, 1, P, False) <= ssm.SSM_NOALLOC_SCRATCH_BYTES
        dA, dfl, dx0 = (torch.from_numpy(a).cuda() for a in (Abar, fl, x0))
        v_ws, v_na = torch.from_numpy(v).cuda(), torch.from_numpy(v).cuda()
        xl_na = torch.empty((Bt, P), dtype=torch.complex64, device="cuda")
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        ssm.ssm_scan_states_noalloc(dA, v_na, dfl, dx0, x_last=xl_na)
        assert torch.cuda.memory_allocated() == before              # the binding allocated nothing either
        assert ssm.ssm_scan_states_noalloc_status() == ssm.SSM_OK
        _, xl_ws = ssm.ssm_scan_states(dA, v_ws, dfl, dx0)
        torch.cuda.synchronize()
        assert torch.equal(v_na, v_ws), "states differ from ssm_scan_states"
        assert torch.equal(xl_na, xl_ws), "x_last differs from ssm_scan_states"
        # and both are right (integer-exact agreement above, the oracle within the forward tolerance)
        ref = orc.scan(Abar, v, fl, x0)
        assert_close(v_na.cpu().numpy(), ref, TOL_FWD, "no-alloc x")


def test_no_allocation_entry_point_refuses_shapes_beyond_its_scratch():
    import torch
    Bt, L, P = 64, 8192, 256
    assert ssm.ssm_workspace_bytes(Bt, L, 1, P, False) > ssm.SSM_NOALLOC_SCRATCH_BYTES
    dummy = torch.zeros(8, dtype=torch.complex64, device="cuda")      # never touched: the call fails before any launch
    rc = ssm.lib().ssm_scan_states_noalloc(dummy.data_ptr(), dummy.data_ptr(), None, None, Bt, L, P, None, None)
    assert rc == ssm.SSM_ERR_SCRATCH_LIMIT
