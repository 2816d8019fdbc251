"""GPU parity of the lambda-return and the half-GLU gate (and their adjoints) with the float64
oracle, element by element through the C ABI."""
import numpy as np
import pytest

from oracle import block_oracle as borc
from paper_2502_20168_amd import workloads as wl
from parity_util import TOL_FWD, TOL_GRAD, assert_close

pytestmark = pytest.mark.gpu

GAMMA, LAM = 0.997, 0.95


def _dev(d):
    import torch
    return {k: torch.from_numpy(v).cuda() for k, v in d.items()}


# several blocks and a ragged tail in N; T from the degenerate single step to beyond the unrolled loop
RETURN_SHAPES = [(16, 1024), (1, 5), (2, 7), (5, 300), (33, 4097), (15, 65536), (256, 513)]


@pytest.mark.parametrize("T,N", RETURN_SHAPES)
def test_lambda_return_matches_oracle(T, N):
    import torch
    from paper_2502_20168_amd import binding as ssm
    inp = wl.gen_returns(T, N, seed=T * 7919 + N)
    d = _dev(inp)
    ret = ssm.ssm_lambda_return(d["reward"], d["cont"], d["value"], GAMMA, LAM)
    dr, dc, dv = ssm.ssm_lambda_return_bwd(d["cont"], d["value"], ret, d["dret"], GAMMA, LAM)
    torch.cuda.synchronize()
    ref = borc.lambda_return(inp["reward"], inp["cont"], inp["value"], GAMMA, LAM)
    rdr, rdc, rdv = borc.lambda_return_grad(inp["reward"], inp["cont"], inp["value"], GAMMA, LAM, inp["dret"])
    ret = ret.cpu().numpy()
    assert np.array_equal(ret[-1], inp["value"][-1])          # V_T = v_T exactly
    assert_close(ret, ref, TOL_FWD, "ret")
    assert_close(dv.cpu().numpy(), rdv, TOL_GRAD, "dvalue")
    if T > 1:
        assert_close(dr.cpu().numpy(), rdr, TOL_GRAD, "dreward")
        assert_close(dc.cpu().numpy(), rdc, TOL_GRAD, "dcont")
    assert not dr[-1].any().item() and not dc[-1].any().item()


def test_lambda_return_extremes_of_lambda():
    import torch
    from paper_2502_20168_amd import binding as ssm
    inp = wl.gen_returns(12, 777, seed=5)
    d = _dev(inp)
    for lam in (0.0, 1.0):
        ret = ssm.ssm_lambda_return(d["reward"], d["cont"], d["value"], 0.9, lam).cpu().numpy()
        assert_close(ret, borc.lambda_return(inp["reward"], inp["cont"], inp["value"], 0.9, lam), TOL_FWD, "ret")
    # an episode end (c = 0) cuts the return: V_k = r_k exactly
    k = 4
    d["cont"][k] = 0.0
    ret = ssm.ssm_lambda_return(d["reward"], d["cont"], d["value"], 0.9, 0.95)
    torch.cuda.synchronize()
    assert torch.equal(ret[k], d["reward"][k])


# (T, H): the benchmark shape, ragged tiles, a width that is no multiple of 4 (scalar tails and the
# guarded GEMM path), the vision width, ragged token tiles at a width that takes two fp16 planes
GLU_SHAPES = [(4096, 512), (128, 32), (300, 96), (1000, 257), (2048, 1024), (5, 3), (3333, 576)]


@pytest.mark.parametrize("T,H", GLU_SHAPES)
def test_half_glu_matches_oracle(T, H):
    import torch
    from paper_2502_20168_amd import binding as ssm
    inp = wl.gen_half_glu(T, H, seed=T + 31 * H)
    d = _dev(inp)
    y, gate = ssm.ssm_half_glu_fwd(d["u"], d["W"])
    du, dW = ssm.ssm_half_glu_bwd(d["u"], d["W"], gate, d["dy"])
    torch.cuda.synchronize()
    ref_y = borc.half_glu(inp["u"], inp["W"])
    ref_gate = borc.sigmoid(borc.gelu(inp["u"]) @ inp["W"].astype(np.float64))
    ref_du, ref_dW = borc.half_glu_grad(inp["u"], inp["W"], inp["dy"])
    assert_close(y.cpu().numpy(), ref_y, TOL_FWD, "y")
    assert_close(gate.cpu().numpy(), ref_gate, TOL_FWD, "gate")
    assert_close(du.cpu().numpy(), ref_du, TOL_GRAD, "du")
    assert_close(dW.cpu().numpy(), ref_dW, TOL_GRAD, "dW")


def test_half_glu_zero_weights_and_no_gate_output():
    import torch
    from paper_2502_20168_amd import binding as ssm
    inp = wl.gen_half_glu(260, 64, seed=3)
    d = _dev(inp)
    y, gate = ssm.ssm_half_glu_fwd(d["u"], torch.zeros_like(d["W"]), want_gate=False)
    torch.cuda.synchronize()
    assert gate is None
    assert torch.equal(y, 0.5 * d["u"])                       # sigmoid(0) = 1/2 exactly


def test_half_glu_is_bitwise_repeatable():
    import torch
    from paper_2502_20168_amd import binding as ssm
    d = _dev(wl.gen_half_glu(1024, 256, seed=4))
    outs = []
    for _ in range(2):
        y, gate = ssm.ssm_half_glu_fwd(d["u"], d["W"])
        du, dW = ssm.ssm_half_glu_bwd(d["u"], d["W"], gate, d["dy"])
        torch.cuda.synchronize()
        outs.append((y.clone(), du.clone(), dW.clone()))
    assert all(torch.equal(a, b) for a, b in zip(*outs))


# the benchmark shape (the K halves of y meet in the launch; the gate on two fp16 planes), two small ragged ones,
# and one whose output projection runs on 64x128 tiles and hands the gate its row maxima from there
# ... and two whose width is an odd multiple of 64 (the last column tile of the output projection has a wavefront
# with no columns at all: no row maxima from there), with separate scan kernels and with scanning projections
@pytest.mark.parametrize("Bt,L,H,P", [(16, 256, 512, 512), (3, 129, 50, 33), (2, 600, 96, 40), (8, 512, 512, 64),
                                      (81, 50, 576, 288), (16, 256, 576, 512)])
def test_s5_block_matches_oracle_composition(Bt, L, H, P):
    """SSM layer + half-GLU gate in one call (GELU of the layer's output formed in the output
    projection's store) against the two oracles composed: forward outputs, then every gradient."""
    import torch
    from oracle import ssm_oracle as sorc
    from paper_2502_20168_amd import binding as ssm
    w = wl.custom("block", Bt, L, H, P, backward=True, p_reset=0.02, force_first=True, with_x0=True, seed=41)
    inp = wl.gen_inputs(w)
    W = wl.gen_half_glu(4, H, seed=42)["W"]
    par = (inp["Lambda"], inp["B"], inp["C"], inp["D"], inp["log_delta"])
    rf = sorc.forward(*par, inp["u"], inp["is_first"], inp["x0"], nthreads=8)
    y2 = rf["y"].reshape(Bt * L, H)
    ref_out = borc.half_glu(y2, W).reshape(Bt, L, H)
    dy_pre, ref_dW = borc.half_glu_grad(y2, W, inp["dy"].reshape(Bt * L, H))
    rb = sorc.backward(*par, inp["u"], inp["is_first"], inp["x0"], rf["x"], dy_pre.reshape(Bt, L, H), nthreads=8)
    d = ssm.to_device(inp)
    Wd = torch.from_numpy(W).cuda()
    f = ssm.ssm_block_fwd(d["Lambda"], d["B"], d["C"], d["D"], d["log_delta"], Wd, d["u"], d["is_first"], d["x0"])
    b = ssm.ssm_block_bwd(d["Lambda"], d["B"], d["C"], d["D"], d["log_delta"], Wd, d["u"], d["is_first"], d["x0"],
                          f["x"], f["y"], f["gate"], d["dy"])
    torch.cuda.synchronize()
    assert_close(f["y"].cpu().numpy(), rf["y"], TOL_FWD, "block y")
    assert_close(f["out"].cpu().numpy(), ref_out, TOL_FWD, "block out")
    assert_close(f["x_last"].cpu().numpy(), rf["x_last"], TOL_FWD, "block x_last")
    assert_close(b["dW"].cpu().numpy(), ref_dW, TOL_GRAD, "block dW")
    for k in ("du", "dLambda", "dB", "dC", "dD", "dlog_delta", "dx0"):
        assert_close(b[k].cpu().numpy(), rb[k], TOL_GRAD, "block " + k)
    # the fused call equals the two separate calls bit for bit
    f2 = ssm.ssm_scan_fwd(d["Lambda"], d["B"], d["C"], d["D"], d["log_delta"], d["u"], d["is_first"], d["x0"])
    out2, gate2 = ssm.ssm_half_glu_fwd(f2["y"].reshape(Bt * L, H), Wd)
    torch.cuda.synchronize()
    assert torch.equal(f2["y"], f["y"]) and torch.equal(out2.reshape(Bt, L, H), f["out"])


def _block_random_shapes(n, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    return [(int(rng.integers(1, 3000)), int(rng.choice([rng.integers(1, 40), rng.integers(40, 400), 4 * rng.integers(8, 130)])))
            for _ in range(n)]


@pytest.mark.parametrize("T,H", _block_random_shapes(8, 424242))
def test_half_glu_seeded_random_shapes(T, H):
    test_half_glu_matches_oracle(T, H)


@pytest.mark.parametrize("T,N", [(int(t), int(n)) for t, n in
                                 np.random.Generator(np.random.PCG64(7)).integers([1, 1], [70, 9000], size=(8, 2))])
def test_lambda_return_seeded_random_shapes(T, N):
    test_lambda_return_matches_oracle(T, N)


@pytest.mark.parametrize("Bt,L,H,P", [(16, 256, 512, 512), (81, 50, 576, 288), (16, 256, 576, 512), (4, 4096, 256, 256),
                                      (24, 100, 512, 512), (13, 100, 1200, 256), (3, 129, 50, 33), (64, 16, 704, 520),
                                      (292, 7, 668, 128), (16, 64, 256, 256)])
def test_no_call_writes_outside_its_workspace(Bt, L, H, P):
    """Layer, S5 block and gate, forward and gradient pass, each on a workspace of exactly the size the library
    asks for, between two guard zones filled with a pattern: the zones are untouched afterwards."""
    import torch
    from paper_2502_20168_amd import binding as ssm
    guard = 1 << 16

    def guarded(nbytes):
        buf = torch.full((guard + nbytes + guard,), 0xA5, dtype=torch.uint8, device="cuda")
        return buf, buf[guard:guard + nbytes]

    def check(buf, nbytes, what):
        assert bool((buf[:guard] == 0xA5).all()), "write below the workspace: " + what
        assert bool((buf[guard + nbytes:] == 0xA5).all()), "write past the workspace: " + what

    w = wl.custom("guard", Bt, L, H, P, backward=True, p_reset=0.02, force_first=True, with_x0=True, seed=5)
    d = ssm.to_device(wl.gen_inputs(w))
    par = (d["Lambda"], d["B"], d["C"], d["D"], d["log_delta"])
    Wd = torch.from_numpy(wl.gen_half_glu(4, H, seed=7)["W"]).cuda()
    T = Bt * L
    sizes = {"layer": (ssm.ssm_workspace_bytes(Bt, L, H, P, False), ssm.ssm_workspace_bytes(Bt, L, H, P, True)),
             "block": (ssm.ssm_block_workspace_bytes(Bt, L, H, P, False), ssm.ssm_block_workspace_bytes(Bt, L, H, P, True)),
             "gate": (ssm.ssm_half_glu_workspace_bytes(T, H, False), ssm.ssm_half_glu_workspace_bytes(T, H, True))}
    bufs = {k: (guarded(nf), guarded(nb)) for k, (nf, nb) in sizes.items()}
    f = ssm.ssm_scan_fwd(*par, d["u"], d["is_first"], d["x0"], workspace=bufs["layer"][0][1])
    ssm.ssm_scan_bwd(*par, d["u"], d["is_first"], d["x0"], f["x"], d["dy"], workspace=bufs["layer"][1][1])
    fb = ssm.ssm_block_fwd(*par, Wd, d["u"], d["is_first"], d["x0"], workspace=bufs["block"][0][1])
    ssm.ssm_block_bwd(*par, Wd, d["u"], d["is_first"], d["x0"], fb["x"], fb["y"], fb["gate"], d["dy"],
                      workspace=bufs["block"][1][1])
    u2 = d["u"].reshape(T, H)
    y, gate = ssm.ssm_half_glu_fwd(u2, Wd, workspace=bufs["gate"][0][1])
    ssm.ssm_half_glu_bwd(u2, Wd, gate, d["dy"].reshape(T, H), workspace=bufs["gate"][1][1])
    torch.cuda.synchronize()
    for k, (nf, nb) in sizes.items():
        check(bufs[k][0][0], nf, k + " forward")
        check(bufs[k][1][0], nb, k + " gradient pass")
