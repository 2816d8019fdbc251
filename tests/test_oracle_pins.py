"""Pins for the float64 CPU oracle: everything here checks the oracle against something that
is NOT the oracle -- the values the paper prints (Eq. 7), closed forms, library routines
(numpy.convolve, scipy.signal.cont2discrete), invariants of the reset operator (Eq. 9-10) and
brute-force finite differences.  No GPU needed."""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import ssm_oracle as orc
from paper_2502_20168_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def small_inputs(Bt=2, L=9, H=3, P=4, seed=1, p_reset=0.0, force_first=False, with_x0=False,
                 **kw):
    w = wl.custom("t", Bt, L, H, P, p_reset=p_reset, force_first=force_first, with_x0=with_x0,
                  seed=seed, **kw)
    return wl.gen_inputs(w)


def naive_discretize(Lambda, log_delta):
    """Textbook ZOH written directly: Abar = exp(Lambda Delta), g = (Abar - 1)/Lambda."""
    Lambda = np.asarray(Lambda, np.complex128)
    delta = np.exp(np.asarray(log_delta, np.float64))
    Abar = np.exp(Lambda * delta)
    return Abar, (Abar - 1.0) / Lambda


# ------------------------------------------------------------------ the paper's operator
def op_plain(ei, ej):
    """S5 binary operator, Eq. 5, for diagonal Abar (products are element-wise)."""
    return (ej[0] * ei[0], ej[0] * ei[1] + ej[1])


def op_reset(ei, ej):
    """Resettable operator, Eq. 10: a set flag on the right element discards the left one."""
    if ej[2] == 0:
        return (ej[0] * ei[0], ej[0] * ei[1] + ej[1], ei[2])
    return (ej[0], ej[1], ej[2])


def test_eq7_worked_unrolling_matches_printed_values():
    rows = [tuple(int(v) for v in ln.split()) for ln in open(os.path.join(GOLDEN, "eq7_unrolling.txt"))
            if ln.strip() and not ln.startswith("#")]
    assert rows == [(1, 1, 1), (2, 2, 2), (3, 3, 3)]
    rng = np.random.default_rng(0)
    P = 5
    Abar = rng.normal(size=P) * 0.5 + 1j * rng.normal(size=P) * 0.5
    v = rng.normal(size=(1, 3, P)) + 1j * rng.normal(size=(1, 3, P))
    x = orc.scan(Abar, v)                       # oracle states x_1..x_3 from x_0 = 0
    acc = (Abar, v[0, 0])
    for k, a_exp, x_idx in rows:
        if k > 1:
            acc = op_plain(acc, (Abar, v[0, k - 1]))
        np.testing.assert_allclose(acc[0], Abar ** a_exp, rtol=1e-14)
        np.testing.assert_allclose(acc[1], x[0, x_idx - 1], rtol=1e-13, atol=1e-15)


def test_reset_operator_is_associative_for_all_flag_patterns():
    rng = np.random.default_rng(1)
    for flags in itertools.product((0, 1), repeat=3):
        e = [(rng.normal() + 1j * rng.normal(), rng.normal() + 1j * rng.normal(), f) for f in flags]
        left = op_reset(op_reset(e[0], e[1]), e[2])
        right = op_reset(e[0], op_reset(e[1], e[2]))
        # the b component is what the method outputs; it and the flag must agree exactly up to
        # rounding, the a component only when no reset occurred (it is unused after a reset)
        assert abs(left[1] - right[1]) < 1e-13
        assert (left[2] or flags[1] or flags[2]) == (right[2] or flags[1] or flags[2])
        if not any(flags[1:]):
            assert abs(left[0] - right[0]) < 1e-13


def _hillis_steele(elems):
    n = len(elems)
    cur = list(elems)
    d = 1
    while d < n:
        nxt = list(cur)
        for i in range(d, n):
            nxt[i] = op_reset(cur[i - d], cur[i])
        cur = nxt
        d *= 2
    return cur


def _tree_scan(elems):
    """Recursive pairwise (up-sweep/down-sweep) inclusive scan: a different bracketing."""
    n = len(elems)
    if n == 1:
        return list(elems)
    pairs = [op_reset(elems[2 * i], elems[2 * i + 1]) for i in range(n // 2)]
    sub = _tree_scan(pairs)
    out = [None] * n
    for i in range(n):
        if i == 0:
            out[i] = elems[0]
        elif i % 2 == 1:
            out[i] = sub[i // 2]
        else:
            out[i] = op_reset(sub[i // 2 - 1], elems[i])
    return out


@pytest.mark.parametrize("L", [1, 2, 7, 16, 37])
def test_parallel_scan_bracketings_equal_the_sequential_oracle(L):
    """Eq. 4 with the operator of Eq. 10, bracketed two different ways, gives the states of the
    sequential recurrence.  The flag element is 1 - c_k = is_first (Eq. 9)."""
    rng = np.random.default_rng(L)
    P = 3
    Abar = 0.9 * np.exp(1j * rng.uniform(0, np.pi, size=P))
    v = rng.normal(size=(1, L, P)) + 1j * rng.normal(size=(1, L, P))
    flags = (rng.random(size=(1, L)) < 0.3).astype(np.uint8)
    x = orc.scan(Abar, v, flags)
    for p in range(P):
        elems = [(Abar[p], v[0, t, p], int(flags[0, t])) for t in range(L)]
        for scanned in (_hillis_steele(elems), _tree_scan(elems)):
            got = np.array([e[1] for e in scanned])
            np.testing.assert_allclose(got, x[0, :, p], rtol=1e-12, atol=1e-13)


# ------------------------------------------------------------------ recurrence, no reset
def test_constant_input_gives_geometric_series():
    inp = small_inputs(Bt=1, L=40, H=3, P=4)
    ubar = np.array([0.7, -1.3, 0.2])
    u = np.broadcast_to(ubar, (1, 40, 3)).copy()
    out = orc.forward(inp["Lambda"], inp["B"], inp["C"], inp["D"], inp["log_delta"], u)
    Abar, g = naive_discretize(inp["Lambda"], inp["log_delta"])
    Bu = g * (inp["B"].astype(np.complex128) @ ubar)
    t = np.arange(40)[:, None]
    expect = Bu * (1.0 - Abar ** (t + 1)) / (1.0 - Abar)
    np.testing.assert_allclose(out["x"][0], expect, rtol=1e-11, atol=1e-15)


def test_impulse_response_and_convolution_against_numpy():
    inp = small_inputs(Bt=1, L=33, H=2, P=5, seed=3)
    L, H, P = 33, 2, 5
    Abar, g = naive_discretize(inp["Lambda"], inp["log_delta"])
    Bbar = g[:, None] * inp["B"].astype(np.complex128)
    C = inp["C"].astype(np.complex128)
    D = inp["D"].astype(np.float64)
    # kernel K[k][h_out, h_in] = Re(C diag(Abar^k) Bbar)
    K = np.stack([np.real(C @ (Abar[:, None] ** k * Bbar)) for k in range(L)])
    # impulse in channel 1 at t0 = 4
    u = np.zeros((1, L, H))
    u[0, 4, 1] = 1.0
    y = orc.forward(inp["Lambda"], inp["B"], inp["C"], inp["D"], inp["log_delta"], u)["y"][0]
    expect = np.zeros((L, H))
    expect[4:, :] = K[: L - 4, :, 1]
    expect[4, 1] += D[1]
    np.testing.assert_allclose(y, expect, rtol=1e-12, atol=1e-15)
    # general input: causal convolution computed by the library routine
    u = inp["u"].astype(np.float64)
    y = orc.forward(inp["Lambda"], inp["B"], inp["C"], inp["D"], inp["log_delta"], u)["y"][0]
    conv = np.zeros((L, H))
    for ho in range(H):
        for hi in range(H):
            conv[:, ho] += np.convolve(u[0, :, hi], K[:, ho, hi])[:L]
    conv += D * u[0]
    np.testing.assert_allclose(y, conv, rtol=1e-11, atol=1e-13)


def test_linearity_in_u():
    inp = small_inputs(Bt=2, L=12, H=3, P=4, seed=5, p_reset=0.2)
    rng = np.random.default_rng(0)
    u1 = rng.normal(size=(2, 12, 3))
    u2 = rng.normal(size=(2, 12, 3))
    f = lambda u: orc.forward(inp["Lambda"], inp["B"], inp["C"], inp["D"], inp["log_delta"], u,
                              inp["is_first"])["y"]
    np.testing.assert_allclose(f(2.5 * u1 - 0.75 * u2), 2.5 * f(u1) - 0.75 * f(u2),
                               rtol=1e-12, atol=1e-13)


def test_zero_transition_is_pure_feedthrough():
    """Abar = 0: no memory.  Scan level: x = v.  Layer level: Lambda Delta -> -inf makes
    Abar underflow to exactly 0 and g = -1/Lambda."""
    rng = np.random.default_rng(2)
    v = rng.normal(size=(2, 7, 3)) + 1j * rng.normal(size=(2, 7, 3))
    x = orc.scan(np.zeros(3, np.complex128), v, None, rng.normal(size=(2, 3)) + 0j)
    assert np.array_equal(x, v)
    inp = small_inputs(Bt=2, L=7, H=3, P=3, seed=2)
    Lambda = np.array([-50.0 + 1j, -80.0 - 2j, -60.0 + 0j])
    log_delta = np.full(3, 10.0)
    out = orc.forward(Lambda, inp["B"], inp["C"], inp["D"], log_delta, inp["u"])
    u = inp["u"].astype(np.float64)
    Bbar = (-1.0 / Lambda)[:, None] * inp["B"].astype(np.complex128)
    expect = np.real(np.einsum("op,pi,bli->blo", inp["C"].astype(np.complex128), Bbar, u)) \
        + inp["D"].astype(np.float64) * u
    np.testing.assert_allclose(out["y"], expect, rtol=1e-12, atol=1e-14)


# ------------------------------------------------------------------ resets and carries
def test_reset_makes_outputs_independent_of_the_prefix():
    inp = small_inputs(Bt=3, L=20, H=3, P=4, seed=7, with_x0=True)
    flags = np.zeros((3, 20), np.uint8)
    flags[0, 6] = flags[1, 11] = flags[2, 0] = 1
    a = orc.forward(inp["Lambda"], inp["B"], inp["C"], inp["D"], inp["log_delta"], inp["u"], flags,
                    inp["x0"])
    rng = np.random.default_rng(9)
    u2 = inp["u"].astype(np.float64).copy()
    u2[0, :6] = rng.normal(size=(6, 3))
    u2[1, :11] = rng.normal(size=(11, 3))
    x02 = rng.normal(size=(3, 4)) + 1j * rng.normal(size=(3, 4))
    b = orc.forward(inp["Lambda"], inp["B"], inp["C"], inp["D"], inp["log_delta"], u2, flags, x02)
    for bi, k in ((0, 6), (1, 11), (2, 0)):
        assert np.array_equal(a["y"][bi, k:], b["y"][bi, k:])      # bit-identical
        assert np.array_equal(a["x"][bi, k:], b["x"][bi, k:])
    assert not np.allclose(a["y"][0, :6], b["y"][0, :6])


def test_segments_between_resets_behave_as_separate_sequences():
    inp = small_inputs(Bt=1, L=30, H=3, P=4, seed=8)
    flags = np.zeros((1, 30), np.uint8)
    cuts = [0, 5, 6, 19]
    flags[0, cuts] = 1
    full = orc.forward(inp["Lambda"], inp["B"], inp["C"], inp["D"], inp["log_delta"], inp["u"], flags)
    for s, e in zip(cuts, cuts[1:] + [30]):
        seg = orc.forward(inp["Lambda"], inp["B"], inp["C"], inp["D"], inp["log_delta"],
                          inp["u"][:, s:e])
        np.testing.assert_allclose(full["y"][:, s:e], seg["y"], rtol=1e-13, atol=1e-15)
    # every step flagged: x_t = Bbar u_t (same as Abar = 0)
    ones = np.ones((1, 30), np.uint8)
    allr = orc.forward(inp["Lambda"], inp["B"], inp["C"], inp["D"], inp["log_delta"], inp["u"], ones)
    _, g = naive_discretize(inp["Lambda"], inp["log_delta"])
    v = np.einsum("ph,blh->blp", g[:, None] * inp["B"].astype(np.complex128),
                  inp["u"].astype(np.float64))
    np.testing.assert_allclose(allr["x"], v, rtol=1e-12, atol=1e-15)


def test_x0_carry_split_equals_one_run():
    inp = small_inputs(Bt=2, L=24, H=3, P=4, seed=4, p_reset=0.1, with_x0=True)
    args = (inp["Lambda"], inp["B"], inp["C"], inp["D"], inp["log_delta"])
    full = orc.forward(*args, inp["u"], inp["is_first"], inp["x0"])
    h1 = orc.forward(*args, inp["u"][:, :10], inp["is_first"][:, :10], inp["x0"])
    h2 = orc.forward(*args, inp["u"][:, 10:], inp["is_first"][:, 10:], h1["x_last"])
    np.testing.assert_allclose(np.concatenate([h1["y"], h2["y"]], 1), full["y"], rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(h2["x_last"], full["x_last"], rtol=1e-13, atol=1e-15)
    # x0 = None is the same as zeros, and a first-step flag makes x0 irrelevant
    z = orc.forward(*args, inp["u"], inp["is_first"], None)
    zz = orc.forward(*args, inp["u"], inp["is_first"], np.zeros((2, 4), np.complex128))
    assert np.array_equal(z["y"], zz["y"])
    fl = inp["is_first"].copy()
    fl[:, 0] = 1
    assert np.array_equal(orc.forward(*args, inp["u"], fl, inp["x0"])["y"],
                          orc.forward(*args, inp["u"], fl, None)["y"])


# ------------------------------------------------------------------ discretisation
def test_discretize_matches_textbook_form_and_limits():
    rng = np.random.default_rng(0)
    Lambda = -rng.uniform(0.1, 1, 64) + 1j * rng.uniform(0, np.pi, 64)
    log_delta = rng.uniform(math.log(1e-3), math.log(1e-1), 64)
    Abar, g = orc.discretize(Lambda, log_delta)
    Abar_n, g_n = naive_discretize(Lambda, log_delta)
    np.testing.assert_allclose(Abar, Abar_n, rtol=1e-15)
    np.testing.assert_allclose(g, g_n, rtol=1e-10)        # |z| >= 1e-4: naive form still fine
    # Euler limit Delta -> 0: Abar -> 1 + Lambda Delta, g -> Delta (first-order error)
    tiny = np.full(64, math.log(1e-7))
    Abar, g = orc.discretize(Lambda, tiny)
    np.testing.assert_allclose(Abar, 1 + Lambda * 1e-7, atol=1e-12)
    np.testing.assert_allclose(g, 1e-7 * (1 + Lambda * 1e-7 / 2), rtol=1e-12)
    # Lambda = 0 exactly: the z -> 0 limit, no division by zero
    Abar, g = orc.discretize(np.zeros(2), np.log([0.5, 2.0]))
    np.testing.assert_allclose(Abar, 1.0)
    np.testing.assert_allclose(g, [0.5, 2.0])


def test_zoh_against_scipy_and_exact_ode_solution():
    sig = pytest.importorskip("scipy.signal")
    lam = np.array([-0.3, -1.7, -0.05])
    dt = 0.07
    A = np.diag(lam)
    Bm = np.array([[1.0, 0.5], [-2.0, 0.3], [0.7, 0.7]])
    Ad, Bd, *_ = sig.cont2discrete((A, Bm, np.eye(3), np.zeros((3, 2))), dt, method="zoh")
    Abar, g = orc.discretize(lam + 0j, np.full(3, math.log(dt)))
    np.testing.assert_allclose(np.diag(Ad), Abar.real, rtol=1e-13)
    np.testing.assert_allclose(Bd, (g[:, None] * Bm).real, rtol=1e-12)
    assert np.max(np.abs(Abar.imag)) == 0 and np.max(np.abs(g.imag)) == 0
    # exact solution of dx/dt = lam x + B u for constant u from x(0)=0 at sample times (Eq. 2)
    ubar = np.array([0.4, -1.1])
    L = 25
    out = orc.forward(lam + 0j, Bm + 0j, np.eye(2, 3) + 0j, np.zeros(2), np.full(3, math.log(dt)),
                      np.broadcast_to(ubar, (1, L, 2)).copy())
    k = np.arange(1, L + 1)[:, None]
    exact = (np.exp(lam * k * dt) - 1) / lam * (Bm @ ubar)
    np.testing.assert_allclose(out["x"][0].real, exact, rtol=1e-11)


# ------------------------------------------------------------------ gradients
GRAD_KEYS = ("du", "dLambda", "dB", "dC", "dD", "dlog_delta", "dx0")


def _analytic(inp, dy):
    fwd = orc.forward(inp["Lambda"], inp["B"], inp["C"], inp["D"], inp["log_delta"], inp["u"],
                      inp["is_first"], inp["x0"])
    return orc.backward(inp["Lambda"], inp["B"], inp["C"], inp["D"], inp["log_delta"], inp["u"],
                        inp["is_first"], inp["x0"], fwd["x"], dy)


@pytest.mark.parametrize("case", ["reset_mid_x0", "no_reset_no_x0", "first_step_reset_x0"])
def test_analytic_gradients_match_brute_force_finite_differences(case):
    inp = small_inputs(Bt=2, L=5, H=3, P=2, seed=11, with_x0=(case != "no_reset_no_x0"))
    flags = np.zeros((2, 5), np.uint8)
    if case == "reset_mid_x0":
        flags[0, 2] = flags[1, 4] = 1
    elif case == "first_step_reset_x0":
        flags[:, 0] = 1
        flags[1, 3] = 1
    inp["is_first"] = None if case == "no_reset_no_x0" else flags
    dy = inp["dy"].astype(np.float64)
    ana = _analytic(inp, dy)
    fd = orc.fd_gradients(inp["Lambda"], inp["B"], inp["C"], inp["D"], inp["log_delta"], inp["u"],
                          inp["is_first"], inp["x0"], dy)
    for k in GRAD_KEYS:
        if k == "dx0" and inp["x0"] is None:
            continue
        scale = max(1.0, float(np.max(np.abs(fd[k]))))
        assert np.max(np.abs(ana[k] - fd[k])) <= 2e-7 * scale, k


def test_gradients_for_tiny_lambda_delta_use_the_stable_series():
    """|Lambda Delta| ~ 1e-6: the closed form of d g / d Lambda cancels; FD still pins it."""
    inp = small_inputs(Bt=1, L=6, H=2, P=2, seed=12)
    Lambda = np.array([-1e-3 + 2e-3j, -3e-3 + 0j])
    log_delta = np.log([1e-3, 2e-3])
    dy = inp["dy"].astype(np.float64)
    fwd = orc.forward(Lambda, inp["B"], inp["C"], inp["D"], log_delta, inp["u"])
    ana = orc.backward(Lambda, inp["B"], inp["C"], inp["D"], log_delta, inp["u"], None, None,
                       fwd["x"], dy)
    fd = orc.fd_gradients(Lambda, inp["B"], inp["C"], inp["D"], log_delta, inp["u"], None, None, dy,
                          eps=1e-4)
    for k in ("dLambda", "dlog_delta", "dB"):
        scale = max(1e-12, float(np.max(np.abs(fd[k]))))
        assert np.max(np.abs(ana[k] - fd[k])) <= 1e-6 * scale, k
    # moderately small z where both the series and the closed form are accurate:
    # d g/d Lambda by central difference of the oracle's own discretisation
    lam, ld = np.array([-0.3 + 0.4j]), np.array([math.log(0.9)])   # |z| = 0.45 (series side)
    lam2 = np.array([-0.5 + 0.5j])                                  # |z| = 0.64 (closed form)
    for lm in (lam, lam2):
        eps = 1e-6
        num = (orc.discretize(lm + eps, ld)[1] - orc.discretize(lm - eps, ld)[1]) / (2 * eps)
        # choose B, C, u so that l = Re(g): one state, H = 1, L = 1
        fwd = orc.forward(lm, np.ones((1, 1)), np.ones((1, 1)), np.zeros(1), ld, np.ones((1, 1, 1)))
        ana = orc.backward(lm, np.ones((1, 1)), np.ones((1, 1)), np.zeros(1), ld, np.ones((1, 1, 1)),
                           None, None, fwd["x"], np.ones((1, 1, 1)))
        np.testing.assert_allclose(ana["dLambda"], np.conj(num), rtol=1e-8)


def test_directional_finite_difference_at_medium_size():
    w = wl.custom("m", 3, 48, 24, 20, p_reset=0.05, force_first=False, with_x0=True, seed=21)
    inp = wl.gen_inputs(w)
    dy = inp["dy"].astype(np.float64)
    ana = _analytic(inp, dy)
    rng = np.random.default_rng(5)
    direction, inner = {}, 0.0
    for k, gk in (("Lambda", "dLambda"), ("B", "dB"), ("C", "dC"), ("D", "dD"),
                  ("log_delta", "dlog_delta"), ("u", "du"), ("x0", "dx0")):
        shape = np.shape(inp[k])
        if np.iscomplexobj(inp[k]):
            d = rng.normal(size=shape) + 1j * rng.normal(size=shape)
            inner += float(np.sum(ana[gk].real * d.real + ana[gk].imag * d.imag))
        else:
            d = rng.normal(size=shape)
            inner += float(np.sum(ana[gk] * d))
        direction[k] = d
    fd = orc.fd_directional(inp, direction, dy, eps=1e-6)
    assert abs(fd - inner) <= 1e-7 * max(1.0, abs(inner))


def test_adjoint_identity_and_no_gradient_leak_across_a_reset():
    inp = small_inputs(Bt=2, L=16, H=4, P=5, seed=13)
    flags = np.zeros((2, 16), np.uint8)
    flags[:, 9] = 1
    args = (inp["Lambda"], inp["B"], inp["C"], inp["D"], inp["log_delta"])
    dy = inp["dy"].astype(np.float64)
    inp["is_first"] = flags
    ana = _analytic(inp, dy)
    # y is linear in u for x0 = 0: <dy, y(u')> = <du, u'>
    rng = np.random.default_rng(3)
    up = rng.normal(size=(2, 16, 4))
    yp = orc.forward(*args, up, flags)["y"]
    assert abs(np.sum(dy * yp) - np.sum(ana["du"] * up)) <= 1e-11 * abs(np.sum(dy * yp))
    # changing dy at/after the reset must not change du before it
    dy2 = dy.copy()
    dy2[:, 9:] = rng.normal(size=(2, 7, 4))
    ana2 = _analytic(inp, dy2)
    assert np.array_equal(ana["du"][:, :9], ana2["du"][:, :9])
    assert not np.allclose(ana["du"][:, 9:], ana2["du"][:, 9:])


def test_threads_only_distribute_sequences():
    w = wl.custom("thr", 6, 20, 8, 8, p_reset=0.1, with_x0=True, seed=2)
    inp = wl.gen_inputs(w)
    a = orc.run_workload(inp, True, nthreads=1)
    b = orc.run_workload(inp, True, nthreads=4)
    assert np.array_equal(a["y"], b["y"]) and np.array_equal(a["du"], b["du"])
    for k in ("dLambda", "dB", "dC", "dD", "dlog_delta"):
        np.testing.assert_allclose(a[k], b[k], rtol=1e-12, atol=1e-14)


def test_workload_generator_shapes_and_recipe():
    for w in wl.CONFIGS:
        if w.tokens * w.H > 1 << 22:
            continue
        inp = wl.gen_inputs(w)
        assert inp["u"].shape == (w.Bt, w.L, w.H) and inp["u"].dtype == np.float32
        assert inp["Lambda"].dtype == np.complex64 and inp["Lambda"].shape == (w.P,)
        assert np.all(inp["Lambda"].real < 0) and np.all(inp["Lambda"].imag >= 0)
        assert (inp["is_first"] is None) == (w.p_reset == 0 and not w.force_first)
        if w.force_first:
            assert np.all(inp["is_first"][:, 0] == 1)
        assert (inp["x0"] is not None) == w.with_x0
    a, b = wl.gen_inputs(wl.CONFIGS[1]), wl.gen_inputs(wl.CONFIGS[1])
    assert all(np.array_equal(a[k], b[k]) for k in a if a[k] is not None)
