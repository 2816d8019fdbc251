"""Pins of the float64 oracle for the lambda-return (actor-critic section) and the half-GLU gate
(S5 sequence layer appendix) against closed forms, library routines, brute force and finite
differences.  None of these tests touches the GPU."""
import math

import numpy as np
import pytest
from scipy import special, stats

from oracle import block_oracle as orc


def _rand(T, N, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    r = rng.normal(size=(T, N))
    c = rng.uniform(0.0, 1.0, size=(T, N))
    v = rng.normal(size=(T, N))
    return rng, r, c, v


# ------------------------------------------------------------------------------------ lambda-return
def test_last_step_is_the_critic_value():
    _, r, c, v = _rand(7, 3, 0)
    ret = orc.lambda_return(r, c, v, 0.97, 0.9)
    assert np.array_equal(ret[-1], v[-1])


def test_lambda_zero_is_the_one_step_target():
    _, r, c, v = _rand(9, 4, 1)
    ret = orc.lambda_return(r, c, v, 0.95, 0.0)
    np.testing.assert_allclose(ret[:-1], r[:-1] + 0.95 * c[:-1] * v[:-1], rtol=1e-14)


def test_lambda_one_is_the_discounted_sum_with_bootstrap():
    # c = 1: V_t = sum_k gamma^k r_{t+k} + gamma^(T-1-t) v_{T-1}; evaluated with numpy's polynomial routine
    _, r, _, v = _rand(12, 2, 2)
    c = np.ones_like(r)
    gamma = 0.9
    ret = orc.lambda_return(r, c, v, gamma, 1.0)
    for n in range(r.shape[1]):
        for t in range(r.shape[0]):
            coef = list(r[t:-1, n]) + [v[-1, n]]
            assert ret[t, n] == pytest.approx(np.polynomial.polynomial.polyval(gamma, coef), rel=1e-13)


def test_unrolled_sum():
    # V_t = sum_k (prod_{j<k} gamma lambda c_{t+j}) (r_{t+k} + gamma c_{t+k} (1-lambda) v_{t+k})
    #       + (prod over all remaining steps) v_{T-1}
    _, r, c, v = _rand(10, 3, 3)
    gamma, lam = 0.93, 0.8
    ret = orc.lambda_return(r, c, v, gamma, lam)
    T, N = r.shape
    for n in range(N):
        for t in range(T):
            total, prod = 0.0, 1.0
            for k in range(t, T - 1):
                total += prod * (r[k, n] + gamma * c[k, n] * (1 - lam) * v[k, n])
                prod *= gamma * lam * c[k, n]
            total += prod * v[T - 1, n]
            assert ret[t, n] == pytest.approx(total, rel=1e-12, abs=1e-13)


def test_mixture_of_n_step_returns():
    # textbook form of the lambda-return with this paper's indices (the n-step return bootstraps
    # with v_{t+n-1}, the complete one with v_{T-1}):
    #   V_t = (1-lambda) sum_{n=1..N} lambda^(n-1) G_n + lambda^N G_full,   N = T-1-t
    _, r, _, v = _rand(11, 2, 4)
    c = np.ones_like(r)
    gamma, lam = 0.9, 0.7
    ret = orc.lambda_return(r, c, v, gamma, lam)
    T, Nb = r.shape
    for b in range(Nb):
        for t in range(T - 1):
            N = T - 1 - t
            disc = lambda n: sum(gamma ** k * r[t + k, b] for k in range(n))
            mix = sum((1 - lam) * lam ** (n - 1) * (disc(n) + gamma ** n * v[t + n - 1, b]) for n in range(1, N + 1))
            mix += lam ** N * (disc(N) + gamma ** N * v[T - 1, b])
            assert ret[t, b] == pytest.approx(mix, rel=1e-12, abs=1e-13)


def test_constant_inputs_closed_form():
    T, gamma, lam, r0, v0 = 15, 0.99, 0.95, 0.3, 2.0
    r = np.full((T, 1), r0); c = np.ones((T, 1)); v = np.full((T, 1), v0)
    ret = orc.lambda_return(r, c, v, gamma, lam)
    a, b = r0 + gamma * (1 - lam) * v0, gamma * lam
    for t in range(T):
        n = T - 1 - t
        assert ret[t, 0] == pytest.approx(a * (1 - b ** n) / (1 - b) + b ** n * v0, rel=1e-13)


def test_episode_end_cuts_the_return():
    rng, r, c, v = _rand(10, 3, 5)
    k = 4
    c[k] = 0.0
    ret = orc.lambda_return(r, c, v, 0.97, 0.9)
    np.testing.assert_array_equal(ret[k], r[k])
    r2, c2, v2 = r.copy(), c.copy(), v.copy()
    r2[k + 1:] = rng.normal(size=r2[k + 1:].shape)
    c2[k + 1:] = rng.uniform(size=c2[k + 1:].shape)
    v2[k:] = rng.normal(size=v2[k:].shape)
    ret2 = orc.lambda_return(r2, c2, v2, 0.97, 0.9)
    np.testing.assert_array_equal(ret[:k + 1], ret2[:k + 1])


def test_lambda_return_gradient_against_central_differences():
    rng, r, c, v = _rand(6, 2, 6)
    g = rng.normal(size=r.shape)
    gamma, lam = 0.96, 0.85
    dr, dc, dv = orc.lambda_return_grad(r, c, v, gamma, lam, g)
    loss = lambda rr, cc, vv: float(np.sum(g * orc.lambda_return(rr, cc, vv, gamma, lam)))
    eps = 1e-6
    for arr, grad, idx in ((r, dr, 0), (c, dc, 1), (v, dv, 2)):
        for pos in np.ndindex(arr.shape):
            args_p = [r.copy(), c.copy(), v.copy()]
            args_m = [r.copy(), c.copy(), v.copy()]
            args_p[idx][pos] += eps
            args_m[idx][pos] -= eps
            fd = (loss(*args_p) - loss(*args_m)) / (2 * eps)
            assert grad[pos] == pytest.approx(fd, rel=1e-7, abs=1e-8)


def test_last_step_reward_and_continue_have_no_gradient():
    rng, r, c, v = _rand(5, 3, 7)
    dr, dc, _ = orc.lambda_return_grad(r, c, v, 0.9, 0.9, rng.normal(size=r.shape))
    assert not dr[-1].any() and not dc[-1].any()


# ------------------------------------------------------------------------------------ half-GLU
def test_gelu_is_x_times_the_normal_cdf():
    x = np.linspace(-6, 6, 241)
    np.testing.assert_allclose(orc.gelu(x), x * stats.norm.cdf(x), rtol=1e-13, atol=1e-300)
    assert orc.gelu(np.array([0.0]))[0] == 0.0
    assert orc.gelu(np.array([1.0]))[0] == pytest.approx(0.8413447460685429, rel=1e-15)
    assert orc.gelu(np.array([-1.0]))[0] == pytest.approx(-0.15865525393145707, rel=1e-14)


def test_gelu_derivative_against_central_differences():
    x = np.linspace(-4, 4, 33)
    eps = 1e-6
    fd = (orc.gelu(x + eps) - orc.gelu(x - eps)) / (2 * eps)
    np.testing.assert_allclose(orc.gelu_grad(x), fd, rtol=1e-8, atol=1e-9)


def test_sigmoid_against_library_and_symmetry():
    z = np.array([-800.0, -30.0, -1.0, 0.0, 1.0, 30.0, 800.0])
    np.testing.assert_allclose(orc.sigmoid(z), special.expit(z), rtol=1e-15)
    np.testing.assert_allclose(orc.sigmoid(z) + orc.sigmoid(-z), 1.0, rtol=1e-15)
    assert orc.sigmoid(np.array([0.0]))[0] == 0.5


def test_zero_weights_halve_the_input():
    rng = np.random.Generator(np.random.PCG64(8))
    u = rng.normal(size=(5, 7))
    np.testing.assert_array_equal(orc.half_glu(u, np.zeros((7, 7))), 0.5 * u)


def test_weight_orientation_single_entry():
    # only W[i, j] != 0: output channel j is gated by input channel i, every other channel by 1/2
    rng = np.random.Generator(np.random.PCG64(9))
    H, i, j, w = 6, 1, 4, 1.7
    u = rng.normal(size=(3, H))
    W = np.zeros((H, H)); W[i, j] = w
    y = orc.half_glu(u, W)
    for t in range(u.shape[0]):
        gi = u[t, i] * stats.norm.cdf(u[t, i])
        for h in range(H):
            want = u[t, h] * (special.expit(w * gi) if h == j else 0.5)
            assert y[t, h] == pytest.approx(want, rel=1e-14)


def test_half_glu_elementwise_definition():
    rng = np.random.Generator(np.random.PCG64(10))
    T, H = 4, 5
    u, W = rng.normal(size=(T, H)), rng.normal(size=(H, H))
    y = orc.half_glu(u, W)
    for t in range(T):
        x1 = [u[t, i] * 0.5 * (1 + math.erf(u[t, i] / math.sqrt(2))) for i in range(H)]
        for j in range(H):
            z = sum(W[i, j] * x1[i] for i in range(H))
            assert y[t, j] == pytest.approx(u[t, j] / (1 + math.exp(-z)), rel=1e-13)


def test_half_glu_gradient_against_central_differences():
    rng = np.random.Generator(np.random.PCG64(11))
    T, H = 3, 4
    u, W, dy = rng.normal(size=(T, H)), rng.normal(size=(H, H)), rng.normal(size=(T, H))
    du, dW = orc.half_glu_grad(u, W, dy)
    loss = lambda uu, ww: float(np.sum(dy * orc.half_glu(uu, ww)))
    eps = 1e-6
    for pos in np.ndindex(u.shape):
        up, um = u.copy(), u.copy(); up[pos] += eps; um[pos] -= eps
        assert du[pos] == pytest.approx((loss(up, W) - loss(um, W)) / (2 * eps), rel=1e-7, abs=1e-9)
    for pos in np.ndindex(W.shape):
        wp, wm = W.copy(), W.copy(); wp[pos] += eps; wm[pos] -= eps
        assert dW[pos] == pytest.approx((loss(u, wp) - loss(u, wm)) / (2 * eps), rel=1e-7, abs=1e-9)


def test_saturated_gate():
    u = np.array([[3.0, -2.0]])
    W = np.array([[500.0, -500.0], [0.0, 0.0]])
    y = orc.half_glu(u, W)          # z = (500 gelu(3), -500 gelu(3)): gate -> (1, 0)
    assert y[0, 0] == pytest.approx(3.0, rel=1e-15) and abs(y[0, 1]) < 1e-300
