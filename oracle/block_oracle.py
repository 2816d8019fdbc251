"""Float64 CPU oracle of the two operations around the SSM layer: the bootstrapped lambda-return
of the actor-critic section and the half-GLU gate of the S5 sequence layer (appendix).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's
CPU-baseline leg.  Nothing here imports, links or calls the HIP library, and the HIP package
never imports this module.  Plain numpy, float64, the definitions written out step by step.
"""
from __future__ import annotations

import math

import numpy as np


# ------------------------------------------------------------------------------------------------
# lambda-return (actor-critic section, the critic's target):
#     V_t = r_t + gamma c_t ((1 - lambda) v_t + lambda V_{t+1}),      V_T = v_T
# Arrays are time-major, [T, N]: row t holds step t of N imagined trajectories; row T-1 is the
# paper's last step T, whose return is the critic's value itself.
# ------------------------------------------------------------------------------------------------
def lambda_return(reward, cont, value, gamma: float, lam: float):
    r = np.asarray(reward, dtype=np.float64)
    c = np.asarray(cont, dtype=np.float64)
    v = np.asarray(value, dtype=np.float64)
    T = r.shape[0]
    ret = np.empty_like(v)
    ret[T - 1] = v[T - 1]
    for t in range(T - 2, -1, -1):
        ret[t] = r[t] + gamma * c[t] * ((1.0 - lam) * v[t] + lam * ret[t + 1])
    return ret


def lambda_return_grad(reward, cont, value, gamma: float, lam: float, dret):
    """Gradients of sum(dret * V) with respect to reward, cont and value (same shapes).

    Chain rule over the definition: G_t, the total derivative with respect to V_t, collects dret_t
    and what flows back from V_{t-1} through the factor gamma c_{t-1} lambda.
    """
    r = np.asarray(reward, dtype=np.float64)
    c = np.asarray(cont, dtype=np.float64)
    v = np.asarray(value, dtype=np.float64)
    g = np.asarray(dret, dtype=np.float64)
    T = r.shape[0]
    ret = lambda_return(r, c, v, gamma, lam)
    dr, dc, dv = np.zeros_like(r), np.zeros_like(c), np.zeros_like(v)
    G = np.zeros_like(g[0])
    for t in range(T):
        G = g[t] + (gamma * c[t - 1] * lam * G if t > 0 else 0.0)
        if t < T - 1:
            dr[t] = G
            dc[t] = G * gamma * ((1.0 - lam) * v[t] + lam * ret[t + 1])
            dv[t] = G * gamma * c[t] * (1.0 - lam)
        else:
            dv[t] = G
    return dr, dc, dv


# ------------------------------------------------------------------------------------------------
# half-GLU (S5 sequence layer appendix):   x1 = GELU(u),   y = u * sigmoid(W^T x1)
# u: [T, H] rows of features, W: [H, H] weights of a linear layer applied to the feature axis:
# (W^T x1)_j = sum_i W[i, j] x1_i.  GELU is the exact Gaussian one, x * Phi(x).
# ------------------------------------------------------------------------------------------------
_erfc = np.vectorize(math.erfc, otypes=[np.float64])


def _normal_cdf(x):
    # Phi(x) = erfc(-x / sqrt 2) / 2: no cancellation in the lower tail
    return 0.5 * _erfc(-x / math.sqrt(2.0))


def gelu(x):
    x = np.asarray(x, dtype=np.float64)
    return x * _normal_cdf(x)


def gelu_grad(x):
    x = np.asarray(x, dtype=np.float64)
    cdf = _normal_cdf(x)
    pdf = np.exp(-0.5 * x * x) / math.sqrt(2.0 * math.pi)
    return cdf + x * pdf


def sigmoid(z):
    z = np.asarray(z, dtype=np.float64)
    out = np.empty_like(z)
    pos = z >= 0
    out[pos] = 1.0 / (1.0 + np.exp(-z[pos]))
    e = np.exp(z[~pos])
    out[~pos] = e / (1.0 + e)
    return out


def half_glu(u, W):
    u = np.asarray(u, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    x1 = gelu(u)
    z = x1 @ W                       # z[t, j] = sum_i x1[t, i] W[i, j]
    return u * sigmoid(z)


def half_glu_grad(u, W, dy):
    """Gradients of sum(dy * y) with respect to u and W."""
    u = np.asarray(u, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    dy = np.asarray(dy, dtype=np.float64)
    x1 = gelu(u)
    z = x1 @ W
    s = sigmoid(z)
    dz = dy * u * s * (1.0 - s)
    dx1 = dz @ W.T
    du = dy * s + dx1 * gelu_grad(u)
    dW = x1.T @ dz
    return du, dW
