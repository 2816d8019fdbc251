"""Seeded synthetic workloads for the resettable S5 scan layer.

This module only draws random numbers and shapes them; it contains none of the
method's arithmetic (no discretisation, no recurrence, no projections), so the
HIP path and the CPU oracle can both be fed from it without sharing any
computation.  The arrays stand in for the paper's replay windows (batch x length
windows of fused latent/action features with episode boundaries; hyper-parameter
tables of the state-based and vision tasks give width 512/1024 and state size
256/512), which need a simulator and trained encoders that are not available.

Draw order is fixed (Lambda_re, Lambda_im, B_re, B_im, C_re, C_im, D, log_delta,
u, is_first, dy, x0_re, x0_im) from numpy's PCG64 in float64, then every array is
rounded once to fp32 / complex64.  Both sides consume the rounded values.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, Optional

import numpy as np


@dataclasses.dataclass(frozen=True)
class Workload:
    """Shape and distribution recipe for one batch of sequences."""

    name: str
    Bt: int                 # sequences in the batch
    L: int                  # steps per sequence
    H: int                  # width of u and y
    P: int                  # number of complex diagonal states
    backward: bool          # does the config exercise the gradient pass
    p_reset: float          # Bernoulli probability of is_first at each step
    force_first: bool       # is_first[:, 0] = 1
    with_x0: bool           # supply an initial state per sequence
    lam_re_lo: float = 0.1  # Re(Lambda) = -U(lam_re_lo, lam_re_hi)
    lam_re_hi: float = 1.0
    seed: int = 0

    @property
    def tokens(self) -> int:
        return self.Bt * self.L


# The five benchmark configurations (0-indexed).  Config 2 is the headline one.
CONFIGS = (
    Workload("cfg0_tiny_fwd", Bt=2, L=64, H=32, P=32, backward=False,
             p_reset=0.0, force_first=False, with_x0=False),
    Workload("cfg1_small_fwdbwd", Bt=16, L=64, H=256, P=256, backward=True,
             p_reset=0.02, force_first=True, with_x0=False),
    Workload("cfg2_worldmodel_fwdbwd", Bt=16, L=256, H=512, P=512, backward=True,
             p_reset=0.01, force_first=True, with_x0=False),
    Workload("cfg3_longseq_fwdbwd", Bt=4, L=4096, H=256, P=256, backward=True,
             p_reset=0.001, force_first=True, with_x0=False,
             lam_re_lo=0.001, lam_re_hi=0.1),
    Workload("cfg4_imagination_fwd", Bt=1024, L=16, H=512, P=512, backward=False,
             p_reset=0.0, force_first=False, with_x0=True),
)


def gen_inputs(w: Workload, seed: Optional[int] = None) -> Dict[str, Optional[np.ndarray]]:
    """Draw one batch for workload `w`.

    Returns a dict with keys Lambda [P] c64, B [P,H] c64, C [H,P] c64, D [H] f32,
    log_delta [P] f32, u [Bt,L,H] f32, is_first [Bt,L] u8 (or None when the
    workload has no resets at all), dy [Bt,L,H] f32, x0 [Bt,P] c64 or None.
    """
    rng = np.random.Generator(np.random.PCG64(w.seed if seed is None else seed))
    Bt, L, H, P = w.Bt, w.L, w.H, w.P
    lam_re = -rng.uniform(w.lam_re_lo, w.lam_re_hi, size=P)
    lam_im = rng.uniform(0.0, math.pi, size=P)
    std = 1.0 / math.sqrt(H)
    B_re = rng.normal(0.0, std, size=(P, H))
    B_im = rng.normal(0.0, std, size=(P, H))
    C_re = rng.normal(0.0, std, size=(H, P))
    C_im = rng.normal(0.0, std, size=(H, P))
    D = rng.normal(0.0, 1.0, size=H)
    log_delta = rng.uniform(math.log(1e-3), math.log(1e-1), size=P)
    u = rng.normal(0.0, 1.0, size=(Bt, L, H))
    flags = rng.random(size=(Bt, L)) < w.p_reset
    dy = rng.normal(0.0, 1.0, size=(Bt, L, H))
    x0_re = rng.normal(0.0, 1.0, size=(Bt, P))
    x0_im = rng.normal(0.0, 1.0, size=(Bt, P))

    is_first = flags.astype(np.uint8)
    if w.force_first:
        is_first[:, 0] = 1
    has_flags = w.p_reset > 0.0 or w.force_first
    return {
        "Lambda": (lam_re + 1j * lam_im).astype(np.complex64),
        "B": (B_re + 1j * B_im).astype(np.complex64),
        "C": (C_re + 1j * C_im).astype(np.complex64),
        "D": D.astype(np.float32),
        "log_delta": log_delta.astype(np.float32),
        "u": u.astype(np.float32),
        "is_first": is_first if has_flags else None,
        "dy": dy.astype(np.float32),
        "x0": (x0_re + 1j * x0_im).astype(np.complex64) if w.with_x0 else None,
    }


def custom(name: str, Bt: int, L: int, H: int, P: int, *, backward: bool = True,
           p_reset: float = 0.0, force_first: bool = False, with_x0: bool = False,
           lam_re_lo: float = 0.1, lam_re_hi: float = 1.0, seed: int = 0) -> Workload:
    """Ad-hoc workload for edge-case tests (ragged sizes, all-reset, ...)."""
    return Workload(name, Bt, L, H, P, backward, p_reset, force_first, with_x0,
                    lam_re_lo, lam_re_hi, seed)


def gen_returns(T: int, N: int, seed: int = 0, p_end: float = 0.05) -> Dict[str, np.ndarray]:
    """Seeded synthetic imagination roll-out for the lambda-return, time-major [T, N] float32:
    rewards and critic values ~ N(0,1); continuation flags sampled in {0, 1} with
    P(episode end) = p_end for the even trajectories and continuous probabilities U(0,1) for
    the odd ones; dret ~ N(0,1).  Draw order: reward, cont_binary, cont_prob, value, dret."""
    rng = np.random.Generator(np.random.PCG64(seed))
    reward = rng.normal(size=(T, N))
    cb = (rng.random(size=(T, N)) >= p_end).astype(np.float64)
    cp = rng.random(size=(T, N))
    cont = np.where((np.arange(N) % 2 == 0)[None, :], cb, cp)
    value = rng.normal(size=(T, N))
    dret = rng.normal(size=(T, N))
    f = lambda a: np.ascontiguousarray(a, dtype=np.float32)
    return {"reward": f(reward), "cont": f(cont), "value": f(value), "dret": f(dret)}


def gen_half_glu(T: int, H: int, seed: int = 0) -> Dict[str, np.ndarray]:
    """Seeded synthetic input of the half-GLU gate: u, dy ~ N(0,1) [T, H]; W ~ N(0, 1/sqrt(H))
    [H, H] (the scale of a freshly initialised linear layer).  Draw order: u, W, dy."""
    rng = np.random.Generator(np.random.PCG64(seed))
    u = rng.normal(size=(T, H))
    W = rng.normal(size=(H, H)) / np.sqrt(H)
    dy = rng.normal(size=(T, H))
    f = lambda a: np.ascontiguousarray(a, dtype=np.float32)
    return {"u": f(u), "W": f(W), "dy": f(dy)}
