"""Host logic that decides what a call launches (no GPU needed): which shapes scan inside the projections,
how many planes, tile tiers, K slabs of the reductions and which work items go first.  The decisions are
read back through ssm_plan_describe (include/ssm_measure.h); the expectations are the rules the design
states, evaluated here independently in Python for the scheduling model."""
import heapq

import pytest

from paper_2502_20168_amd import binding as ssm
from paper_2502_20168_amd import workloads as wl


def test_benchmark_configurations_take_the_paths_the_design_states():
    plans = [ssm.ssm_plan_describe(w.Bt, w.L, w.H, w.P) for w in wl.CONFIGS]
    assert [p["scans_in_projections"] for p in plans] == [0, 0, 1, 1, 1]
    assert [p["planes"] for p in plans] == [3, 3, 2, 2, 2]
    assert [p["products_per_gradient_launch"] for p in plans] == [2, 2, 3, 3, 3]
    # the benchmark shape: eight slabs per reduction behind du, the output projection on 64x128 tiles
    assert plans[2]["slabs_dC"] == 8 and plans[2]["slabs_dBbar"] == 8 and plans[2]["slabs_first"] == 0
    assert plans[2]["tier_out"] == 1 and plans[2]["tier_in"] == 0
    # 1024 x 16 tokens: few long slab items, dispatched first
    assert plans[4]["slabs_dC"] == 4 and plans[4]["slabs_first"] == 1
    # the small configurations run everything on 64x64x64 tiles
    assert plans[0]["tier_in"] == 2 and plans[0]["tier_out"] == 2 and plans[1]["tier_in"] == 2


def _tier(M, N):
    r = lambda bm, bn: -(-(-(-M // bm) * -(-N // bn)) // 256)
    c0, c1, c2 = 10 * r(128, 128), 10 * r(64, 128), 6 * r(64, 64)
    if c2 < c0 and c2 < c1:
        return 2
    return 1 if c1 <= c0 else 0


@pytest.mark.parametrize("Bt,L,H,P", [(30, 100, 512, 512), (64, 100, 512, 512), (18, 100, 1024, 512), (8, 100, 256, 256),
                                      (16, 1000, 256, 256), (5, 77, 96, 40), (100, 100, 256, 128)])
def test_tile_tier_is_rounds_of_workgroups_times_time_per_k_step(Bt, L, H, P):
    p = ssm.ssm_plan_describe(Bt, L, H, P)
    assert p["scans_in_projections"] == 0
    assert p["tier_in"] == _tier(Bt * L, 2 * P) and p["tier_out"] == _tier(Bt * L, H)


def test_192_tiles_of_128_take_one_round_of_large_tiles():
    # 3000 tokens x 1024 columns: 192 tiles of 128x128 (one round) against 376 of 64x128 (two rounds)
    assert ssm.ssm_plan_describe(30, 100, 512, 512)["tier_in"] == 0


def _makespan(first, second):
    """List scheduling of (count, length) items on 256 machines in the given order."""
    h = [0] * 256
    heapq.heapify(h)
    for n, ln in (first, second):
        for _ in range(n):
            heapq.heappush(h, heapq.heappop(h) + ln)
    return max(h)


def _model(T, main_tiles, k_main, red_tiles, split_bytes):
    a = -(-k_main // 32)
    per = 0.2 + 0.6 * split_bytes / (2 << 20)
    best = None
    for sp in (1, 2, 3, 4, 5, 6, 8, 10, 12, 16, 24, 32, 48, 64):
        if sp > 1 and sp > T // 256:
            break
        b = -(-(-(-T // sp)) // 32)
        m_main, m_red = _makespan((main_tiles, a), (red_tiles * sp, b)), _makespan((red_tiles * sp, b), (main_tiles, a))
        cost = min(m_main, m_red) + per * sp
        if best is None or cost < best[0]:
            best = (cost, sp, m_red < m_main, b >= 2 * a)
    return best


@pytest.mark.parametrize("Bt,L,H,P", [(16, 256, 512, 512), (4, 4096, 256, 256), (1024, 16, 512, 512), (32, 128, 1024, 512),
                                      (256, 64, 256, 256), (8, 1024, 512, 512)])
def test_slabs_of_the_three_product_launch_follow_the_schedule_model(Bt, L, H, P):
    T = Bt * L
    p = ssm.ssm_plan_describe(Bt, L, H, P)
    assert p["products_per_gradient_launch"] == 3
    c = lambda x, y: -(-x // y)
    _, sp, _, twice = _model(T, c(T, 128) * c(H, 128), 2 * P, 2 * c(2 * P, 128) * c(H, 128), 2 * 2 * P * H * 4)
    assert p["slabs_dC"] == sp and p["slabs_dBbar"] == sp
    assert p["slabs_first"] == int(twice)


@pytest.mark.parametrize("Bt,L,H,P", [(64, 100, 512, 512), (16, 1000, 256, 256), (24, 200, 1024, 512), (20, 300, 512, 256),
                                      (10, 1000, 512, 512)])
def test_slabs_and_order_of_the_two_product_launches_follow_the_schedule_model(Bt, L, H, P):
    T = Bt * L
    p = ssm.ssm_plan_describe(Bt, L, H, P)
    assert p["products_per_gradient_launch"] == 2 and p["scans_in_projections"] == 0
    c = lambda x, y: -(-x // y)
    red = c(H, 128) * c(2 * P, 128)
    _, spC, firstC, _ = _model(T, c(T, 128) * c(2 * P, 128), H, red, H * 2 * P * 4)
    assert p["slabs_dC"] == spC and p["dC_first"] == int(firstC)
    halves = p["du_as_two_k_halves"]
    _, spB, firstB, _ = _model(T, c(T, 128) * c(H, 128) * (2 if halves else 1), P if halves else 2 * P, red, H * 2 * P * 4)
    assert p["slabs_dBbar"] == spB and p["dBbar_first"] == int(bool(halves) or firstB)


def test_every_plan_is_bounded_and_repeatable():
    import numpy as np
    rng = np.random.Generator(np.random.PCG64(123))
    for _ in range(300):
        Bt, L = int(rng.integers(1, 600)), int(rng.choice([1, 16, 64, 100, 128, 256, 300, 1000, 4096]))
        H, P = int(rng.choice([3, 32, 96, 256, 512, 1024])), int(rng.choice([1, 40, 128, 256, 512]))
        a, b = ssm.ssm_plan_describe(Bt, L, H, P), ssm.ssm_plan_describe(Bt, L, H, P)
        assert a == b
        for k in ("slabs_dC", "slabs_dBbar"):
            assert 1 <= a[k] <= 64 and (a[k] == 1 or -(-Bt * L // a[k]) >= 64)       # a slab keeps at least one K step of 64
        assert a["planes"] in (2, 3) and a["tier_in"] in (0, 1, 2) and a["tier_out"] in (0, 1, 2)
        assert ssm.ssm_workspace_bytes(Bt, L, H, P, True) > 0 and ssm.ssm_workspace_bytes(Bt, L, H, P, False) > 0


def test_plan_rejects_what_the_library_rejects():
    with pytest.raises(ssm.SsmError):
        ssm.ssm_plan_describe(0, 16, 8, 8)
    with pytest.raises(ssm.SsmError):
        ssm.ssm_plan_describe(1, 16, 1 << 20, 8)


def test_the_binding_loads_torch_before_the_library():
    """A host-only call (no GPU work) must not bind the library to the system's copy of the HIP runtime: torch
    brings its own, and with two copies in the process every later launch on torch's memory fails.  In a fresh
    interpreter, a plan query before any `import torch` leaves torch loaded first."""
    import os, subprocess, sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    code = ("import sys; sys.path.insert(0, %r)\n"
            "from paper_2502_20168_amd import binding as ssm\n"
            "assert 'torch' not in sys.modules\n"
            "print(ssm.ssm_plan_describe(16, 256, 512, 512)['planes'])\n"
            "assert 'torch' in sys.modules\n" % root)
    out = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=300)
    assert out.returncode == 0, out.stderr
    assert out.stdout.strip().splitlines()[-1] == "2"
