"""GPU parity: the HIP path, called through the C ABI, against the float64 oracle on the same
seeded inputs -- the five benchmark configurations at full size and the edge cases."""
import numpy as np
import pytest

from oracle import ssm_oracle as orc
from paper_2502_20168_amd import binding as ssm
from paper_2502_20168_amd import workloads as wl
from tests.parity_util import (GRAD_KEYS, TOL_FWD, TOL_GRAD, assert_close, assert_close_elementwise, check_workload,
                               run_gpu)

pytestmark = pytest.mark.gpu
FWD_KEYS_ALL = ("y", "x", "x_last") + GRAD_KEYS


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    ssm.lib()


@pytest.mark.parametrize("idx", [0, 1, 2, 3, 4])
def test_benchmark_config_matches_oracle(idx):
    w = wl.CONFIGS[idx]
    print("config", idx, w, flush=True)
    rep = check_workload(w, backward=True if idx in (1, 2, 3) else False)
    print({k: "/".join("%.1e" % e for e in v) for k, v in rep.items()}, flush=True)


@pytest.mark.parametrize("idx", [0, 4])
def test_forward_only_configs_also_pass_the_gradient_check(idx):
    """Configs 0 and 4 are forward-only workloads; the gradient pass must still be right on
    their shapes (config 4 is cut to 64 sequences to keep the oracle quick)."""
    w = wl.CONFIGS[idx]
    if idx == 4:
        w = wl.custom("cfg4_cut", 64, 16, 512, 512, with_x0=True)
    check_workload(w, backward=True)


EDGE = [
    # name, Bt, L, H, P, p_reset, force_first, with_x0
    ("L1", 3, 1, 8, 8, 0.0, False, True),
    ("L1_reset", 3, 1, 8, 8, 1.0, True, True),
    ("ragged_L", 2, 37, 24, 20, 0.1, False, True),
    ("ragged_all", 3, 129, 50, 33, 0.05, True, False),
    ("P_not_mult_64", 2, 70, 64, 100, 0.05, False, True),
    ("H_ne_P_paper_state_task", 4, 128, 512, 256, 0.02, True, False),
    ("H_small_P_large", 2, 40, 4, 300, 0.1, False, True),
    ("all_reset", 2, 48, 16, 16, 1.0, True, True),
    ("no_reset_x0", 2, 300, 32, 48, 0.0, False, True),
    ("multi_block_time", 2, 1000, 32, 40, 0.01, False, True),
    ("multi_block_time_no_reset", 1, 2049, 16, 24, 0.0, False, False),
    ("Bt1", 1, 64, 32, 32, 0.0, True, False),
    ("tiny_everything", 1, 2, 1, 1, 0.0, False, True),
]


@pytest.mark.parametrize("case", EDGE, ids=[c[0] for c in EDGE])
def test_edge_shapes(case):
    name, Bt, L, H, P, pr, ff, x0 = case
    print("edge", case, flush=True)
    w = wl.custom(name, Bt, L, H, P, p_reset=pr, force_first=ff, with_x0=x0, seed=7)
    check_workload(w, backward=True)


def _random_shapes(n, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    out = []
    for i in range(n):
        Bt = int(rng.integers(1, 10))
        L = int(rng.choice([rng.integers(1, 40), rng.integers(40, 300), rng.integers(300, 900)]))
        H = int(rng.choice([rng.integers(1, 20), rng.integers(20, 200), 4 * rng.integers(5, 60)]))
        P = int(rng.choice([rng.integers(1, 20), rng.integers(20, 150), 2 * rng.integers(8, 90)]))
        out.append(("rand%d" % i, Bt, L, H, P, float(rng.choice([0.0, 0.02, 0.3])), bool(rng.integers(0, 2)),
                    bool(rng.integers(0, 2)), 100 + i))
    return out


RANDOM_SHAPES = _random_shapes(16, 20250220)


@pytest.mark.parametrize("case", RANDOM_SHAPES, ids=["%s_%dx%dx%dx%d" % c[:5] for c in RANDOM_SHAPES])
def test_seeded_random_shapes(case):
    """Shapes nobody picked by hand: every combination of ragged tiles, guarded and fast GEMM paths,
    one or several workgroups along time, flags and initial states that the seeded draw produces."""
    name, Bt, L, H, P, pr, ff, x0, seed = case
    print("random shape", case, flush=True)
    check_workload(wl.custom(name, Bt, L, H, P, p_reset=pr, force_first=ff, with_x0=x0, seed=seed), backward=True)


def _random_large_shapes(n, seed):
    """Seeded shapes on the paths that small random shapes never reach: separate scan kernels with two scaled
    fp16 planes (H, P >= 512, L no multiple of 128), more scanning tiles than CUs (two workgroups per CU in
    both projections), and 64-255 scanning tiles with layer widths around the K-step rule of the output
    projection."""
    rng = np.random.Generator(np.random.PCG64(seed))
    out = []
    for i in range(n):
        kind = i % 3
        if kind == 0:
            L = int(rng.choice([50, 100, 200, 300, 77, 130]))
            Bt = int(rng.integers(max(1, 1500 // L), max(2, 5000 // L)))
            H = int(rng.choice([512, 576, 640, 768, 1024, 520, 1100]))
            P = int(rng.choice([512, 520, 600, 640, 768, 1000]))
        elif kind == 1:
            L = int(rng.choice([16, 32, 64, 128, 256, 512, 1024, 2048, 4096]))
            Bt = max(1, int(rng.choice([4096, 8192, 6144])) // L)
            H = int(rng.choice([rng.integers(8, 200), 64 * rng.integers(1, 9)]))
            P = int(rng.choice([320, 384, 500, 512, 640, 700]))
        else:
            L = int(rng.choice([32, 64, 128, 256, 512]))
            Bt = max(1, int(rng.choice([1024, 2048, 4096])) // L)
            H = int(rng.choice([256, 320, 512, 576, 1024, 130]))
            P = int(rng.choice([256, 288, 480, 510, 512]))
        out.append(("large%d" % i, Bt, L, H, P, float(rng.choice([0.0, 0.01, 0.2])), bool(rng.integers(0, 2)),
                    bool(rng.integers(0, 2)), 300 + i))
    return out


RANDOM_LARGE_SHAPES = _random_large_shapes(12, 20250221)


@pytest.mark.parametrize("case", RANDOM_LARGE_SHAPES, ids=["%s_%dx%dx%dx%d" % c[:5] for c in RANDOM_LARGE_SHAPES])
def test_seeded_random_shapes_on_the_large_paths(case):
    name, Bt, L, H, P, pr, ff, x0, seed = case
    print("random large shape", case, ssm.ssm_plan_describe(Bt, L, H, P), flush=True)
    check_workload(wl.custom(name, Bt, L, H, P, p_reset=pr, force_first=ff, with_x0=x0, seed=seed), backward=True)


@pytest.mark.parametrize("Bt,L,H,P", [(2, 5, 8, 65536), (2, 5, 65536, 4), (1, 300, 4, 8192)])
def test_maximum_widths(Bt, L, H, P):
    """The widest state and layer the library accepts (SSM_MAX_WIDTH = 65536) with few tokens: index
    arithmetic, grids with tens of thousands of workgroups along the width, one lane group per
    state block of the scan."""
    check_workload(wl.custom("maxw", Bt, L, H, P, p_reset=0.1, with_x0=True, seed=77), backward=True)


# Shapes whose sequences are whole numbers of 128-step tiles and that fill the chip: here the input
# projection and C^H dy run the scans on their own output tiles (chains of tiles with look-back).
SCANNING_TILES = [
    # name, Bt, L, H, P, p_reset, force_first, with_x0
    ("two_tiles_per_sequence", 16, 256, 24, 512, 0.02, True, True),
    ("chain_of_32_tiles", 1, 4096, 16, 512, 0.002, False, True),
    ("ragged_state_width", 4, 512, 48, 840, 0.05, False, True),
    ("three_sequences_column_groups", 3, 1024, 40, 600, 0.01, True, False),
    ("seven_sequences", 7, 512, 20, 520, 0.0, False, True),
    ("every_step_resets", 8, 256, 16, 1024, 1.0, True, True),
    ("no_reset_no_x0", 8, 384, 16, 640, 0.0, False, False),
    # more tiles than CUs with chains: both projections run two workgroups per CU
    ("chains_in_more_than_one_round_of_tiles", 5, 1024, 24, 520, 0.01, False, True),
    # more tiles than the chip holds at once (2 x 256): later tiles start when earlier ones have left
    ("chains_in_more_tiles_than_are_resident", 9, 2048, 16, 512, 0.002, False, True),
    # several whole sequences per 128-token tile: no chain, a sequence starts at a chunk inside the tile
    ("eight_sequences_per_tile", 256, 16, 16, 1024, 0.05, False, True),
    ("four_sequences_per_tile", 128, 32, 24, 520, 0.05, True, True),
    ("two_sequences_per_tile", 64, 64, 16, 1024, 0.03, False, False),
    ("one_sequence_per_tile", 32, 128, 16, 1024, 0.02, False, True),
    # layer widths that take the other paths of the row-maximum pass: rows longer than 512 values, and a
    # width that is no multiple of 4 (scalar loads)
    ("wide_layer", 16, 256, 1024, 512, 0.02, True, True),
    ("layer_width_50", 16, 256, 50, 512, 0.02, False, True),
    # 64-199 tiles: less than the chip, still scanning tiles
    ("ninety_six_tiles", 24, 128, 512, 256, 0.02, True, True),
    ("sixty_four_tiles", 8, 128, 40, 512, 0.05, False, True),
    ("sixty_four_tiles_of_whole_sequences", 64, 16, 24, 512, 0.05, False, True),
    # more than eight row-maximum words per token (16 column tiles of x and chi, 9 column blocks of dy)
    ("wide_state_many_row_parts", 4, 256, 576, 1024, 0.02, True, True),
]


@pytest.mark.parametrize("case", SCANNING_TILES, ids=[c[0] for c in SCANNING_TILES])
def test_projections_that_scan_their_own_tiles(case):
    name, Bt, L, H, P, pr, ff, x0 = case
    print("scanning tiles", case, flush=True)
    check_workload(wl.custom(name, Bt, L, H, P, p_reset=pr, force_first=ff, with_x0=x0, seed=31), backward=True)


def test_resets_on_the_edges_of_tiles_and_chunks():
    """Flags at the first and last step of 128-step tiles and of the 32-step runs one lane owns,
    at step 0 with an initial state, and at the last step of the sequence."""
    w = wl.custom("edges", 8, 512, 16, 1024, with_x0=True, seed=41)
    inp = wl.gen_inputs(w)
    fl = np.zeros((8, 512), np.uint8)
    fl[0, [127, 128, 129]] = 1
    fl[1, [0, 31, 32, 33, 255, 256]] = 1
    fl[2, [511]] = 1
    fl[3, [128, 384]] = 1
    fl[4, [127, 383, 510]] = 1
    fl[5, [1, 2, 3, 64, 96, 160]] = 1
    fl[6, :] = 0
    fl[7, 256:] = 1
    inp["is_first"] = fl
    check_workload(w, backward=True, inp=inp)


@pytest.mark.parametrize("Bt,L,H,P", [(16, 256, 512, 256), (34, 128, 384, 288), (16, 256, 500, 256), (13, 100, 1200, 256)])
def test_products_with_too_few_tiles_as_two_k_halves(Bt, L, H, P):
    """y and du have 100-199 tiles of 128 x 128 at these shapes: y runs on 64 x 128 tiles, du (where it
    shares its launch with the dBbar slabs only) as two halves of the state dimension that the parameter
    epilogue's launch adds (vector path, and the scalar path for a width that is no multiple of 4).  The
    last shape has ragged tiles in both directions and separate scan kernels (three bf16 planes)."""
    print("two K halves", Bt, L, H, P, flush=True)
    check_workload(wl.custom("halves", Bt, L, H, P, p_reset=0.02, with_x0=True, seed=53), backward=True)


@pytest.mark.parametrize("Bt,L,H,P", [(40, 100, 512, 512), (23, 100, 640, 512), (12, 300, 1024, 512)])
def test_separate_scan_kernels_with_two_fp16_planes(Bt, L, H, P):
    """Sequences that are not whole 128-step tiles, with long contraction lengths (H >= 512, P >= 512) and more
    than 64 tiles per product: the scan kernels record the largest magnitude of every token row of x and chi,
    and all six products stage two scaled fp16 planes.  Whole tiles, ragged token tiles, and a chain of scan
    workgroups along time (L = 300)."""
    print("unfused two planes", Bt, L, H, P, flush=True)
    check_workload(wl.custom("unfused2", Bt, L, H, P, p_reset=0.02, with_x0=True, seed=61), backward=True)


def test_separate_scan_kernels_two_planes_wide_range_between_tokens():
    """The same path with token magnitudes spread over six decades (every token row of u, x, dy and chi gets its
    own scale): per-tensor checks would hide the small tokens, so du and y are compared row by row."""
    w = wl.custom("unfused2_range", 40, 100, 512, 512, p_reset=0.02, with_x0=False, seed=67)
    inp = wl.gen_inputs(w)
    rng = np.random.Generator(np.random.PCG64(5))
    scale = (10.0 ** rng.uniform(-3, 3, size=(w.Bt, 1, 1))).astype(np.float32)      # one magnitude per sequence
    inp["u"] = (inp["u"] * scale).astype(np.float32)
    inp["dy"] = (inp["dy"] * scale).astype(np.float32)
    d = ssm.to_device(inp)
    par = (d["Lambda"], d["B"], d["C"], d["D"], d["log_delta"])
    f = ssm.ssm_scan_fwd(*par, d["u"], d["is_first"], d["x0"])
    g = ssm.ssm_scan_bwd(*par, d["u"], d["is_first"], d["x0"], f["x"], d["dy"])
    ref = orc.run_workload(inp, True)
    for name, got, tol in (("y", f["y"], TOL_FWD), ("du", g["du"], TOL_GRAD)):
        a = got.cpu().numpy().astype(np.float64).reshape(w.Bt, -1)
        r = ref[name].astype(np.float64).reshape(w.Bt, -1)
        rel = np.linalg.norm(a - r, axis=1) / np.linalg.norm(r, axis=1)
        assert rel.max() <= tol, "%s: worst sequence %d, relative error %.3e" % (name, int(rel.argmax()), rel.max())


def test_flag_array_at_an_odd_address():
    """is_first only needs byte alignment: the 16-byte flag loads of the scanning tiles and of the
    scan kernel must fall back to byte loads for a buffer that starts at an odd address."""
    import torch
    for Bt, L, H, P in ((8, 256, 16, 1024), (128, 16, 16, 1024), (3, 200, 16, 48)):
        w = wl.custom("oddflags", Bt, L, H, P, p_reset=0.05, with_x0=True, seed=47)
        inp = wl.gen_inputs(w)
        ref = orc.run_workload(inp, True, nthreads=4)
        d = ssm.to_device(inp)
        raw = torch.zeros(Bt * L + 3, dtype=torch.uint8, device="cuda")
        flags = raw[3:].view(Bt, L)
        flags.copy_(d["is_first"])
        assert flags.data_ptr() % 2 == 1 and flags.is_contiguous()
        par = (d["Lambda"], d["B"], d["C"], d["D"], d["log_delta"])
        fwd = ssm.ssm_scan_fwd(*par, d["u"], flags, d["x0"])
        bwd = ssm.ssm_scan_bwd(*par, d["u"], flags, d["x0"], fwd["x"], d["dy"])
        torch.cuda.synchronize()
        assert_close(fwd["x"].cpu().numpy(), ref["x"], TOL_FWD, "odd flags x")
        assert_close(fwd["y"].cpu().numpy(), ref["y"], TOL_FWD, "odd flags y")
        for k in GRAD_KEYS:
            assert_close(bwd[k].cpu().numpy(), ref[k], TOL_GRAD, "odd flags " + k)


def test_scanning_tiles_are_bitwise_repeatable():
    import torch
    w = wl.custom("repeat", 8, 512, 32, 640, p_reset=0.02, with_x0=True, seed=43)
    inp = wl.gen_inputs(w)
    a = run_gpu(inp, True)
    b = run_gpu(inp, True)
    for k in FWD_KEYS_ALL:
        assert np.array_equal(a[k], b[k]), k


def test_reset_at_last_step_and_x0_with_first_step_reset():
    w = wl.custom("last", 3, 50, 16, 24, with_x0=True, seed=3)
    inp = wl.gen_inputs(w)
    fl = np.zeros((3, 50), np.uint8)
    fl[0, 49] = 1          # reset at the very last step
    fl[1, 0] = 1           # first-step reset: x0 must be ignored for this sequence
    fl[2, 16] = fl[2, 17] = 1   # adjacent resets across a chunk boundary
    inp["is_first"] = fl
    check_workload(w, backward=True, inp=inp)


def test_slow_decay_long_sequence_accumulated_error():
    """Config-3-like: |Abar| ~ 1 over thousands of steps, several workgroups along time."""
    w = wl.custom("slow", 2, 3000, 32, 48, p_reset=0.001, force_first=True, lam_re_lo=0.001,
                  lam_re_hi=0.1, seed=5)
    check_workload(w, backward=True)


def test_inference_path_without_saved_states():
    import torch
    w = wl.custom("infer", 4, 96, 32, 48, p_reset=0.05, with_x0=True, seed=9)
    inp = wl.gen_inputs(w)
    ref = orc.run_workload(inp, False)
    d = ssm.to_device(inp)
    out = ssm.ssm_scan_fwd(d["Lambda"], d["B"], d["C"], d["D"], d["log_delta"], d["u"], d["is_first"],
                           d["x0"], want_x=False, want_x_last=False)
    torch.cuda.synchronize()
    assert out["x"] is None and out["x_last"] is None
    assert_close(out["y"].cpu().numpy(), ref["y"], TOL_FWD, "infer y")


def test_carry_split_equals_one_run_on_gpu():
    import torch
    w = wl.custom("carry", 3, 200, 32, 40, p_reset=0.02, with_x0=True, seed=11)
    inp = wl.gen_inputs(w)
    d = ssm.to_device(inp)
    args = (d["Lambda"], d["B"], d["C"], d["D"], d["log_delta"])
    full = ssm.ssm_scan_fwd(*args, d["u"], d["is_first"], d["x0"])
    h1 = ssm.ssm_scan_fwd(*args, d["u"][:, :77].contiguous(), d["is_first"][:, :77].contiguous(), d["x0"])
    h2 = ssm.ssm_scan_fwd(*args, d["u"][:, 77:].contiguous(), d["is_first"][:, 77:].contiguous(), h1["x_last"])
    torch.cuda.synchronize()
    y12 = torch.cat([h1["y"], h2["y"]], 1).cpu().numpy()
    assert_close(y12, full["y"].cpu().numpy().astype(np.float64), 1e-5, "carry y")
    assert_close(h2["x_last"].cpu().numpy(), full["x_last"].cpu().numpy().astype(np.complex128), 1e-5, "carry x_last")


def test_discretize_matches_oracle():
    import torch
    rng = np.random.default_rng(0)
    P, H = 300, 20
    Lam = (-rng.uniform(1e-3, 1.0, P) + 1j * rng.uniform(0, np.pi, P)).astype(np.complex64)
    Lam[:4] = [0.0, -1e-6 + 1e-6j, -40.0 + 3j, -1e-3]
    ld = rng.uniform(np.log(1e-3), np.log(1e-1), P).astype(np.float32)
    ld[2] = 3.0
    B = (rng.normal(size=(P, H)) + 1j * rng.normal(size=(P, H))).astype(np.complex64)
    A_ref, g_ref = orc.discretize(Lam, ld)
    A, Bb = ssm.ssm_discretize(torch.from_numpy(Lam).cuda(), torch.from_numpy(B).cuda(),
                               torch.from_numpy(ld).cuda())
    torch.cuda.synchronize()
    A, Bb = A.cpu().numpy(), Bb.cpu().numpy()
    # element-wise: every state is its own number here, so no norm can hide a bad one
    assert np.max(np.abs(A - A_ref) / np.maximum(np.abs(A_ref), 1e-30)) < 5e-7
    Bref = g_ref[:, None] * B.astype(np.complex128)
    assert np.max(np.abs(Bb - Bref) / np.abs(Bref)) < 1e-6
    A2, none = ssm.ssm_discretize(torch.from_numpy(Lam).cuda(), None, torch.from_numpy(ld).cuda())
    assert none is None and np.array_equal(A2.cpu().numpy(), A)


@pytest.mark.parametrize("shape", [(2, 40, 8, 12), (16, 256, 32, 512)], ids=["small", "scanning_tiles"])
def test_discretisation_adjoint_over_the_whole_range_of_lambda_delta(shape):
    """dLambda, dlog_delta and dB element by element for |Lambda Delta| in {0, 1e-6, 0.6, 3, 50}: the
    adjoint of the zero-order hold evaluates psi'(z) = d/dz (e^z - 1)/z by a series for small |z| and by
    the closed form elsewhere, and has the limit Lambda = 0; every regime feeds compared values here
    (real and complex z in each), on a shape that takes the scan kernels and on one whose projections
    scan their own tiles."""
    Bt, L, H, P = shape
    w = wl.custom("zoh_adjoint", Bt, L, H, P, p_reset=0.05, with_x0=True, seed=71)
    inp = wl.gen_inputs(w)
    mags = [0.0, 1e-6, 0.6, 3.0, 50.0, 0.6, 3.0, 1e-6, 50.0, 0.49, 0.51, 0.0]
    args = [np.pi, np.pi, np.pi, np.pi, np.pi, 2.0, 2.4, 1.7, 2.8, 2.0, 2.0, 0.0]     # pi: real negative z
    delta = np.exp(inp["log_delta"].astype(np.float64))
    lam = np.array(inp["Lambda"], dtype=np.complex128)
    n = len(mags)
    planted = np.array(mags) * np.exp(1j * np.array(args)) / delta[:n]
    real_z = np.array(args) == np.pi
    planted[real_z] = -np.array(mags)[real_z] / delta[:n][real_z]
    lam[:n] = planted
    inp["Lambda"] = lam.astype(np.complex64)
    z = inp["Lambda"].astype(np.complex128)[:n] * delta[:n]
    assert np.all(z.real <= 0.0) and abs(z[0]) == 0.0 and abs(z[-1]) == 0.0
    assert np.sum(np.abs(z) ** 2 < 0.25) >= 5 and np.sum(np.abs(z) ** 2 >= 0.25) >= 6     # both evaluations are fed
    ref = orc.run_workload(inp, True)
    got = run_gpu(inp, True)
    worst = {}
    for k in ("dLambda", "dlog_delta"):
        assert_close(got[k], ref[k], TOL_GRAD, "zoh adjoint " + k)
        worst[k] = assert_close_elementwise(got[k], ref[k], TOL_GRAD, "zoh adjoint " + k)
        # the planted states on their own, against their own rms
        worst[k + "[planted]"] = assert_close_elementwise(got[k][:n], ref[k][:n], TOL_GRAD, "zoh adjoint planted " + k)
    for p in range(n):                                       # every planted row of dB against its own scale
        worst["dB[%d]" % p] = assert_close(got["dB"][p], ref["dB"][p], TOL_GRAD, "zoh adjoint dB row %d" % p)[1]
    assert_close(got["dB"], ref["dB"], TOL_GRAD, "zoh adjoint dB")
    for k in ("y", "x"):
        assert_close(got[k], ref[k], TOL_FWD, "zoh adjoint " + k)
    print({k: "%.2e" % v for k, v in worst.items()}, flush=True)


def test_wide_range_inside_one_token_and_inside_one_weight_row():
    """One token whose features span 1e-6 .. 1e3, and one row of B likewise, through the benchmark
    shape.  Under one power-of-two scale with largest magnitude m an element is held with an absolute
    error of max(2^-22 |a|, 2^-39 m) (the bound the header states): the small features of the token
    reach x and y only next to its large ones, so the token's outputs keep the tolerances against
    their own scale, and so does the planted state."""
    w = wl.CONFIGS[2]
    inp = dict(wl.gen_inputs(w))
    rng = np.random.default_rng(5)
    span = (10.0 ** rng.uniform(-6, 3, w.H)).astype(np.float32)
    u = inp["u"].copy(); u[4, 100] *= span; inp["u"] = u
    dy = inp["dy"].copy(); dy[6, 30] *= span; inp["dy"] = dy
    B = inp["B"].copy(); B[17] *= span; inp["B"] = B
    ref = orc.run_workload(inp, True)
    got = run_gpu(inp, True)
    for k in ("y", "x", "x_last"):
        assert_close(got[k], ref[k], TOL_FWD, "span " + k)
    for k in GRAD_KEYS:
        assert_close(got[k], ref[k], TOL_GRAD, "span " + k)
    rel = lambda a, b: float(np.linalg.norm((a - b).ravel()) / np.linalg.norm(b.ravel()))
    rep = {"x[4,100]": rel(got["x"][4, 100], ref["x"][4, 100]), "y[4,100]": rel(got["y"][4, 100], ref["y"][4, 100]),
           "du[6,30]": rel(got["du"][6, 30], ref["du"][6, 30]), "x[:,:,17]": rel(got["x"][:, :, 17], ref["x"][:, :, 17]),
           "dB[17]": rel(got["dB"][17], ref["dB"][17])}
    # per-element error of the outputs that the small entries dominate: the columns of dB[17] whose
    # factor is small (dB[17, h] = conj(g) sum_t chi u[t, h] does not depend on B) and the token's du
    small = span < 1e-3
    rep["du[6,30] small features, max rel"] = float(np.max(np.abs(got["du"][6, 30][small] - ref["du"][6, 30][small])
                                                           / np.abs(ref["du"][6, 30][small])))
    print(rep, flush=True)
    assert rep["x[4,100]"] <= TOL_FWD and rep["y[4,100]"] <= TOL_FWD and rep["x[:,:,17]"] <= TOL_FWD, rep
    assert rep["du[6,30]"] <= TOL_GRAD and rep["dB[17]"] <= TOL_GRAD, rep


SCAN_CASES = [(2, 64, 32, 0.05), (1, 16, 700, 0.0), (3, 777, 20, 0.01), (1, 5000, 16, 0.002), (2, 1, 5, 0.0)]


@pytest.mark.parametrize("Bt,L,P,pr", SCAN_CASES)
def test_scan_level_entries_against_oracle_recurrence(Bt, L, P, pr):
    import torch
    print("scan", Bt, L, P, pr, flush=True)
    rng = np.random.default_rng(L)
    Abar = (rng.uniform(0.9, 1.0, P) * np.exp(1j * rng.uniform(0, np.pi, P))).astype(np.complex64)
    v = (rng.normal(size=(Bt, L, P)) + 1j * rng.normal(size=(Bt, L, P))).astype(np.complex64)
    x0 = (rng.normal(size=(Bt, P)) + 1j * rng.normal(size=(Bt, P))).astype(np.complex64)
    fl = (rng.random((Bt, L)) < pr).astype(np.uint8)
    x_ref = orc.scan(Abar, v, fl, x0)
    dA, dv, dfl, dx0 = (torch.from_numpy(a).cuda() for a in (Abar, v, fl, x0))
    xg, xl = ssm.ssm_scan_states(dA, dv.clone(), dfl, dx0)
    torch.cuda.synchronize()
    assert_close(xg.cpu().numpy(), x_ref, TOL_FWD, "scan x")
    assert_close(xl.cpu().numpy(), x_ref[:, -1], TOL_FWD, "scan x_last")
    assert ssm.ssm_workspace_status(ssm.alloc_workspace(Bt, L, 1, P, False)) in (ssm.SSM_OK, ssm.SSM_ERR_INVALID_ARG)
    # reverse scan: chi_t = gx_t + [not first_{t+1}] conj(Abar) chi_{t+1} is the forward recurrence of
    # the oracle on the time-reversed sequence with conj(Abar) and the flags shifted by one
    gx = (rng.normal(size=(Bt, L, P)) + 1j * rng.normal(size=(Bt, L, P))).astype(np.complex64)
    fl_shift = np.zeros_like(fl)
    fl_shift[:, :-1] = fl[:, 1:]                       # flag of step t+1 sits at t
    chi_ref = orc.scan(np.conj(Abar), gx[:, ::-1], fl_shift[:, ::-1])[:, ::-1]
    xs = x_ref.astype(np.complex64)
    prev = np.concatenate([x0[:, None, :].astype(np.complex128), xs[:, :-1].astype(np.complex128)], 1)
    dA_ref = np.sum((1 - fl)[:, :, None] * np.conj(prev) * chi_ref, axis=(0, 1))
    dx0_ref = (1 - fl[:, 0])[:, None] * np.conj(Abar.astype(np.complex128)) * chi_ref[:, 0]
    ws = ssm.alloc_workspace(Bt, L, 1, P, True)
    chi, dAg, dx0g = ssm.ssm_scan_states_reverse(dA, torch.from_numpy(gx).cuda(), torch.from_numpy(xs).cuda(),
                                                 dfl, dx0, workspace=ws)
    assert ssm.ssm_workspace_status(ws) == ssm.SSM_OK
    assert_close(chi.cpu().numpy(), chi_ref, TOL_FWD, "chi")
    assert_close(dAg.cpu().numpy(), dA_ref, TOL_GRAD, "dA_bar")
    assert_close(dx0g.cpu().numpy(), dx0_ref, TOL_GRAD, "dx0")


def test_zero_transition_scan_is_identity():
    import torch
    rng = np.random.default_rng(1)
    v = (rng.normal(size=(2, 300, 24)) + 1j * rng.normal(size=(2, 300, 24))).astype(np.complex64)
    x0 = torch.from_numpy((rng.normal(size=(2, 24)) + 0j).astype(np.complex64)).cuda()
    xg, _ = ssm.ssm_scan_states(torch.zeros(24, dtype=torch.complex64, device="cuda"),
                                torch.from_numpy(v).cuda(), None, x0)
    torch.cuda.synchronize()
    assert np.array_equal(xg.cpu().numpy(), v)


def test_repeated_runs_are_bitwise_identical():
    """The cross-workgroup hand-over must not depend on scheduling."""
    import torch
    w = wl.custom("det", 2, 2500, 32, 48, p_reset=0.002, force_first=True, lam_re_lo=0.001, lam_re_hi=0.1)
    inp = wl.gen_inputs(w)
    first = run_gpu(inp, True)
    for rep in range(5):
        again = run_gpu(inp, True)
        for k, v in first.items():
            if v is not None:
                assert np.array_equal(v, again[k]), (rep, k)


def test_projections_have_fp32_class_accuracy():
    """The projections run on the 16-bit matrix cores with an exact three-way bf16 split of every fp32
    operand at this shape (too few tiles for the scanning projections).  With Abar = 0 the states are
    the bare input projection x = Bbar u, so their error is the product's alone: it must sit at the
    level of fp32 rounding (a length-512 dot product accumulated in fp32: about sqrt(512) * 6e-8 / 2),
    far inside the 1e-4 budget."""
    w = wl.custom("gemm_acc", 4, 64, 512, 256, seed=17)
    inp = wl.gen_inputs(w)
    inp["Lambda"] = np.full(256, -50.0 + 1.0j, np.complex64)
    inp["log_delta"] = np.full(256, 10.0, np.float32)       # Lambda * Delta -> -1e6: Abar underflows to 0
    ref = orc.run_workload(inp, True)
    got = run_gpu(inp, True)
    errs = {k: assert_close(got[k], ref[k], 3e-6, "bf16x3 " + k)[0] for k in ("x", "y", "du", "dC", "dB")}
    print(errs, flush=True)
    assert max(errs.values()) <= 1.2e-6, errs


def _bare_projections(Bt, L, H, P, seed):
    """Inputs whose Abar underflows to zero, so that x, y and the gradients are bare matrix products."""
    inp = wl.gen_inputs(wl.custom("bare", Bt, L, H, P, seed=seed))
    inp["Lambda"] = np.full(P, -50.0 + 1.0j, np.complex64)
    inp["log_delta"] = np.full(P, 10.0, np.float32)
    return inp


def test_two_scaled_fp16_planes_are_as_accurate_as_fp32_products():
    """Where every operand of a product brings its largest magnitude, the product is staged as two
    scaled fp16 planes per operand (three matrix instructions per k block).  Its error against the
    float64 oracle must sit at the level of a plain fp32 product (measured for the fp32 matrix
    instruction on the same bare projections: x 4.1e-7, dC 5.8e-7, dB 7.1e-7 normwise)."""
    inp = _bare_projections(16, 256, 512, 512, 17)
    ref = orc.run_workload(inp, True)
    got = run_gpu(inp, True)
    errs = {k: assert_close(got[k], ref[k], 2e-6, "fp16x2 " + k)[0] for k in ("x", "y", "du", "dC", "dB")}
    print(errs, flush=True)
    assert errs["x"] <= 4.5e-7 and errs["dC"] <= 6e-7 and errs["dB"] <= 7.5e-7, errs


@pytest.mark.parametrize("scale_u,scale_dy", [(1e-20, 1e15), (3e18, 1e-25), (1.0, 0.0)])
def test_scaled_fp16_planes_follow_the_magnitude_of_the_operands(scale_u, scale_dy):
    """The power-of-two scale of an operand comes from its largest magnitude, measured on the device
    for every call: inputs far outside the fp16 range (and all-zero ones) give the same relative
    accuracy as inputs of order one."""
    inp = dict(wl.gen_inputs(wl.CONFIGS[2]))
    inp["u"] = (inp["u"].astype(np.float64) * scale_u).astype(np.float32)
    inp["dy"] = (inp["dy"].astype(np.float64) * scale_dy).astype(np.float32)
    ref = orc.run_workload(inp, True)
    got = run_gpu(inp, True)
    for k in ("y", "x", "x_last"):
        assert_close(got[k], ref[k], TOL_FWD, "scaled " + k)
    for k in ("du", "dLambda", "dB", "dC", "dD", "dlog_delta"):
        if scale_dy == 0.0:
            assert np.all(got[k] == 0), k                    # zero gradients exactly, no NaN from the scales
        else:
            assert_close(got[k], ref[k], TOL_GRAD, "scaled " + k)


def test_scaled_fp16_planes_with_a_wide_range_inside_one_operand():
    """u, x, dy and chi enter their products with tokens as rows, and every token row gets its own
    power-of-two scale (a single scale per matrix would hold a token ten orders of magnitude below
    the largest element of the batch as a fixed-point number).  Pinned here: a sequence scaled by
    1e-10 next to an outlier element of 1e4 keeps the stated tolerances when its own y, x and du are
    looked at alone, and the whole tensors keep them as well."""
    inp = dict(wl.gen_inputs(wl.CONFIGS[2]))
    u = inp["u"].copy(); u[3] *= 1e-10; u[5, 7, 11] = 1e4; inp["u"] = u
    dy = inp["dy"].copy(); dy[2] *= 1e-10; dy[9, 100, 3] = -1e4; inp["dy"] = dy
    ref = orc.run_workload(inp, True)
    got = run_gpu(inp, True)
    for k in ("y", "x", "x_last"):
        assert_close(got[k], ref[k], TOL_FWD, "wide " + k)
    for k in ("du", "dLambda", "dB", "dC", "dD", "dlog_delta"):
        assert_close(got[k], ref[k], TOL_GRAD, "wide " + k)
    rel = lambda a, b: float(np.linalg.norm((a - b).ravel()) / np.linalg.norm(b.ravel()))
    small = {"y[3]": rel(got["y"][3], ref["y"][3]), "x[3]": rel(got["x"][3], ref["x"][3]), "du[2]": rel(got["du"][2], ref["du"][2])}
    print(small, flush=True)
    assert small["y[3]"] <= 1e-5 and small["x[3]"] <= 1e-5 and small["du[2]"] <= 1e-5, small


def test_bounded_wait_reports_instead_of_hanging():
    """A spin limit of zero lets every cross-workgroup wait give up at once: the kernels must
    still terminate, and either the status call reports the give-up and the outputs that depend on
    the missing state are NaN, or (if every predecessor happened to be ready) the results are right."""
    import torch
    w = wl.custom("spin0", 2, 2048, 16, 32, p_reset=0.0, seed=3)
    inp = wl.gen_inputs(w)
    d = ssm.to_device(inp)
    ws = ssm.alloc_workspace(w.Bt, w.L, w.H, w.P, False)
    old = ssm.ssm_set_spin_limit(0)
    try:
        out = ssm.ssm_scan_fwd(d["Lambda"], d["B"], d["C"], d["D"], d["log_delta"], d["u"], d["is_first"], d["x0"],
                               workspace=ws)
        status = ssm.ssm_workspace_status(ws)
    finally:
        ssm.ssm_set_spin_limit(old)
    assert status in (ssm.SSM_OK, ssm.SSM_ERR_SCAN_TIMEOUT)
    if status == ssm.SSM_OK:
        ref = orc.run_workload(inp, False)
        assert_close(out["y"].cpu().numpy(), ref["y"], TOL_FWD, "spin0 y")
    else:
        assert bool(torch.isnan(out["y"]).any()) and bool(torch.isnan(out["x"].real).any()), "a give-up must poison its outputs"
    # and with the default limit the same call is clean
    out = ssm.ssm_scan_fwd(d["Lambda"], d["B"], d["C"], d["D"], d["log_delta"], d["u"], d["is_first"], d["x0"],
                           workspace=ws)
    assert ssm.ssm_workspace_status(ws) == ssm.SSM_OK
    assert not bool(torch.isnan(out["y"]).any())


@pytest.mark.parametrize("Bt", [1, 2])
def test_bounded_wait_inside_the_scanning_projections(Bt):
    """The same for the waits along the chain of tiles of a sequence (32 tiles here) inside the input
    projection and inside C^H dy: with a spin limit of zero both passes terminate; each reports and
    poisons, or is right.  One sequence: 256 tiles, one workgroup per CU; two: 512 tiles, the variants with
    two workgroups per CU."""
    import torch
    w = wl.custom("spin0_tiles", Bt, 4096, 16, 512, p_reset=0.001, with_x0=True, seed=5)
    inp = wl.gen_inputs(w)
    d = ssm.to_device(inp)
    par = (d["Lambda"], d["B"], d["C"], d["D"], d["log_delta"])
    ws_f = ssm.alloc_workspace(w.Bt, w.L, w.H, w.P, False)
    ws_b = ssm.alloc_workspace(w.Bt, w.L, w.H, w.P, True)
    good = ssm.ssm_scan_fwd(*par, d["u"], d["is_first"], d["x0"], workspace=ws_f)
    assert ssm.ssm_workspace_status(ws_f) == ssm.SSM_OK
    x_good = good["x"].clone()
    old = ssm.ssm_set_spin_limit(0)
    try:
        out = ssm.ssm_scan_fwd(*par, d["u"], d["is_first"], d["x0"], workspace=ws_f)
        st_f = ssm.ssm_workspace_status(ws_f)
        grads = ssm.ssm_scan_bwd(*par, d["u"], d["is_first"], d["x0"], x_good, d["dy"], workspace=ws_b)
        st_b = ssm.ssm_workspace_status(ws_b)
    finally:
        ssm.ssm_set_spin_limit(old)
    assert st_f in (ssm.SSM_OK, ssm.SSM_ERR_SCAN_TIMEOUT) and st_b in (ssm.SSM_OK, ssm.SSM_ERR_SCAN_TIMEOUT)
    ref = orc.run_workload(inp, True)
    if st_f == ssm.SSM_OK:
        assert_close(out["y"].cpu().numpy(), ref["y"], TOL_FWD, "spin0 tiles y")
    else:
        assert bool(torch.isnan(out["y"]).any()), "a give-up must poison its outputs"
    if st_b == ssm.SSM_OK:
        assert_close(grads["du"].cpu().numpy(), ref["du"], TOL_GRAD, "spin0 tiles du")
    else:
        assert bool(torch.isnan(grads["du"]).any()), "a give-up must poison its outputs"
    # with the default limit the same calls on the same workspaces are clean and right
    out = ssm.ssm_scan_fwd(*par, d["u"], d["is_first"], d["x0"], workspace=ws_f)
    grads = ssm.ssm_scan_bwd(*par, d["u"], d["is_first"], d["x0"], out["x"], d["dy"], workspace=ws_b)
    assert ssm.ssm_workspace_status(ws_f) == ssm.SSM_OK and ssm.ssm_workspace_status(ws_b) == ssm.SSM_OK
    assert_close(out["y"].cpu().numpy(), ref["y"], TOL_FWD, "tiles y")
    assert_close(grads["dLambda"].cpu().numpy(), ref["dLambda"], TOL_GRAD, "tiles dLambda")


def test_two_stacked_layers_at_the_vision_shape():
    """Vision-task shape of the paper's hyper-parameter table (layer width 1024, state 512, two SSM
    layers): layer 2 consumes layer 1's output, the gradient pass chains back through both.  The
    oracle is chained the same way, so this checks H != P at the large width and back-to-back calls
    on one stream sharing a workspace."""
    import torch
    Bt, L, H, P = 8, 64, 1024, 512
    w1 = wl.custom("vision_l1", Bt, L, H, P, p_reset=0.02, force_first=True, seed=31)
    w2 = wl.custom("vision_l2", Bt, L, H, P, p_reset=0.02, force_first=True, seed=32)
    i1, i2 = wl.gen_inputs(w1), wl.gen_inputs(w2)
    i2["is_first"] = i1["is_first"]                       # same episode boundaries for both layers
    # oracle: forward 1 -> forward 2 -> backward 2 -> backward 1
    nt = 8
    r1 = orc.forward(i1["Lambda"], i1["B"], i1["C"], i1["D"], i1["log_delta"], i1["u"], i1["is_first"], None, nt)
    u2 = r1["y"].astype(np.float32)                        # layer 2 sees the fp32-rounded activations
    r2 = orc.forward(i2["Lambda"], i2["B"], i2["C"], i2["D"], i2["log_delta"], u2, i2["is_first"], None, nt)
    g2 = orc.backward(i2["Lambda"], i2["B"], i2["C"], i2["D"], i2["log_delta"], u2, i2["is_first"], None,
                      r2["x"], i2["dy"], nt)
    g1 = orc.backward(i1["Lambda"], i1["B"], i1["C"], i1["D"], i1["log_delta"], i1["u"], i1["is_first"], None,
                      r1["x"], g2["du"].astype(np.float32), nt)
    d1, d2 = ssm.to_device(i1), ssm.to_device(i2)
    ws_f = ssm.alloc_workspace(Bt, L, H, P, False)
    ws_b = ssm.alloc_workspace(Bt, L, H, P, True)
    f1 = ssm.ssm_scan_fwd(d1["Lambda"], d1["B"], d1["C"], d1["D"], d1["log_delta"], d1["u"], d1["is_first"], None,
                          workspace=ws_f)
    f2 = ssm.ssm_scan_fwd(d2["Lambda"], d2["B"], d2["C"], d2["D"], d2["log_delta"], f1["y"], d1["is_first"], None,
                          workspace=ws_f)
    b2 = ssm.ssm_scan_bwd(d2["Lambda"], d2["B"], d2["C"], d2["D"], d2["log_delta"], f1["y"], d1["is_first"], None,
                          f2["x"], d2["dy"], workspace=ws_b)
    b1 = ssm.ssm_scan_bwd(d1["Lambda"], d1["B"], d1["C"], d1["D"], d1["log_delta"], d1["u"], d1["is_first"], None,
                          f1["x"], b2["du"], workspace=ws_b)
    torch.cuda.synchronize()
    assert_close(f2["y"].cpu().numpy(), r2["y"], TOL_FWD, "layer 2 y")
    assert_close(b2["dC"].cpu().numpy(), g2["dC"], TOL_GRAD, "layer 2 dC")
    for k in ("du", "dLambda", "dB", "dC", "dD", "dlog_delta"):
        assert_close(b1[k].cpu().numpy(), g1[k], TOL_GRAD, "layer 1 " + k)


def test_two_stacked_layers_at_the_vision_shape_and_batch_eager_and_as_a_graph():
    """The vision task's sequence model as the hyper-parameter table gives it: two layers of width
    1024 with 512 states on a batch of 32 windows of length 128.  Here the projections scan their own
    tiles and stage two fp16 planes.  Forward through both layers and back through both, against the
    oracle chained the same way; then the same eight calls captured into one HIP graph and replayed
    (with eager work in between) must reproduce the eager results bit for bit."""
    import torch
    Bt, L, H, P = 32, 128, 1024, 512
    w1 = wl.custom("vision_l1", Bt, L, H, P, p_reset=0.01, force_first=True, seed=33)
    w2 = wl.custom("vision_l2", Bt, L, H, P, p_reset=0.01, force_first=True, seed=34)
    i1, i2 = wl.gen_inputs(w1), wl.gen_inputs(w2)
    i2["is_first"] = i1["is_first"]
    nt = 8
    par1 = (i1["Lambda"], i1["B"], i1["C"], i1["D"], i1["log_delta"])
    par2 = (i2["Lambda"], i2["B"], i2["C"], i2["D"], i2["log_delta"])
    r1 = orc.forward(*par1, i1["u"], i1["is_first"], None, nt)
    u2 = r1["y"].astype(np.float32)                        # layer 2 sees the fp32-rounded activations
    r2 = orc.forward(*par2, u2, i2["is_first"], None, nt)
    g2 = orc.backward(*par2, u2, i2["is_first"], None, r2["x"], i2["dy"], nt)
    g1 = orc.backward(*par1, i1["u"], i1["is_first"], None, r1["x"], g2["du"].astype(np.float32), nt)
    d1, d2 = ssm.to_device(i1), ssm.to_device(i2)
    p1 = (d1["Lambda"], d1["B"], d1["C"], d1["D"], d1["log_delta"])
    p2 = (d2["Lambda"], d2["B"], d2["C"], d2["D"], d2["log_delta"])
    ws_f = ssm.alloc_workspace(Bt, L, H, P, False)
    ws_b = ssm.alloc_workspace(Bt, L, H, P, True)
    cx = lambda: torch.empty((Bt, L, P), dtype=torch.complex64, device="cuda")
    c0 = lambda: torch.empty((Bt, P), dtype=torch.complex64, device="cuda")
    o = {"f1": {"y": torch.empty_like(d1["u"]), "x": cx(), "x_last": c0()},
         "f2": {"y": torch.empty_like(d1["u"]), "x": cx(), "x_last": c0()}}
    for name, d in (("b2", d2), ("b1", d1)):
        o[name] = {"du": torch.empty_like(d["u"]), "dLambda": torch.empty_like(d["Lambda"]), "dB": torch.empty_like(d["B"]),
                   "dC": torch.empty_like(d["C"]), "dD": torch.empty_like(d["D"]), "dlog_delta": torch.empty_like(d["log_delta"]),
                   "dx0": c0()}

    def stack():
        ssm.ssm_scan_fwd(*p1, d1["u"], d1["is_first"], None, workspace=ws_f, out=o["f1"])
        ssm.ssm_scan_fwd(*p2, o["f1"]["y"], d1["is_first"], None, workspace=ws_f, out=o["f2"])
        ssm.ssm_scan_bwd(*p2, o["f1"]["y"], d1["is_first"], None, o["f2"]["x"], d2["dy"], workspace=ws_b, out=o["b2"])
        ssm.ssm_scan_bwd(*p1, d1["u"], d1["is_first"], None, o["f1"]["x"], o["b2"]["du"], workspace=ws_b, out=o["b1"])

    stack()
    torch.cuda.synchronize()
    assert ssm.ssm_workspace_status(ws_f) == ssm.SSM_OK and ssm.ssm_workspace_status(ws_b) == ssm.SSM_OK
    assert_close(o["f1"]["y"].cpu().numpy(), r1["y"], TOL_FWD, "layer 1 y")
    assert_close(o["f2"]["y"].cpu().numpy(), r2["y"], TOL_FWD, "layer 2 y")
    assert_close(o["f2"]["x"].cpu().numpy(), r2["x"], TOL_FWD, "layer 2 x")
    for k in ("du", "dLambda", "dB", "dC", "dD", "dlog_delta"):
        assert_close(o["b2"][k].cpu().numpy(), g2[k], TOL_GRAD, "layer 2 " + k)
        assert_close(o["b1"][k].cpu().numpy(), g1[k], TOL_GRAD, "layer 1 " + k)
    for k in ("dLambda", "dlog_delta", "dD"):
        assert_close_elementwise(o["b1"][k].cpu().numpy(), g1[k], TOL_GRAD, "layer 1 " + k)
    eager = {n: {k: v.clone() for k, v in t.items()} for n, t in o.items()}
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        stack()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            stack()
    torch.cuda.synchronize()
    for rep in range(3):
        for t in o.values():
            for v in t.values():
                v.zero_()                                   # eager work between the replays
        junk = torch.randn(1 << 20, device="cuda").sum().item()
        assert np.isfinite(junk)
        graph.replay()
        torch.cuda.synchronize()
        for n, t in o.items():
            for k, v in t.items():
                assert torch.equal(v, eager[n][k]), "replay %d differs from the eager result in %s %s" % (rep, n, k)
        assert ssm.ssm_workspace_status(ws_f) == ssm.SSM_OK and ssm.ssm_workspace_status(ws_b) == ssm.SSM_OK


@pytest.mark.parametrize("Bt,H,P,steps", [(1024, 512, 512, 10), (37, 50, 33, 6)])
def test_step_mode_rollout_equals_oracle_sequence(Bt, H, P, steps):
    """Imagination-style roll-out: `steps` dependent calls of ssm_step, each fed the previous
    state, against the oracle run over the same inputs as one sequence (stepping and scanning
    reach the same states)."""
    import torch
    w = wl.custom("step", Bt, steps, H, P, p_reset=0.1, with_x0=True, seed=23)
    inp = wl.gen_inputs(w)
    ref = orc.forward(inp["Lambda"], inp["B"], inp["C"], inp["D"], inp["log_delta"], inp["u"], inp["is_first"],
                      inp["x0"], nthreads=8)
    d = ssm.to_device(inp)
    plan = ssm.ssm_step_prepare(d["Lambda"], d["B"], d["C"], d["log_delta"])
    x = d["x0"]
    ys = []
    for t in range(steps):
        x, y = ssm.ssm_step(plan, d["D"], d["u"][:, t].contiguous(), x, d["is_first"][:, t].contiguous())
        ys.append(y)
    torch.cuda.synchronize()
    y_all = torch.stack(ys, 1).cpu().numpy()
    assert_close(y_all, ref["y"], TOL_FWD, "step y")
    assert_close(x.cpu().numpy(), ref["x_last"], TOL_FWD, "step x")
    # no previous state and no flags: x = Bbar u
    x1, y1 = ssm.ssm_step(plan, d["D"], d["u"][:, 0].contiguous(), None, None, P=P)
    ref1 = orc.forward(inp["Lambda"], inp["B"], inp["C"], inp["D"], inp["log_delta"], inp["u"][:, :1], None, None)
    assert_close(y1.cpu().numpy()[:, None], ref1["y"], TOL_FWD, "step y (no state)")


@pytest.mark.parametrize("Bt,H,P,steps", [(1024, 512, 512, 10), (37, 50, 33, 6)])
def test_step_mode_adjoint_rollout_equals_oracle_gradient(Bt, H, P, steps):
    """First-order gradients through an imagined trajectory: `steps` dependent calls of
    ssm_step_bwd in reverse order, each fed the state gradient of the step after it, against the
    oracle's gradient pass over the same inputs as one sequence (du of every step, and the
    gradient that reaches the initial state)."""
    import torch
    w = wl.custom("stepb", Bt, steps, H, P, backward=True, p_reset=0.1, with_x0=True, seed=29)
    inp = wl.gen_inputs(w)
    par = (inp["Lambda"], inp["B"], inp["C"], inp["D"], inp["log_delta"])
    ref_f = orc.forward(*par, inp["u"], inp["is_first"], inp["x0"], nthreads=8)
    ref_b = orc.backward(*par, inp["u"], inp["is_first"], inp["x0"], ref_f["x"], inp["dy"], nthreads=8)
    d = ssm.to_device(inp)
    plan = ssm.ssm_step_prepare(d["Lambda"], d["B"], d["C"], d["log_delta"])
    dx, dus = None, []
    for t in reversed(range(steps)):
        _, du, dx = ssm.ssm_step_bwd(plan, d["D"], d["dy"][:, t].contiguous(), dx, d["is_first"][:, t].contiguous(), P=P)
        dus.append(du)
    torch.cuda.synchronize()
    du_all = torch.stack(dus[::-1], 1).cpu().numpy()
    assert_close(du_all, ref_b["du"], TOL_GRAD, "step du")
    assert_close(dx.cpu().numpy(), ref_b["dx0"], TOL_GRAD, "step dx0")
    # no incoming gradient, no flags, no dx_prev wanted: du = Re(Bbar^H C^H dy) + D dy
    gx, du1, none = ssm.ssm_step_bwd(plan, d["D"], d["dy"][:, steps - 1].contiguous(), None, None, P=P,
                                     want_dx_prev=False)
    ref1 = orc.backward(*par, inp["u"][:, :1], None, None,
                        orc.forward(*par, inp["u"][:, :1], None, None)["x"], inp["dy"][:, steps - 1:steps])
    torch.cuda.synchronize()
    assert none is None
    assert_close(du1.cpu().numpy()[:, None], ref1["du"], TOL_GRAD, "step du (single)")


@pytest.mark.parametrize("Bt,L,H,P", [(4, 256, 128, 96), (2, 1500, 64, 80), (4, 512, 32, 840), (128, 16, 32, 1024),
                                      (24, 100, 512, 512)])
def test_captured_graph_replays_equal_eager(Bt, L, H, P):
    """The non-profiled entry points only enqueue kernels (no allocation, no memset, no wait), so
    one forward + gradient pass can be captured into a HIP graph.  Every replay, with eager work
    and synchronisations of the program in between, must reproduce the eager results bit for bit
    (second shape: several workgroups along time, i.e. the clear kernel and the look-back; third and
    fourth: the projections scan their own tiles, as a chain of tiles and with whole sequences per tile; fifth:
    separate scan kernels that record the row maxima of their output with atomics, two fp16 planes)."""
    import torch
    w = wl.custom("graph", Bt, L, H, P, backward=True, p_reset=0.01, with_x0=True, seed=61)
    d = ssm.to_device(wl.gen_inputs(w))
    par = (d["Lambda"], d["B"], d["C"], d["D"], d["log_delta"])
    ws_f = ssm.alloc_workspace(Bt, L, H, P, False)
    ws_b = ssm.alloc_workspace(Bt, L, H, P, True)
    out_f = {"y": torch.empty_like(d["u"]), "x": torch.empty((Bt, L, P), dtype=torch.complex64, device="cuda"),
             "x_last": torch.empty((Bt, P), dtype=torch.complex64, device="cuda")}
    out_b = {"du": torch.empty_like(d["u"]), "dLambda": torch.empty_like(d["Lambda"]), "dB": torch.empty_like(d["B"]),
             "dC": torch.empty_like(d["C"]), "dD": torch.empty_like(d["D"]),
             "dlog_delta": torch.empty_like(d["log_delta"]),
             "dx0": torch.empty((Bt, P), dtype=torch.complex64, device="cuda")}

    def step():
        ssm.ssm_scan_fwd(*par, d["u"], d["is_first"], d["x0"], workspace=ws_f, out=out_f)
        ssm.ssm_scan_bwd(*par, d["u"], d["is_first"], d["x0"], out_f["x"], d["dy"], workspace=ws_b, out=out_b)

    step()
    torch.cuda.synchronize()
    ref = {k: v.clone() for k, v in list(out_f.items()) + list(out_b.items())}
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for rep in range(3):
        for v in list(out_f.values()) + list(out_b.values()):
            v.zero_()                                   # eager work between the replays
        junk = torch.randn(1 << 20, device="cuda").sum().item()
        assert np.isfinite(junk)
        graph.replay()
        torch.cuda.synchronize()
        for k, v in list(out_f.items()) + list(out_b.items()):
            assert torch.equal(v, ref[k]), "replay %d differs from the eager result in %s" % (rep, k)
        assert ssm.ssm_workspace_status(ws_f) == ssm.SSM_OK and ssm.ssm_workspace_status(ws_b) == ssm.SSM_OK


def test_host_only_call_before_torch_does_not_break_later_launches():
    """A fresh interpreter that asks for a plan (host logic only) before it ever imports torch, then runs a
    forward pass: the launches work on torch's memory (one copy of the HIP runtime in the process)."""
    import os, subprocess, sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    code = ("import sys; sys.path.insert(0, %r)\n"
            "from paper_2502_20168_amd import binding as ssm, workloads as wl\n"
            "ssm.ssm_plan_describe(32, 32, 512, 510)\n"
            "import torch\n"
            "d = ssm.to_device(wl.gen_inputs(wl.custom('order', 4, 32, 24, 40, p_reset=0.05, seed=3)))\n"
            "out = ssm.ssm_scan_fwd(d['Lambda'], d['B'], d['C'], d['D'], d['log_delta'], d['u'], d['is_first'], d['x0'])\n"
            "torch.cuda.synchronize()\n"
            "assert bool(torch.isfinite(out['y']).all())\n"
            "print('ok')\n" % root)
    out = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=300)
    assert out.returncode == 0, out.stderr[-2000:]
    assert out.stdout.strip().splitlines()[-1] == "ok"


@pytest.mark.parametrize("Bt,L,H,P", [(16, 256, 512, 512), (24, 100, 512, 512), (6, 200, 100, 96)])
def test_operands_at_addresses_that_are_only_element_aligned_on_a_side_stream(Bt, L, H, P):
    """Every input (and the saved states handed to the gradient pass) one to three elements behind an aligned
    allocation -- 4-byte aligned floats, 8-byte aligned complex values, nothing more, which is what the header
    asks for -- and the calls on a stream of their own: the 16-byte loaders step aside, the results hold."""
    import torch
    rng = np.random.Generator(np.random.PCG64(Bt + L))

    def shifted(t, off):
        if t is None:
            return None
        flat = torch.empty(t.numel() + 8, dtype=t.dtype, device=t.device)
        v = flat[off:off + t.numel()].view(t.shape)
        v.copy_(t)
        return v

    w = wl.custom("offsets", Bt, L, H, P, p_reset=0.02, force_first=True, with_x0=True, seed=61)
    inp = wl.gen_inputs(w)
    ref = orc.run_workload(inp, True, nthreads=8)
    d = ssm.to_device(inp)
    e = {k: shifted(v, int(rng.integers(1, 4))) for k, v in d.items()}
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        fwd = ssm.ssm_scan_fwd(e["Lambda"], e["B"], e["C"], e["D"], e["log_delta"], e["u"], e["is_first"], e["x0"], stream=side)
        xs = shifted(fwd["x"], 1)
        bwd = ssm.ssm_scan_bwd(e["Lambda"], e["B"], e["C"], e["D"], e["log_delta"], e["u"], e["is_first"], e["x0"], xs,
                               e["dy"], stream=side)
    torch.cuda.synchronize()
    for k in ("y", "x", "x_last"):
        assert_close(fwd[k].cpu().numpy(), ref[k], TOL_FWD, "offsets " + k)
    for k in GRAD_KEYS:
        assert_close(bwd[k].cpu().numpy(), ref[k], TOL_GRAD, "offsets " + k)


def test_two_million_tokens_are_512_copies_of_the_benchmark_batch():
    """Index arithmetic past 2^31 elements (x has 2^31 floats here, 8 GiB): the benchmark batch repeated 512 times
    along the batch.  Sequences are independent and every token row carries its own scale, so every copy's y, x,
    x_last, du and dx0 must equal the first copy's bit for bit, and the first copy's must equal the results on
    the batch alone; the parameter gradients are 512 times the batch's within the accumulation error."""
    import torch
    Bt0, L, H, P, copies = 16, 256, 512, 512, 512
    w = wl.custom("big", Bt0, L, H, P, p_reset=0.01, force_first=True, with_x0=True, seed=3)
    d = ssm.to_device(wl.gen_inputs(w))
    par = (d["Lambda"], d["B"], d["C"], d["D"], d["log_delta"])
    small_f = ssm.ssm_scan_fwd(*par, d["u"], d["is_first"], d["x0"])
    small_b = ssm.ssm_scan_bwd(*par, d["u"], d["is_first"], d["x0"], small_f["x"], d["dy"])
    rep = lambda t: t.repeat((copies,) + (1,) * (t.dim() - 1)).contiguous()
    u, flags, x0, dy = rep(d["u"]), rep(d["is_first"]), rep(d["x0"]), rep(d["dy"])
    f = ssm.ssm_scan_fwd(*par, u, flags, x0)
    b = ssm.ssm_scan_bwd(*par, u, flags, x0, f["x"], dy)
    torch.cuda.synchronize()
    for big, small, name in [(f[k], small_f[k], k) for k in ("y", "x", "x_last")] + [(b[k], small_b[k], k) for k in ("du", "dx0")]:
        v = big.view((copies,) + tuple(small.shape))
        assert torch.equal(v[0], small), name + ": the first copy differs from the batch alone"
        assert bool((v == v[0:1]).all()), name + ": a copy differs from the first"
    for k in ("dLambda", "dB", "dC", "dD", "dlog_delta"):
        ref = small_b[k].to(torch.complex128 if small_b[k].is_complex() else torch.float64) * copies
        err = float((b[k].to(ref.dtype) - ref).abs().max()) / float(ref.abs().max())
        assert err < 1e-3, "%s: %.2e" % (k, err)


def test_concurrent_calls_from_four_host_threads_on_their_own_streams_and_workspaces():
    """The header's promise: concurrent calls are safe as long as they use distinct workspaces.  Four host
    threads (the binding's calls release the interpreter lock), each with a stream and two workspaces of its
    own, repeat the forward and the gradient pass of their shape; every result equals the single-threaded one
    bit for bit."""
    import threading
    import torch
    shapes = [(16, 256, 512, 512), (24, 100, 512, 512), (8, 100, 256, 256), (4, 4096, 256, 256)]
    data = []
    for i, shp in enumerate(shapes):
        d = ssm.to_device(wl.gen_inputs(wl.custom("thr%d" % i, *shp, p_reset=0.01, force_first=True, with_x0=True, seed=10 + i)))
        par = (d["Lambda"], d["B"], d["C"], d["D"], d["log_delta"])
        f = ssm.ssm_scan_fwd(*par, d["u"], d["is_first"], d["x0"])
        b = ssm.ssm_scan_bwd(*par, d["u"], d["is_first"], d["x0"], f["x"], d["dy"])
        torch.cuda.synchronize()
        data.append((shp, d, par, f, b))
    errors = []

    def worker(tid):
        try:
            st = torch.cuda.Stream()
            shp, d, par, f0, b0 = data[tid]
            ws_f, ws_b = ssm.alloc_workspace(*shp, False), ssm.alloc_workspace(*shp, True)
            for it in range(10):
                with torch.cuda.stream(st):
                    f = ssm.ssm_scan_fwd(*par, d["u"], d["is_first"], d["x0"], workspace=ws_f, stream=st)
                    b = ssm.ssm_scan_bwd(*par, d["u"], d["is_first"], d["x0"], f["x"], d["dy"], workspace=ws_b, stream=st)
                st.synchronize()
                errors.extend((tid, it, k) for k in ("y", "x", "x_last") if not torch.equal(f[k], f0[k]))
                errors.extend((tid, it, k) for k in GRAD_KEYS if not torch.equal(b[k], b0[k]))
                if ssm.ssm_workspace_status(ws_f, st) != ssm.SSM_OK or ssm.ssm_workspace_status(ws_b, st) != ssm.SSM_OK:
                    errors.append((tid, it, "status"))
        except Exception as e:          # a thread's exception must fail the test, not vanish
            errors.append((tid, repr(e)))

    threads = [threading.Thread(target=worker, args=(t,)) for t in range(len(shapes))]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors[:10]
