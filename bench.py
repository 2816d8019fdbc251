#!/usr/bin/env python3
"""Benchmark of the resettable S5 scan layer on one MI355X.

One "step" is one pass of the whole hot path -- forward (discretise, input projection, resettable
scan, output projection) plus the gradient pass (C^H dy, reverse scan, du, parameter gradients)
-- over one synthetic world-model-shaped batch (Bt=16, L=256, H=P=512) that is already resident
in HBM.  Prints ONE JSON line:
  metric/value : whole-job throughput in Mtokens/s (token = one (sequence, step) pair)
  parity       : the outputs of the timed steps against the float64 oracle on the same batch, with the
                 tolerances of the parity tests; the run fails on a mismatch
  roofline     : the dominant kernel (the launch of the projection GEMM with the largest share of the
                 step: fp32 in/out, operands staged as two scaled fp16 planes, three fp16 MFMA products
                 per multiply-add) against the fp16 matrix peak, its duration measured with HIP events on
                 the launch stream inside the library's *_profiled entry points; the fp32-equivalent rate
                 is given next to it, and every launch of the kernel below
  scan_roofline: the two scan kernels against the HBM peak (algorithmic bytes / event time): at the
                 benchmark shape warm (buffers resident in the 256 MB last-level cache) and cold (rotating
                 over more than 1 GiB of distinct buffers), and cold at working sets well past that cache
                 (the long-sequence configuration, and the benchmark shape with eight times the batch);
                 at shapes where the projections scan their own output tiles these kernels are not in the
                 path and are timed through the scan-level entry points
  whole_step_traffic: HBM bytes of all launches of one step (rocprofv3 counters, from profiles/)
  cpu_baseline : the float64 CPU oracle timed on the host cores on a bounded sample
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0          # MI355X HBM3E
PEAK_FP32_MFMA_TFLOPS = 157.3  # MI355X dense fp32 matrix
PEAK_F16_MFMA_TFLOPS = 2500.0  # MI355X dense fp16 / bf16 matrix
# HBM bytes per launch at config 2 from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by what the same
# counters read for a copy-like kernel of known size (profiles/gemm_scan_cfg2_fwd_bwd.md, which names the
# commit it was taken at).  Counters cannot be read from inside this process: these are constants of that
# profile, not measurements of this run.
PROFILE_TRAFFIC = {
    "source": "profiles/gemm_scan_cfg2_fwd_bwd.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE at commit 4199d0f, counters scaled by "
              "a 64 MiB element-wise kernel of the same run); constants of that profile, not measured by this run",
    "read_bytes": 267.4 * 2 ** 20, "write_bytes": 99.4 * 2 ** 20, "total_bytes": 366.8 * 2 ** 20,
    "algorithmic_bytes": 88.1e6, "total_over_algorithmic": 4.4,
    "dominant_launch_bytes": (91.9 + 40.4) * 2 ** 20,
    "dominant_launch_algorithmic_bytes": (74 + 40) * 2 ** 20,
    "dominant_launch_mfma_busy": 0.448,
}


def gate_products(T, H):
    """Partial products per multiply-add of the gate's products: two scaled fp16 planes per operand (three) at
    widths that are multiples of 64 from 512 on with enough tokens, else three bf16 planes (six)."""
    return 3 if (H % 64 == 0 and H >= 512 and ((T + 63) // 64) * ((H + 127) // 128) >= 200) else 6


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=2, help="index into the benchmark configurations")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--profile-iters", type=int, default=30)
    ap.add_argument("--counter-calibration", action="store_true",
                    help="also run torch's element-wise add on 64 MiB (reads 64 MiB, writes 64 MiB) a few times, so that "
                         "a rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE run of this command holds a kernel of known traffic "
                         "to scale the counters by")
    ap.add_argument("--path-only", action="store_true",
                    help="skip the sections beside the hot path (scan kernels alone, block_ops, step_mode, s5_block): "
                         "used for the rocprofv3 runs so that every kernel in the trace belongs to one role")
    ap.add_argument("--scan-only", action="store_true",
                    help="run only the two scan kernels at working sets past the last-level cache (scan_large) and print "
                         "their figures: the command behind profiles/scan_kernels_large_working_set.md")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2502_20168_amd import binding as ssm
    from paper_2502_20168_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    ssm.lib()                                  # fail loudly if the HIP library is missing
    if args.scan_only:
        if args.counter_calibration:
            src = torch.randn(16 << 20, device="cuda")
            dst = torch.empty_like(src)
            for _ in range(5):
                torch.add(src, 1.0, out=dst)
            torch.cuda.synchronize()
            del src, dst
        print(json.dumps({"scan_large": scan_large(ssm, torch, wl)}))
        return
    w = wl.CONFIGS[args.config]
    Bt, L, H, P = w.Bt, w.L, w.H, w.P
    T = w.tokens
    inp = wl.gen_inputs(w)
    d = ssm.to_device(inp)
    par = (d["Lambda"], d["B"], d["C"], d["D"], d["log_delta"])

    ws_f = ssm.alloc_workspace(Bt, L, H, P, False)
    ws_b = ssm.alloc_workspace(Bt, L, H, P, True)
    out_f = {"y": torch.empty_like(d["u"]),
             "x": torch.empty((Bt, L, P), dtype=torch.complex64, device="cuda"),
             "x_last": torch.empty((Bt, P), dtype=torch.complex64, device="cuda")}
    out_b = {"du": torch.empty_like(d["u"]), "dLambda": torch.empty_like(d["Lambda"]),
             "dB": torch.empty_like(d["B"]), "dC": torch.empty_like(d["C"]), "dD": torch.empty_like(d["D"]),
             "dlog_delta": torch.empty_like(d["log_delta"]),
             "dx0": torch.empty((Bt, P), dtype=torch.complex64, device="cuda")}

    def step(profile=False):
        f = ssm.ssm_scan_fwd(*par, d["u"], d["is_first"], d["x0"], workspace=ws_f, out=out_f, profile=profile)
        b = ssm.ssm_scan_bwd(*par, d["u"], d["is_first"], d["x0"], out_f["x"], d["dy"], workspace=ws_b,
                             out=out_b, profile=profile)
        return f, b

    if args.counter_calibration:
        src = torch.randn(16 << 20, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            torch.add(src, 1.0, out=dst)              # an element-wise kernel (a same-type copy_ would be a memcpy)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    mtok = T / (ms_per_step * 1e-3) / 1e6
    # a cross-workgroup wait that gave up would have been flagged in the workspace (and its outputs are NaN)
    for ws, name in ((ws_f, "forward"), (ws_b, "gradient pass")):
        st = ssm.ssm_workspace_status(ws)
        if st != ssm.SSM_OK:
            raise ssm.SsmError(st, "timed loop, %s" % name)
    timed_out = {k: v.cpu().numpy() for k, v in list(out_f.items()) + list(out_b.items())}

    # ---- distribution of single steps: one event pair per step (adds a little per-step overhead)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for e0, e1 in evs:
        e0.record()
        step()
        e1.record()
    torch.cuda.synchronize()
    per_step = np.sort(np.array([e0.elapsed_time(e1) for e0, e1 in evs])) * 1e3
    step_dist = {"median_us": round(float(np.median(per_step)), 1),
                 "p10_us": round(float(per_step[int(0.1 * (len(per_step) - 1))]), 1),
                 "p90_us": round(float(per_step[int(0.9 * (len(per_step) - 1))]), 1),
                 "note": "HIP events around every single step (forward + gradient pass)"}

    # ---- the same step captured once into a HIP graph and replayed: what a caller gets who removes the
    # host's per-launch cost that way (the entry points only enqueue kernels, so they can be captured);
    # it matters at the small shapes, where the eight or nine launches of a step are shorter than their enqueue
    graph_ms = graph_time_ms(torch, lambda i: step(), 10)
    graph_replay = {"ms_per_step": round(graph_ms, 4), "Mtokens_per_s": round(T / (graph_ms * 1e-3) / 1e6, 3),
                    "note": "ten steps captured into one HIP graph, the median of five replays timed with events; not the headline value"}

    # ---- per-kernel durations from HIP events recorded on the launch stream (library side)
    fs = np.zeros(ssm.SSM_FWD_STAGES)
    bs = np.zeros(ssm.SSM_BWD_STAGES)
    for _ in range(args.profile_iters):
        f, b = step(profile=True)
        fs += np.array(f["stage_ms"])
        bs += np.array(b["stage_ms"])
    fs /= args.profile_iters
    bs /= args.profile_iters
    stages = {"fwd_" + n: round(float(v) * 1e3, 2) for n, v in zip(ssm.FWD_STAGE_NAMES, fs)}
    stages.update({"bwd_" + n: round(float(v) * 1e3, 2) for n, v in zip(ssm.BWD_STAGE_NAMES, bs)})

    gemm_flops = 2.0 * T * (2 * P) * H                    # fp32 flops of every one of the six projections
    # where the projections scan their own tiles every operand comes with its largest magnitude and is staged
    # as two scaled fp16 planes (three products per multiply-add); elsewhere as three bf16 planes (six)
    scans = (((L % 128 == 0 and L // 128 <= 32) or (L in (16, 32, 64) and T % 128 == 0))
             and (T // 128) * ((2 * P + 127) // 128) >= 64)
    products = 3 if scans else 6
    t128 = ((T + 127) // 128) * ((H + 127) // 128)
    out_split = t128 < 200 and 2 * t128 >= 200 and P >= 256 and (2 * P) % 64 == 0
    # every launch of the projection kernel in one step: role, fp32 flops, duration
    if scans:
        launches = [
            {"role": "input projection + forward scan in the tile (S2 + S3)", "gemms": 1, "ms": fs[1]},
            {"role": "output projection" + (" + D u on 64x128 tiles" if out_split else " + D u")
                     + " (S4)", "gemms": 1, "ms": fs[3]},
            {"role": "C^H dy + reverse scan in the tile (S5 + S6)", "gemms": 1, "ms": bs[1]},
            {"role": "Re(Bbar^H chi) + D dy, the dBbar slabs and the dC slabs, one launch, two workgroups per CU (S7 + S5)",
             "gemms": 3, "ms": bs[3]},
        ]
    else:
        launches = [
            {"role": "input projection (S2)", "gemms": 1, "ms": fs[1]},
            {"role": "output projection + D u (S4)", "gemms": 1, "ms": fs[3]},
            {"role": "C^H dy and the dC slabs, one launch (S5)", "gemms": 2, "ms": bs[1]},
            {"role": "Re(Bbar^H chi) + D dy and the dBbar slabs, one launch (S7)", "gemms": 2, "ms": bs[3]},
        ]
    for l in launches:
        l["fp32_flops"] = l["gemms"] * gemm_flops
        l["fp32_equivalent_tflops"] = round(l["fp32_flops"] / (l["ms"] * 1e-3) / 1e12, 2)
        l["executed_tflops"] = round(products * l["fp32_flops"] / (l["ms"] * 1e-3) / 1e12, 1)
        l["frac_of_f16_matrix_peak"] = round(l["executed_tflops"] / PEAK_F16_MFMA_TFLOPS, 4)
        l["us"] = round(float(l.pop("ms")) * 1e3, 2)
    # Dominant kernel = the launch of gemm_ws_kernel with the largest share of the step.  Its algorithmic
    # work: the partial products per multiply-add that its operand split needs.
    dom = max(launches, key=lambda l: l["us"])
    dom_fp32_tflops = dom["fp32_flops"] / (dom["us"] * 1e-6) / 1e12
    ach = products * dom_fp32_tflops
    roofline = {"kernel": "gemm_ws_kernel (%s)" % dom["role"],
                "bound": "mfma", "achieved": round(ach, 1), "peak": PEAK_F16_MFMA_TFLOPS, "unit": "TFLOP/s",
                "frac": round(ach / PEAK_F16_MFMA_TFLOPS, 4),
                "traffic": None,
                "note": "achieved counts the %d %s MFMA products per fp32 multiply-add that the kernel executes by "
                        "design (peak: the dense fp16 / bf16 matrix rate, the same for both); fp32-equivalent rate "
                        "and its ratio to the fp32 matrix peak below" % (products, "fp16" if scans else "bf16"),
                "fp32_equivalent_tflops": round(dom_fp32_tflops, 2),
                "fp32_equivalent_over_fp32_matrix_peak": round(dom_fp32_tflops / PEAK_FP32_MFMA_TFLOPS, 4),
                "flops_per_launch_fp32": dom["fp32_flops"], "avg_launch_us": dom["us"], "all_launches": launches}
    whole = None
    if PROFILE_TRAFFIC and args.config == 2:
        whole = dict(PROFILE_TRAFFIC)
        roofline["traffic"] = PROFILE_TRAFFIC.get("dominant_launch_bytes")

    # ---- scans against the HBM roofline: algorithmic bytes = 16 B (forward: read v, write x) and
    # 24 B (reverse: read gx, read x, write chi) per (token, state).  Where the projections scan their
    # own tiles there is no scan kernel in the path; the scan-level entry points are timed on their own.
    fwd_bytes, rev_bytes = 16.0 * T * P, 24.0 * T * P
    scan = {"bound": "hbm", "peak": PEAK_HBM_GBS, "unit": "GB/s",
            "fwd_bytes_per_launch": fwd_bytes, "rev_bytes_per_launch": rev_bytes,
            "in_path": {"fwd": "inside the input projection" if scans else "scan_kernel<false>",
                        "rev": "inside the C^H dy launch" if scans else "scan_kernel<true>"},
            "in_path_fwd_us": None if scans else round(float(fs[2]) * 1e3, 2),
            "in_path_rev_us": None if scans else round(float(bs[2]) * 1e3, 2),
            "in_path_fwd_GBs": None if scans else round(fwd_bytes / (fs[2] * 1e-3) / 1e9, 1),
            "in_path_rev_GBs": None if scans else round(rev_bytes / (bs[2] * 1e-3) / 1e9, 1)}
    if not args.path_only:
        scan.update(scan_cold_warm(ssm, torch, d, Bt, L, P, fwd_bytes, rev_bytes))
        scan["frac"] = round(scan["cold_fwd_GBs"] / PEAK_HBM_GBS, 4)
        scan["frac_of_copy_kernel_cold"] = round(scan["cold_fwd_GBs"] / scan["copy_cold_GBs"], 4)
        scan["large_working_sets"] = scan_large(ssm, torch, wl)

    result = {
        "metric": "SSM scan fwd+bwd Mtokens/s (B=16, L=256, H=P=512); achieved HBM GB/s in scan_roofline and composite_hbm", "value": round(mtok, 3), "unit": "Mtokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32",
        "arith": "fp32 I/O and accumulation; projections on " +
                 ("fp16 MFMA on two scaled fp16 planes per operand (three products, fp32-class accuracy; an element more "
                  "than 2^17 below the largest magnitude under its scale is fixed-point)" if scans else
                  "bf16 MFMA with an exact 3-way bf16 split of both operands (fp32-class accuracy)"),
        "data": "synthetic",
        "config": {"workload": "%s: Bt=%d L=%d H=%d P=%d fwd+bwd, fp32 I/O, complex64 state, seed %d"
                               % (w.name, Bt, L, H, P, w.seed), "tokens_per_step": T},
        "roofline": roofline, "scan_roofline": scan, "stage_us": stages, "step_time": step_dist,
        "composite_hbm": {"algorithmic_bytes_per_step": compulsory_bytes(Bt, L, H, P),
                          "GBs": round(compulsory_bytes(Bt, L, H, P) / (ms_per_step * 1e-3) / 1e9, 1),
                          "frac_of_hbm_peak": round(compulsory_bytes(Bt, L, H, P) / (ms_per_step * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                          "note": "whole forward + gradient pass against the HBM peak, for reference only: the path "
                                  "is matrix-core bound (about 290 flop per compulsory byte at this shape)"},
        "whole_step_traffic": whole, "graph_replay": graph_replay,
    }
    if not args.path_only:
        result["block_ops"] = block_ops(ssm, torch, wl, T, H)
        result["step_mode"] = step_mode(ssm, torch, d, H, P)
        result["s5_block"] = s5_block(ssm, torch, wl, d, Bt, L, H, P)
    # the oracle on the same batch: checks what the timed steps produced, and is the CPU baseline
    oracle = oracle_check_and_time(w, inp, timed_out, want_timing=not args.no_cpu_baseline)
    result["parity"] = oracle["parity"]
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = oracle["cpu_baseline"]
    print(json.dumps(result))
    if not oracle["parity"]["ok"]:
        print("bench.py: the timed outputs do not match the oracle: %s" % oracle["parity"]["failed"], file=sys.stderr)
        sys.exit(1)


def oracle_check_and_time(w, inp, got, want_timing, budget_s=12.0):
    """Runs the float64 oracle (plain C, OpenMP over sequences) on the whole batch of the timed steps:
    every output of the last timed step is compared with it (normwise and max-abs, 1e-4 forward / 1e-3
    gradients, as in the parity tests), and the same calls, repeated for about `budget_s` seconds, are
    the CPU baseline."""
    import numpy as np
    from oracle import ssm_oracle as orc
    cores = max(1, min(len(os.sched_getaffinity(0)), orc.max_threads()))
    threads = min(cores, w.Bt)
    t0 = time.perf_counter()
    ref = orc.run_workload(inp, True, nthreads=threads)
    first = time.perf_counter() - t0
    worst, failed = {}, []
    for k, tol in (("y", 1e-4), ("x", 1e-4), ("x_last", 1e-4), ("du", 1e-3), ("dLambda", 1e-3), ("dB", 1e-3),
                   ("dC", 1e-3), ("dD", 1e-3), ("dlog_delta", 1e-3), ("dx0", 1e-3)):
        g, r = got[k], ref[k]
        diff = g.astype(r.dtype) - r
        nr, mr = float(np.linalg.norm(r.ravel())), float(np.max(np.abs(r)))
        # (an all-zero reference, e.g. dx0 when every sequence starts with a reset, must be met exactly)
        ne = float(np.linalg.norm(diff.ravel())) / (nr if nr > 0 else 1.0)
        me = float(np.max(np.abs(diff))) / (mr if mr > 0 else 1.0)
        worst[k] = round(max(ne, me) / tol, 4)
        if not (np.all(np.isfinite(g)) and ne <= tol and me <= tol):
            failed.append(k)
    res = {"parity": {"ok": not failed, "failed": failed, "worst_error_over_tolerance": worst,
                      "what": "outputs of the last timed step against the float64 oracle on the same batch, per tensor "
                              "normwise and max-abs (1e-4 forward, 1e-3 gradients)"}}
    if want_timing:
        reps, spent = 1, first
        while spent < budget_s and reps < 64:
            t0 = time.perf_counter()
            orc.run_workload(inp, True, nthreads=threads)
            spent += time.perf_counter() - t0
            reps += 1
        # single-threaded leg on a smaller sample
        n1 = min(w.Bt, 2)
        sub1 = {k: (v[:n1] if (v is not None and k in ("u", "is_first", "dy", "x0")) else v) for k, v in inp.items()}
        t0 = time.perf_counter()
        orc.run_workload(sub1, True, nthreads=1)
        dt1 = time.perf_counter() - t0
        res["cpu_baseline"] = {"value": round(reps * w.Bt * w.L / spent / 1e6, 5), "unit": "Mtokens/s", "cores": threads,
                               "kind": "oracle", "seconds": round(spent, 2),
                               "single_thread_value": round(n1 * w.L / dt1 / 1e6, 5), "single_thread_seconds": round(dt1, 2),
                               "single_thread_sample": "first %d sequences" % n1,
                               "sample": "float64 oracle forward + gradient pass on all %d sequences of the same batch, "
                                         "%d times over" % (w.Bt, reps)}
    return res


def compulsory_bytes(Bt, L, H, P):
    """Bytes the method itself must move per forward + gradient pass with everything fused that can be:
    forward u, y, x (saved) and the flags; gradient pass dy, u, x, du and the flags; parameters read twice
    and their gradients written once."""
    T = Bt * L
    fwd = T * (4 * H + 4 * H + 8 * P + 1)
    bwd = T * (4 * H + 4 * H + 8 * P + 4 * H + 1)
    par = 2 * (16 * P * H) + 16 * P * H
    return float(fwd + bwd + par)


def graph_time_ms(torch, fn, iters):
    """Average duration of one fn(i) call, i = 0 .. iters-1, on the GPU: the calls are captured into
    one HIP graph and the graph is replayed, so the launches follow each other without the host's
    per-call cost (argument marshalling takes about as long as one of the small kernels runs).
    Events bracket one replay; the median of five replays is reported (a single replay now and then
    takes several times as long as the others)."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        for i in range(3):
            fn(i)
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            for i in range(iters):
                fn(3 + i)
    torch.cuda.synchronize()
    graph.replay()
    torch.cuda.synchronize()
    times = []
    for _ in range(5):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        graph.replay()
        e1.record()
        torch.cuda.synchronize()
        times.append(e0.elapsed_time(e1))
    return sorted(times)[len(times) // 2] / iters


def step_mode(ssm, torch, d, H, P, Bt=1024, horizon=10):
    """Imagination-shaped use of the layer: `horizon` dependent one-step calls over Bt trajectories
    (each step consumes the state of the step before it), then the adjoint steps in reverse order."""
    plan = ssm.ssm_step_prepare(d["Lambda"], d["B"], d["C"], d["log_delta"])
    u = torch.randn((horizon, Bt, H), device="cuda")
    dy = torch.randn((horizon, Bt, H), device="cuda")
    xs = [torch.zeros((Bt, P), dtype=torch.complex64, device="cuda") for _ in range(horizon + 1)]
    ys = torch.empty_like(u)

    def rollout(i):
        for t in range(horizon):
            ssm.ssm_step(plan, d["D"], u[t], xs[t], None, x=xs[t + 1], y=ys[t])

    def adjoint(i):
        dx = None
        for t in reversed(range(horizon)):
            _, _, dx = ssm.ssm_step_bwd(plan, d["D"], dy[t], dx, None, P=P)

    f_ms = graph_time_ms(torch, rollout, 5) / horizon
    b_ms = graph_time_ms(torch, adjoint, 5) / horizon
    flops = 2 * 2.0 * Bt * (2 * P) * H                      # two products per step, forward and adjoint alike
    exe = lambda ms: 6 * flops / (ms * 1e-3) / 1e12          # three bf16 planes: six products per multiply-add
    return {"shape": "Bt=%d H=%d P=%d horizon=%d" % (Bt, H, P, horizon), "fwd_us_per_step": round(f_ms * 1e3, 2),
            "bwd_us_per_step": round(b_ms * 1e3, 2),
            "roofline": {"bound": "mfma", "unit": "TFLOP/s", "peak": PEAK_F16_MFMA_TFLOPS,
                         "fwd_achieved": round(exe(f_ms), 1), "fwd_frac": round(exe(f_ms) / PEAK_F16_MFMA_TFLOPS, 4),
                         "bwd_achieved": round(exe(b_ms), 1), "bwd_frac": round(exe(b_ms) / PEAK_F16_MFMA_TFLOPS, 4),
                         "fp32_equivalent_tflops_fwd": round(flops / (f_ms * 1e-3) / 1e12, 1)},
            "note": "dependent steps (two GEMM launches each on 64x64x64 tiles, three bf16 planes), replayed as one HIP "
                    "graph; bound by the latency of two dependent launches, not by throughput"}


def s5_block(ssm, torch, wl, d, Bt, L, H, P, iters=10):
    """SSM layer + half-GLU gate through ssm_block_fwd / ssm_block_bwd at the benchmark shape."""
    W = torch.from_numpy(wl.gen_half_glu(4, H, seed=1)["W"]).cuda()
    par = (d["Lambda"], d["B"], d["C"], d["D"], d["log_delta"], W)
    ws_f = torch.empty(ssm.ssm_block_workspace_bytes(Bt, L, H, P, False), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(ssm.ssm_block_workspace_bytes(Bt, L, H, P, True), dtype=torch.uint8, device="cuda")
    f = ssm.ssm_block_fwd(*par, d["u"], d["is_first"], d["x0"], workspace=ws_f)
    f_ms = graph_time_ms(torch, lambda i: ssm.ssm_block_fwd(*par, d["u"], d["is_first"], d["x0"], workspace=ws_f), iters)
    b_ms = graph_time_ms(torch, lambda i: ssm.ssm_block_bwd(*par, d["u"], d["is_first"], d["x0"], f["x"], f["y"], f["gate"],
                                                            d["dy"], workspace=ws_b), iters)
    T = Bt * L
    # forward: the layer's two products and the gate's; gradient pass: the layer's four and the gate's two (two fp16
    # planes everywhere at this shape: three partial products per multiply-add; else three bf16 planes: six)
    gp = gate_products(T, H)
    exe_f = (2 * 3 * 2.0 * T * 2 * P * H + gp * 2.0 * T * H * H) / (f_ms * 1e-3) / 1e12
    exe_b = (4 * 3 * 2.0 * T * 2 * P * H + 2 * gp * 2.0 * T * H * H) / (b_ms * 1e-3) / 1e12
    return {"shape": "Bt=%d L=%d H=%d P=%d" % (Bt, L, H, P), "fwd_us": round(f_ms * 1e3, 1), "bwd_us": round(b_ms * 1e3, 1),
            "Mtokens_per_s": round(T / ((f_ms + b_ms) * 1e-3) / 1e6, 2),
            "roofline": {"bound": "mfma", "unit": "TFLOP/s", "peak": PEAK_F16_MFMA_TFLOPS,
                         "fwd_achieved": round(exe_f, 1), "fwd_frac": round(exe_f / PEAK_F16_MFMA_TFLOPS, 4),
                         "bwd_achieved": round(exe_b, 1), "bwd_frac": round(exe_b / PEAK_F16_MFMA_TFLOPS, 4)},
            "note": "layer + gate, forward and gradient pass, replayed as HIP graphs (includes the binding's output "
                    "allocations inside the graph); GELU of the layer output is formed where the output projection's result is stored (on 64x128 tiles at this shape)"}


def block_ops(ssm, torch, wl, T, H, iters=20):
    """The two operations around the layer at the benchmark shape: half-GLU gate on [T, H] tokens
    (one H x H product forward, two in the gradient pass) and the lambda-return of an imagined
    roll-out (horizon 16, 65536 trajectories)."""
    d = {k: torch.from_numpy(v).cuda() for k, v in wl.gen_half_glu(T, H, seed=0).items()}
    ws_f = torch.empty(ssm.ssm_half_glu_workspace_bytes(T, H, False), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(ssm.ssm_half_glu_workspace_bytes(T, H, True), dtype=torch.uint8, device="cuda")
    y, gate, du, dW = torch.empty_like(d["u"]), torch.empty_like(d["u"]), torch.empty_like(d["u"]), torch.empty_like(d["W"])
    f_ms = graph_time_ms(torch, lambda i: ssm.ssm_half_glu_fwd(d["u"], d["W"], workspace=ws_f, y=y, gate=gate), iters)
    b_ms = graph_time_ms(torch, lambda i: ssm.ssm_half_glu_bwd(d["u"], d["W"], gate, d["dy"], workspace=ws_b,
                                                                du=du, dW=dW), iters)
    flops = 2.0 * T * H * H
    gp = gate_products(T, H)
    hor, ntraj = 16, 65536
    r = {k: torch.from_numpy(v).cuda() for k, v in wl.gen_returns(hor, ntraj, seed=0).items()}
    ret = torch.empty_like(r["reward"])
    lf_ms = graph_time_ms(torch, lambda i: ssm.ssm_lambda_return(r["reward"], r["cont"], r["value"], 0.997, 0.95,
                                                                  ret=ret), iters)
    lb_ms = graph_time_ms(torch, lambda i: ssm.ssm_lambda_return_bwd(r["cont"], r["value"], ret, r["dret"], 0.997,
                                                                      0.95), iters)
    n = hor * ntraj
    return {"half_glu": {"shape": "T=%d H=%d" % (T, H), "fwd_us": round(f_ms * 1e3, 2), "bwd_us": round(b_ms * 1e3, 2),
                         "fwd_fp32_equivalent_tflops": round(flops / (f_ms * 1e-3) / 1e12, 1),
                         "bwd_fp32_equivalent_tflops": round(2 * flops / (b_ms * 1e-3) / 1e12, 1),
                         "roofline": {"bound": "mfma", "unit": "TFLOP/s", "peak": PEAK_F16_MFMA_TFLOPS,
                                      "fwd_achieved": round(gp * flops / (f_ms * 1e-3) / 1e12, 1),
                                      "fwd_frac": round(gp * flops / (f_ms * 1e-3) / 1e12 / PEAK_F16_MFMA_TFLOPS, 4),
                                      "bwd_achieved": round(gp * 2 * flops / (b_ms * 1e-3) / 1e12, 1),
                                      "bwd_frac": round(gp * 2 * flops / (b_ms * 1e-3) / 1e12 / PEAK_F16_MFMA_TFLOPS, 4),
                                      "note": "%d partial products per multiply-add (%s)" % (gp, "two scaled fp16 planes per operand" if gp == 3 else "three bf16 planes per operand")},
                         "note": "fwd = GELU pass + one product with the gate in its store; bwd = element-wise "
                                 "pass + two products + slab sum"},
            "lambda_return": {"shape": "T=%d N=%d (time-major)" % (hor, ntraj), "fwd_us": round(lf_ms * 1e3, 2),
                              "bwd_us": round(lb_ms * 1e3, 2),
                              "fwd_GBs": round(16.0 * n / (lf_ms * 1e-3) / 1e9, 1),
                              "bwd_GBs": round(28.0 * n / (lb_ms * 1e-3) / 1e9, 1),
                              "roofline": {"bound": "hbm", "unit": "GB/s", "peak": PEAK_HBM_GBS,
                                           "fwd_frac": round(16.0 * n / (lf_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                                           "bwd_frac": round(28.0 * n / (lb_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)},
                              "note": "algorithmic bytes: fwd 3 reads + 1 write, bwd 4 reads + 3 writes of 4 B per "
                                      "(step, trajectory); buffers stay in the last-level cache (warm)"}}


def scan_cold_warm(ssm, torch, d, Bt, L, P, fwd_bytes, rev_bytes, iters=40):
    """Times the two scan kernels alone through the scan-level entry points with HIP events on the
    launch stream: warm = one buffer set reused, cold = rotating over > 1 GiB of buffers so that
    neither L2 nor the 256 MB last-level cache holds the data of the next launch."""
    A_bar, _ = ssm.ssm_discretize(d["Lambda"], None, d["log_delta"])
    A_bar = A_bar * 0.5      # the same buffer is scanned in place many times: keep the values bounded
    set_bytes = Bt * L * P * 8
    nsets = max(2, int((1 << 30) // set_bytes) + 1)
    vs = [torch.randn((Bt, L, P), dtype=torch.complex64, device="cuda") * 0.05 for _ in range(nsets)]
    xs = [torch.randn((Bt, L, P), dtype=torch.complex64, device="cuda") * 0.05 for _ in range(min(nsets, 8))]
    ws_f = ssm.alloc_workspace(Bt, L, 1, P, False)
    ws_r = ssm.alloc_workspace(Bt, L, 1, P, True)

    def timed(fn, rotate):
        return graph_time_ms(torch, lambda i: fn(i % nsets if rotate else 0), iters)

    f = lambda i: ssm.ssm_scan_states(A_bar, vs[i], d["is_first"], d["x0"], want_x_last=False, workspace=ws_f)
    r = lambda i: ssm.ssm_scan_states_reverse(A_bar, vs[i], xs[i % len(xs)], d["is_first"], d["x0"],
                                              want_dx0=False, workspace=ws_r)
    out = {}
    # plain device copy of the same bytes as the forward scan (read 8 B + write 8 B per element): what the
    # memory system gives a dependency-free kernel at this size
    cp = lambda i: vs[(i + 1) % nsets].copy_(vs[i])
    for mode in ("warm", "cold"):
        ms = timed(cp, mode == "cold")
        out["copy_%s_us" % mode] = round(ms * 1e3, 2)
        out["copy_%s_GBs" % mode] = round(fwd_bytes / (ms * 1e-3) / 1e9, 1)
    for name, fn, nbytes in (("fwd", f, fwd_bytes), ("rev", r, rev_bytes)):
        for mode in ("warm", "cold"):
            ms = timed(fn, mode == "cold")
            out["%s_%s_us" % (mode, name)] = round(ms * 1e3, 2)
            out["%s_%s_GBs" % (mode, name)] = round(nbytes / (ms * 1e-3) / 1e9, 1)
    out["note"] = ("warm/cold figures: %d calls of the scan-level entry points captured into one HIP graph and "
                   "replayed, so launches follow each other without host gaps (the reverse one includes its small "
                   "partial-sum reduction kernel); in_path figures are single launches between events inside the "
                   "full pass and include the gap between dependent kernels" % iters)
    return out


def scan_large(ssm, torch, wl, iters=12):
    """The two scan kernels cold (rotating over more than 1 GiB of distinct buffers) at working sets well
    past the 256 MB last-level cache, where the launch and the first memory round trip no longer
    dominate: the long-sequence configuration (4 x 4096 steps x 256 states) and the benchmark shape with
    eight times the batch (128 x 256 steps x 512 states).  Algorithmic bytes over event time."""
    import numpy as np
    res = {}
    for name, Bt, L, P, p_reset in (("cfg3_shape_4x4096x256", 4, 4096, 256, 0.001), ("cfg2_shape_x8_batch_128x256x512", 128, 256, 512, 0.01)):
        rng = np.random.Generator(np.random.PCG64(11))
        lam = (rng.uniform(0.5, 0.97, P) * np.exp(1j * rng.uniform(0, np.pi, P))).astype(np.complex64)
        fl = (rng.random((Bt, L)) < p_reset).astype(np.uint8)
        A_bar, flags = torch.from_numpy(lam).cuda(), torch.from_numpy(fl).cuda()
        set_bytes = Bt * L * P * 8
        nsets = max(3, int((5 << 28) // set_bytes) + 1)           # 1.25 GiB of v / gx buffers
        vs = [torch.randn((Bt, L, P), dtype=torch.complex64, device="cuda") * 0.05 for _ in range(nsets)]
        nx = max(2, min(nsets, int((1 << 29) // set_bytes) + 1))  # 0.5 GiB of saved-state buffers
        xs = [torch.randn((Bt, L, P), dtype=torch.complex64, device="cuda") * 0.05 for _ in range(nx)]
        ws_f = ssm.alloc_workspace(Bt, L, 1, P, False)
        ws_r = ssm.alloc_workspace(Bt, L, 1, P, True)
        fwd_bytes, rev_bytes = 16.0 * Bt * L * P, 24.0 * Bt * L * P
        f = lambda i: ssm.ssm_scan_states(A_bar, vs[i % nsets], flags, None, want_x_last=False, workspace=ws_f)
        r = lambda i: ssm.ssm_scan_states_reverse(A_bar, vs[i % nsets], xs[i % nx], flags, None, want_dx0=False, workspace=ws_r)
        cp = lambda i: vs[(i + 1) % nsets].copy_(vs[i % nsets])
        n = max(iters, nsets)
        e = {"working_set_MB": round(2 * set_bytes / 1e6, 1), "buffers_rotated": nsets}
        for key, fn, nbytes in (("copy", cp, fwd_bytes), ("fwd", f, fwd_bytes), ("rev", r, rev_bytes)):
            ms = graph_time_ms(torch, fn, n)
            e[key + "_us"] = round(ms * 1e3, 2)
            e[key + "_GBs"] = round(nbytes / (ms * 1e-3) / 1e9, 1)
            e[key + "_frac_of_hbm_peak"] = round(nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)
        assert ssm.ssm_workspace_status(ws_f) == ssm.SSM_OK and ssm.ssm_workspace_status(ws_r) == ssm.SSM_OK
        res[name] = e
        del vs, xs
        torch.cuda.empty_cache()
    res["note"] = ("cold: every launch works on buffers that no earlier launch of the replayed graph has touched within "
                   "the last 1 GiB of traffic; copy = torch's copy kernel on the same bytes as the forward scan (read 8 B + "
                   "write 8 B per element); the reverse figure includes its small partial-sum reduction kernel")
    return res




if __name__ == "__main__":
    main()
