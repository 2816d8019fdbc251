#!/usr/bin/env python3
"""Benchmark of the resettable S5 scan layer on one MI355X.

One "step" is one pass of the whole hot path -- forward (discretise, input projection, resettable
scan, output projection) plus the gradient pass (C^H dy, reverse scan, du, parameter gradients)
-- over one synthetic world-model-shaped batch (Bt=16, L=256, H=P=512) that is already resident
in HBM.  Prints ONE JSON line:
  metric/value : whole-job throughput in Mtokens/s (token = one (sequence, step) pair)
  roofline     : the dominant kernel (the projection GEMM: fp32 in/out, three-way bf16 operand
                 split, six bf16 MFMAs per k block; the launch with the largest share of the
                 step) against the bf16 matrix peak, its duration measured with HIP events on
                 the launch stream inside the library's *_profiled entry points; the
                 fp32-equivalent rate is given next to it, and every launch of the kernel below
  scan_roofline: the two scan kernels against the HBM peak (algorithmic bytes / event time),
                 warm (buffers resident in the 256 MB last-level cache) and cold (rotating over
                 more than 1 GiB of distinct buffers); at shapes where the projections scan
                 their own output tiles these kernels are not in the path and are timed alone
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
PEAK_BF16_MFMA_TFLOPS = 2500.0 # MI355X dense bf16 matrix
BF16_PRODUCTS = 6              # bf16 MFMA products the GEMM issues per fp32 multiply-add
# HBM bytes per launch of the two largest launches at config 2 from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE,
# scaled by what the same counters read for a copy-like kernel of known size
# (profiles/gemm_bf16x3_scan_cfg2_fwd_bwd.md), next to the algorithmic bytes:
#   C^H dy with the reverse scan in its tiles + the dC slabs: 64.3 MiB read (dy 8 + C 2 per XCD + x 16 for the
#     scan; dy 8 + x 16 for the slabs), 32.9 MiB written (chi 16 + eight dC slabs 16)
#   Re(Bbar^H chi) as two K halves + the dBbar slabs: 60.9 MiB read (chi 16 + Bbar 2 per XCD; chi 16 + u 8),
#     24.3 MiB written (two du slabs 16 + four dBbar slabs 8)
TRAFFIC = {
    "33,0": {"read_bytes": 67.6e6, "write_bytes": 34.5e6, "algorithmic_read_bytes": 52.4e6,
             "algorithmic_write_bytes": 33.6e6, "source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, see profiles/"},
    "1,0": {"read_bytes": 64.2e6, "write_bytes": 25.5e6, "algorithmic_read_bytes": 44.0e6,
            "algorithmic_write_bytes": 25.2e6, "source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, see profiles/"},
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=2, help="index into the benchmark configurations")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--profile-iters", type=int, default=30)
    ap.add_argument("--path-only", action="store_true",
                    help="skip the sections beside the hot path (reduced-precision mode, block_ops, step_mode): "
                         "used for the rocprofv3 runs so that every kernel in the trace belongs to one role")
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
    assert ssm.ssm_workspace_status(ws_f) == ssm.SSM_OK and ssm.ssm_workspace_status(ws_b) == ssm.SSM_OK

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

    # ---- the same step with the three-way bf16 split in every product (SSM_GEMM_SPLIT=3), timed the same
    # way, for comparison with the default (two scaled fp16 planes where the projections scan their tiles)
    three_plane = None
    if not args.path_only and os.environ.get("SSM_GEMM_F32", "") != "1" and os.environ.get("SSM_GEMM_SPLIT", "") != "3":
        os.environ["SSM_GEMM_SPLIT"] = "3"
        try:
            for _ in range(args.warmup):
                step()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                step()
            torch.cuda.synchronize()
            ms3 = (time.perf_counter() - t0) / args.steps * 1e3
        finally:
            os.environ.pop("SSM_GEMM_SPLIT", None)
        three_plane = {"ms_per_step": round(ms3, 4), "Mtokens_per_s": round(T / (ms3 * 1e-3) / 1e6, 3),
                       "note": "SSM_GEMM_SPLIT=3: three bf16 planes per operand and six products in every projection "
                               "(the default uses them only where an operand's largest magnitude is not known)"}
        step()                                              # leave the default-mode results in the output buffers
        torch.cuda.synchronize()

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
    f32_path = os.environ.get("SSM_GEMM_F32", "") == "1"
    fused_env = os.environ.get("SSM_FUSED_SCAN", "")
    shape_scans = (((L % 128 == 0 and L // 128 <= 32) or (L in (16, 32, 64) and T % 128 == 0))
                   and (T // 128) * ((2 * P + 127) // 128) >= 64 and not f32_path)
    fwd_fused = shape_scans and fused_env != "0"
    rev_fused = shape_scans and fused_env not in ("0", "1")
    # two scaled fp16 planes where the pass's projection scans its own tiles (every operand then comes
    # with its largest magnitude), three bf16 planes otherwise
    split3 = os.environ.get("SSM_GEMM_SPLIT", "") == "3"
    npl_f = 2 if (fwd_fused and not split3) else 3
    npl_b = 2 if (rev_fused and not split3) else 3
    kern = lambda tile, lay0, lay1, npl: "gemm_bf16x3_ws_kernel<%s,2,2,8,2,%d,%d,%d>" % (tile, npl, lay0, lay1)
    big = (T // 128) * ((2 * P + 127) // 128) >= 200
    t128 = ((T + 127) // 128) * ((H + 127) // 128)
    out_split = (not f32_path and t128 < 200 and 2 * t128 >= 200 and P >= 256 and (2 * P) % 64 == 0
                 and os.environ.get("SSM_SPLIT_OUT", "") != "0")
    out_tile = "128,128,32" if ((T + 127) // 128) * ((H + 127) // 128) >= 200 else \
               ("64,128,32" if ((T + 63) // 64) * ((H + 127) // 128) >= 200 else "64,64,64")
    in_tile = "128,128,32" if (big or fwd_fused) else ("64,128,32" if ((T + 63) // 64) * ((2 * P + 127) // 128) >= 200 else "64,64,64")
    # every launch of the projection kernel in one step: role, instantiation, fp32 flops, duration
    launches = [
        {"role": "input projection" + (" + forward scan in the tile" if fwd_fused else ""),
         "kernel": kern(in_tile, 31 if fwd_fused else 3, -1, npl_f), "npl": npl_f, "gemms": 1, "ms": fs[1]},
        ({"role": "output projection as two K halves into two slabs (a streaming kernel adds them and D u)",
          "kernel": kern("128,128,32", 3, -1, npl_f), "npl": npl_f, "gemms": 1, "ms": fs[3]} if out_split else
         {"role": "output projection + D u", "kernel": kern(out_tile, 7, -1, npl_f), "npl": npl_f, "gemms": 1, "ms": fs[3]}),
        {"role": "C^H dy" + (" + reverse scan in the tile" if rev_fused else "") + " and the dC slabs, one launch",
         "kernel": kern("128,128,32", 33 if rev_fused else 1, 0, npl_b), "npl": npl_b, "gemms": 2, "ms": bs[1]},
        ({"role": "Re(Bbar^H chi) as two K halves and the dBbar slabs, one launch (a streaming kernel adds the halves and D dy)",
          "kernel": kern("128,128,32", 1, 0, npl_b), "npl": npl_b, "gemms": 2, "ms": bs[3]} if out_split else
         {"role": "Re(Bbar^H chi) + D dy and the dBbar slabs, one launch",
          "kernel": kern("128,128,32", 5, 0, npl_b), "npl": npl_b, "gemms": 2, "ms": bs[3]}),
    ]
    for l in launches:
        l["fp32_flops"] = l["gemms"] * gemm_flops
        l["fp32_equivalent_tflops"] = round(l["fp32_flops"] / (l["ms"] * 1e-3) / 1e12, 2)
        l["us"] = round(float(l.pop("ms")) * 1e3, 2)
    # Dominant kernel = the launch of gemm_bf16x3_ws_kernel with the largest share of the step.  Its
    # algorithmic work: the partial products per multiply-add that its operand split needs (three
    # fp16 ones with two scaled planes, six bf16 ones with three planes).
    dom = max(launches, key=lambda l: l["us"])
    dom_fp32_tflops = dom["fp32_flops"] / (dom["us"] * 1e-6) / 1e12
    if f32_path:
        roofline = {"kernel": "gemm_f32_kernel (%s)" % dom["role"],
                    "bound": "mfma", "achieved": round(dom_fp32_tflops, 2), "peak": PEAK_FP32_MFMA_TFLOPS,
                    "unit": "TFLOP/s", "frac": round(dom_fp32_tflops / PEAK_FP32_MFMA_TFLOPS, 4), "traffic": None}
    else:
        npl = dom["npl"]
        products = 3 if npl == 2 else BF16_PRODUCTS
        ach = products * dom_fp32_tflops
        lay = dom["kernel"].rstrip(">").split(",")[-2] + "," + dom["kernel"].rstrip(">").split(",")[-1]
        known = TRAFFIC.get(lay) if (npl == 2 and args.config == 2 and fused_env == "" and out_split and
                                     dom["kernel"].startswith("gemm_bf16x3_ws_kernel<128,128,32")) else None
        roofline = {"kernel": "%s (%s)" % (dom["kernel"], dom["role"]),
                    "bound": "mfma", "achieved": round(ach, 1), "peak": PEAK_BF16_MFMA_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(ach / PEAK_BF16_MFMA_TFLOPS, 4),
                    "traffic": (known["read_bytes"] + known["write_bytes"]) if known else None,
                    "traffic_detail": known,
                    "note": "achieved counts the %d %s MFMA products per fp32 multiply-add that the kernel executes by "
                            "design (peak: the dense fp16 / bf16 matrix rate, the same for both); fp32-equivalent rate "
                            "and its ratio to the fp32 matrix peak below" % (products, "fp16" if npl == 2 else "bf16"),
                    "fp32_equivalent_tflops": round(dom_fp32_tflops, 2),
                    "fp32_equivalent_over_fp32_matrix_peak": round(dom_fp32_tflops / PEAK_FP32_MFMA_TFLOPS, 4)}
    roofline.update({"flops_per_launch_fp32": dom["fp32_flops"], "avg_launch_us": dom["us"],
                     "all_launches": launches})
    if not f32_path:
        roofline["measured_matrix_only"] = mfma_only_rate(ssm, torch, dom["us"], dom["npl"] == 2)
        roofline["frac_of_measured_matrix_only"] = round(
            roofline["achieved"] / roofline["measured_matrix_only"]["launch_like_the_dominant_one"]["TFLOPs"], 4)

    # ---- scans against the HBM roofline: algorithmic bytes = 16 B (forward: read v, write x) and
    # 24 B (reverse: read gx, read x, write chi) per (token, state).  Where the projections scan their
    # own tiles there is no scan kernel in the path; the scan-level entry points are timed on their own.
    fwd_bytes, rev_bytes = 16.0 * T * P, 24.0 * T * P
    scan = {"bound": "hbm", "peak": PEAK_HBM_GBS, "unit": "GB/s",
            "fwd_bytes_per_launch": fwd_bytes, "rev_bytes_per_launch": rev_bytes,
            "in_path": {"fwd": "inside the input projection" if fwd_fused else "scan_kernel<false>",
                        "rev": "inside the C^H dy launch" if rev_fused else "scan_kernel<true>"},
            "in_path_fwd_us": None if fwd_fused else round(float(fs[2]) * 1e3, 2),
            "in_path_rev_us": None if rev_fused else round(float(bs[2]) * 1e3, 2),
            "in_path_fwd_GBs": None if fwd_fused else round(fwd_bytes / (fs[2] * 1e-3) / 1e9, 1),
            "in_path_rev_GBs": None if rev_fused else round(rev_bytes / (bs[2] * 1e-3) / 1e9, 1)}
    scan.update(scan_cold_warm(ssm, torch, d, Bt, L, P, fwd_bytes, rev_bytes))
    scan["frac"] = round(scan["cold_fwd_GBs"] / PEAK_HBM_GBS, 4)
    scan["frac_of_copy_kernel_cold"] = round(scan["cold_fwd_GBs"] / scan["copy_cold_GBs"], 4)
    if (fwd_fused or rev_fused) and not args.path_only:
        scan["separate_kernels"] = separate_scan_kernels(step, args.warmup, args.steps, T, torch, time)

    result = {
        "metric": "SSM scan fwd+bwd Mtokens/s (B=16, L=256, H=P=512); achieved HBM GB/s in scan_roofline and composite_hbm", "value": round(mtok, 3), "unit": "Mtokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32",
        "arith": "fp32 I/O and accumulation; projections on " + ("fp32 MFMA" if f32_path else
                 ("fp16 MFMA on two scaled fp16 planes per operand (three products, fp32-class accuracy)"
                  if (npl_f == 2 and npl_b == 2) else
                  "bf16 MFMA with an exact 3-way bf16 split of both operands (fp32-class accuracy)")),
        "data": "synthetic",
        "config": {"workload": "%s: Bt=%d L=%d H=%d P=%d fwd+bwd, fp32 I/O, complex64 state, seed %d"
                               % (w.name, Bt, L, H, P, w.seed), "tokens_per_step": T},
        "roofline": roofline, "scan_roofline": scan, "stage_us": stages, "step_time": step_dist,
        "composite_hbm": {"algorithmic_bytes_per_step": compulsory_bytes(Bt, L, H, P),
                          "GBs": round(compulsory_bytes(Bt, L, H, P) / (ms_per_step * 1e-3) / 1e9, 1),
                          "frac_of_hbm_peak": round(compulsory_bytes(Bt, L, H, P) / (ms_per_step * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                          "note": "whole forward + gradient pass against the HBM peak, for reference only: the path "
                                  "is matrix-core bound (about 290 flop per compulsory byte at this shape)"},
        "three_plane_mode": three_plane,
    }
    if not args.path_only:
        result["block_ops"] = block_ops(ssm, torch, wl, T, H)
        result["step_mode"] = step_mode(ssm, torch, d, H, P)
        result["s5_block"] = s5_block(ssm, torch, wl, d, Bt, L, H, P)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, inp)
    print(json.dumps(result))


def mfma_only_rate(ssm, torch, dom_us, fp16):
    """The projection kernel's matrix-instruction stream alone (ssm_mfma_probe: one wavefront per SIMD
    on all 256 CUs, register operands with changing bits): what the matrix cores sustain on this
    device, at the clock they hold under that load, for a launch as long as the dominant one and for
    a long one.  Context for roofline.frac, whose peak is the published 2.4 GHz figure."""
    flops_per_iter = 256 * 4 * 24 * 2.0 * 32 * 32 * 16
    out = torch.empty(256 * 256, dtype=torch.float32, device="cuda")
    res = {}
    # 24 matrix instructions of 8 passes take 768 cycles: about 0.4 us per iteration
    for label, iters in (("launch_like_the_dominant_one", max(8, int(dom_us / 0.42))), ("long_launch", 4000)):
        for _ in range(3):
            ssm.ssm_mfma_probe(256, iters, fp16=fp16, out=out)
        torch.cuda.synchronize()
        reps = 10
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            ssm.ssm_mfma_probe(256, iters, fp16=fp16, out=out)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / reps
        res[label] = {"iters": iters, "us": round(us, 2), "TFLOPs": round(flops_per_iter * iters / (us * 1e-6) / 1e12, 1)}
    res["note"] = ("%s 32x32x16 matrix instructions only, 256 workgroups x 4 wavefronts; includes the launch; "
                   "the published peak assumes 2.4 GHz" % ("fp16" if fp16 else "bf16"))
    return res


def separate_scan_kernels(step, warmup, steps, T, torch, time):
    """The same step with SSM_FUSED_SCAN=0 (projections and scans as separate kernels), for comparison."""
    old = os.environ.get("SSM_FUSED_SCAN")
    os.environ["SSM_FUSED_SCAN"] = "0"
    try:
        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / steps * 1e3
    finally:
        if old is None:
            os.environ.pop("SSM_FUSED_SCAN", None)
        else:
            os.environ["SSM_FUSED_SCAN"] = old
    step()                                                  # leave the default path's results in the buffers
    torch.cuda.synchronize()
    return {"ms_per_step": round(ms, 4), "Mtokens_per_s": round(T / (ms * 1e-3) / 1e6, 3),
            "note": "SSM_FUSED_SCAN=0: scan_kernel<false> / scan_kernel<true> between the projections"}


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
    Events bracket one replay."""
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
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    graph.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters


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
    return {"shape": "Bt=%d H=%d P=%d horizon=%d" % (Bt, H, P, horizon), "fwd_us_per_step": round(f_ms * 1e3, 2),
            "bwd_us_per_step": round(b_ms * 1e3, 2),
            "note": "dependent steps (two GEMM launches each), replayed as one HIP graph; latency bound"}


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
    return {"shape": "Bt=%d L=%d H=%d P=%d" % (Bt, L, H, P), "fwd_us": round(f_ms * 1e3, 1), "bwd_us": round(b_ms * 1e3, 1),
            "Mtokens_per_s": round(T / ((f_ms + b_ms) * 1e-3) / 1e6, 2),
            "note": "layer + gate, forward and gradient pass, replayed as HIP graphs (includes the binding's output "
                    "allocations inside the graph); GELU of the layer output is formed where the output projection's result is stored (in the sum of its two K halves at this shape)"}


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
                         "note": "fwd = GELU pass + one product with the gate in its store; bwd = element-wise "
                                 "pass + two products + slab sum"},
            "lambda_return": {"shape": "T=%d N=%d (time-major)" % (hor, ntraj), "fwd_us": round(lf_ms * 1e3, 2),
                              "bwd_us": round(lb_ms * 1e3, 2),
                              "fwd_GBs": round(16.0 * n / (lf_ms * 1e-3) / 1e9, 1),
                              "bwd_GBs": round(28.0 * n / (lb_ms * 1e-3) / 1e9, 1),
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


def cpu_baseline(w, inp):
    """The float64 oracle (plain C, OpenMP over sequences) on the first sequences of the same batch."""
    from oracle import ssm_oracle as orc
    cores = max(1, min(len(os.sched_getaffinity(0)), orc.max_threads()))
    nseq = min(w.Bt, max(cores, 4))
    sub = {k: (v[:nseq] if (v is not None and k in ("u", "is_first", "dy", "x0")) else v) for k, v in inp.items()}
    threads = min(cores, nseq)
    t0 = time.perf_counter()
    orc.run_workload(sub, True, nthreads=threads)
    dt = time.perf_counter() - t0
    # single-threaded leg on a smaller sample
    n1 = min(nseq, 2)
    sub1 = {k: (v[:n1] if (v is not None and k in ("u", "is_first", "dy", "x0")) else v) for k, v in inp.items()}
    t0 = time.perf_counter()
    orc.run_workload(sub1, True, nthreads=1)
    dt1 = time.perf_counter() - t0
    return {"value": round(nseq * w.L / dt / 1e6, 5), "unit": "Mtokens/s", "cores": threads, "kind": "oracle",
            "seconds": round(dt, 2),
            "single_thread_value": round(n1 * w.L / dt1 / 1e6, 5), "single_thread_seconds": round(dt1, 2),
            "single_thread_sample": "first %d sequences" % n1,
            "sample": "float64 oracle forward + gradient pass on the first %d of %d sequences of the same batch"
                      % (nseq, w.Bt)}


if __name__ == "__main__":
    main()
