"""Builds libssmscan.so (HIP, gfx950 only) in-tree with hipcc: one object per source, compiled in
parallel, then one link."""
from __future__ import annotations

import concurrent.futures
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJDIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libssmscan.so")
SOURCES = ["ssm_api.hip", "gemm.hip", "gemm_inst2.hip", "gemm_inst3.hip", "gemm_pair.hip", "scan.hip", "params.hip",
           "block.hip", "noalloc.hip"]
HEADERS = [os.path.join(CSRC, h) for h in ("ssm_internal.h", "gemm_common.h", "gemm_kernel.h", "lookback.h")] + \
          [os.path.join(os.path.dirname(HERE), "include", h) for h in ("ssm.h", "ssm_measure.h")]
# packed-fp32 instructions are switched off on purpose (target feature removed for device code)
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def _newest_header() -> float:
    return max(os.path.getmtime(h) for h in HEADERS)


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, s) for s in SOURCES] + HEADERS
    return any(os.path.getmtime(d) > t for d in deps)


def _compile(hipcc: str, src: str, obj: str, verbose: bool) -> None:
    cmd = [hipcc] + FLAGS + ["-c", src, "-o", obj]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile every HIP source and link them into one shared library.  Returns its path.
    force=False recompiles only the objects that are older than their source or any header."""
    if not force and not is_stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJDIR, exist_ok=True)
    hdr_t = _newest_header()
    jobs = []
    for s in SOURCES:
        src = os.path.join(CSRC, s)
        obj = os.path.join(OBJDIR, s + ".o")
        fresh = os.path.exists(obj) and os.path.getmtime(obj) >= max(os.path.getmtime(src), hdr_t)
        if force or not fresh:
            jobs.append((src, obj))
    workers = max(1, min(len(jobs), len(os.sched_getaffinity(0)), 8))
    if jobs:
        with concurrent.futures.ThreadPoolExecutor(max_workers=workers) as pool:
            for f in [pool.submit(_compile, hipcc, src, obj, verbose) for src, obj in jobs]:
                f.result()
    tmp = LIB + ".tmp%d" % os.getpid()
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + [os.path.join(OBJDIR, s + ".o") for s in SOURCES] + ["-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    import sys
    print(build(force="--incremental" not in sys.argv, verbose=True))
